"""Compile the HIP library for gfx950 (in-tree: csrc/*.hip -> libquiver_hip.so)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libquiver_hip.so")
SOURCES = ["api.hip", "encode.hip", "rerank.hip", "scan.hip", "build.hip"]
# the search kernel is compiled once per (encoding, code width) pair (64-bit words per bit-plane; 0 = any width
# at run time), for each of the three encodings
SM_WIDTHS = [12, 16, 24, 48, 32, 8, 6, 4, 2, 0]
SEARCH_VARIANTS = [(0, w) for w in SM_WIDTHS] + [(e, w) for e in (1, 2) for w in SM_WIDTHS]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-parameter",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _newest_source() -> float:
    files = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    files.append(os.path.join(HERE, "..", "include", "quiver.h"))
    return max(os.path.getmtime(f) for f in files)


def is_current() -> bool:
    return os.path.exists(LIB) and os.path.getmtime(LIB) >= _newest_source()


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and is_current():
        return LIB
    jobs = [("search.hip", os.path.join(CSRC, f"search_e{e}_w{w}.o"), [f"-DQV_SEARCH_ENC={e}", f"-DQV_SEARCH_WIDTH={w}"])
            for e, w in SEARCH_VARIANTS]
    jobs += [(s, os.path.join(CSRC, s.replace(".hip", ".o")), []) for s in SOURCES]
    objs = [j[1] for j in jobs]

    def compile_one(args):
        src, obj, extra = args
        cmd = [HIPCC] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        # the host pass does not know the device-only target feature; that warning is expected
        noise = "is not a recognized feature for this target"
        rest = [l for l in r.stderr.splitlines() if l.strip() and noise not in l]
        if verbose and rest:
            print("\n".join(rest), file=sys.stderr)

    with ThreadPoolExecutor(min(8, os.cpu_count() or 1)) as ex:
        list(ex.map(compile_one, jobs))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, check=True)
    for o in objs:
        os.remove(o)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
