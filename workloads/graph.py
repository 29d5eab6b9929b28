"""Python front end of the host graph generator (``vamana_host.cpp``) and on-disk caching.

Support code for producing inputs: the navigation graph is built once on the host and handed,
unchanged, to both the CPU oracle and the GPU library.
"""
from __future__ import annotations

import ctypes
import hashlib
import os
import subprocess
import time

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = os.path.join(_HERE, "libvamana_host.so")
_SRCS = [os.path.join(_HERE, f) for f in ("vamana_host.cpp", "vamana_core.inc")]

EMPTY = 0xFFFFFFFF


def build_lib(force: bool = False) -> str:
    newest = max(os.path.getmtime(s) for s in _SRCS)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        common = ["g++", "-O3", "-std=c++17", "-pthread", "-fPIC", "-Wall", "-Wextra", "-c", _SRCS[0]]
        o1 = os.path.join(_HERE, "vamana_host_generic.o")
        o2 = os.path.join(_HERE, "vamana_host_avx512.o")
        subprocess.run(common + ["-mpopcnt", "-o", o1], check=True)
        subprocess.run(common + ["-DVH_VARIANT_ONLY", "-mavx512f", "-mavx512vl", "-mavx512bw", "-mavx512dq",
                                 "-mavx512vpopcntdq", "-mpopcnt", "-o", o2], check=True)
        subprocess.run(["g++", "-shared", "-pthread", "-o", _LIB, o1, o2], check=True)
        os.remove(o1)
        os.remove(o2)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build_lib()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        lib.vh_encode.restype = ctypes.c_int
        lib.vh_encode.argtypes = [P, ctypes.c_int64, ctypes.c_int, P, ctypes.c_int]
        lib.vh_pick_entry.restype = ctypes.c_int64
        lib.vh_pick_entry.argtypes = [P, P, ctypes.c_int64, ctypes.c_int, ctypes.c_int]
        lib.vh_build.restype = ctypes.c_int
        lib.vh_build.argtypes = [P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                 ctypes.c_uint32, P, ctypes.c_int, ctypes.c_char_p, ctypes.c_double, ctypes.c_int64]
        lib.vh_uses_avx512.restype = ctypes.c_int
        _lib = lib
    return _lib


def host_threads() -> int:
    """Worker threads for host-side generation (a 1-GPU machine gives 16 cores whatever nproc says)."""
    return max(1, min(16, os.cpu_count() or 1))


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def build_graph_from_codes(codes: np.ndarray, d: int, R: int, L: int, alpha: float, entry: int,
                           threads: int | None = None, max_batch: int = 1 << 20) -> np.ndarray:
    """The generator's construction on given codes (uint64 [n, 2*ceil(d/64)]) and entry -> adj [n, R]."""
    lib = _load()
    codes = np.ascontiguousarray(codes, dtype=np.uint64)
    n = codes.shape[0]
    adj = np.empty((n, R), dtype=np.uint32)
    rc = lib.vh_build(_p(codes), n, d, R, L, float(alpha), int(entry), _p(adj), threads or host_threads(), None,
                      0.02, max_batch)
    assert rc == 0, rc
    return adj


def build_graph(x: np.ndarray, R: int, L: int, alpha: float, threads: int | None = None,
                progress_path: str | None = None, max_batch: int = 1 << 20):
    """float32 [n, d] -> (adj uint32 [n, R], entry).  Deterministic for given inputs and parameters."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    n, d = x.shape
    threads = threads or host_threads()
    codes = np.empty((n, 2 * ((d + 63) // 64)), dtype=np.uint64)
    assert lib.vh_encode(_p(x), n, d, _p(codes), threads) == 0
    entry = int(lib.vh_pick_entry(_p(x), _p(codes), n, d, threads))
    assert 0 <= entry < n
    adj = np.empty((n, R), dtype=np.uint32)
    pp = progress_path.encode() if progress_path else None
    rc = lib.vh_build(_p(codes), n, d, R, L, float(alpha), entry, _p(adj), threads, pp, 0.02, max_batch)
    assert rc == 0, rc
    return adj, entry


def cache_dir() -> str:
    d = os.environ.get("QUIVER_CACHE", os.path.join("/tmp", "quiver_cache"))
    os.makedirs(d, exist_ok=True)
    return d


def cached_graph(tag: str, x: np.ndarray, R: int, L: int, alpha: float, progress_path: str | None = None):
    """build_graph with a file cache keyed by the parameters and a digest of a sample of the data."""
    h = hashlib.sha256()
    h.update(repr(("v2", tag, x.shape, R, L, alpha)).encode())
    step = max(1, x.shape[0] // 64)
    h.update(np.ascontiguousarray(x[::step]).tobytes())
    path = os.path.join(cache_dir(), f"graph_{tag}_{h.hexdigest()[:16]}.npz")
    if os.path.exists(path):
        z = np.load(path)
        return z["adj"], int(z["entry"])
    t0 = time.time()
    adj, entry = build_graph(x, R, L, alpha, progress_path=progress_path)
    try:
        np.savez(path, adj=adj, entry=np.int64(entry), seconds=time.time() - t0)
    except OSError:
        pass
    return adj, entry
