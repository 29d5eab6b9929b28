"""Host-side contracts that need no GPU: the one-GPU rule of bench.py, the product failing loudly without
its library, and the separation between the product package and the oracle."""
import os
import re
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_package_without_its_library_fails_loudly(tmp_path):
    pkg = tmp_path / "paper_2605_02171_amd"
    pkg.mkdir()
    for f in ("__init__.py", "binding.py", "build.py"):
        shutil.copy(os.path.join(ROOT, "paper_2605_02171_amd", f), pkg / f)
    r = subprocess.run([sys.executable, "-c", "import paper_2605_02171_amd"], cwd=tmp_path, capture_output=True,
                       text=True, timeout=300)
    assert r.returncode != 0, "importing the binding without libquiver_hip.so must raise"
    assert "libquiver_hip.so" in r.stderr


def _sources(top, suffixes):
    for base, _, files in os.walk(os.path.join(ROOT, top)):
        if "__pycache__" in base:
            continue
        for f in files:
            if f.endswith(suffixes):
                yield os.path.join(base, f)


def test_product_and_oracle_do_not_know_each_other():
    for path in _sources("paper_2605_02171_amd", (".py", ".hip", ".h")):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), path
        assert "quiver_oracle" not in text and "orc_" not in text, path
    for path in list(_sources("oracle", (".py", ".c", ".h"))) + [os.path.join(ROOT, "include", "quiver.h")]:
        text = open(path).read()
        assert "paper_2605_02171_amd" not in text and "libquiver_hip" not in text, path
    for path in _sources("oracle", (".c", ".h")):
        assert "quiver.h" not in open(path).read(), path
    # the input generators hold none of the method's arithmetic and load neither side
    for path in _sources("workloads", (".py",)):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+(oracle|paper_2605_02171_amd)\b", text, re.M), path


def test_nothing_committed_reads_the_scratch_folder_or_the_reference():
    for top in ("paper_2605_02171_amd", "oracle", "workloads", "tests"):
        for path in _sources(top, (".py", ".hip", ".h", ".c", ".cpp", ".inc")):
            if path.endswith("test_host_logic.py"):
                continue
            text = open(path).read()
            assert "_work/" not in text and "/root/reference" not in text, path
    for f in ("bench.py", "__graft_entry__.py"):
        text = open(os.path.join(ROOT, f)).read()
        assert "_work/" not in text and "/root/reference" not in text, f


def test_the_library_allocates_no_device_memory():
    """Every buffer is the caller's (inputs, outputs, workspaces) or, for qv_search_static, an array inside the
    library's own device code: no source of the library calls an allocating HIP routine."""
    allocating = re.compile(r"\bhip(Ext)?(Malloc|Free|HostMalloc|HostAlloc|HostFree|MallocAsync|FreeAsync|MallocManaged|"
                            r"MallocFromPoolAsync|MallocWithFlags|MemPoolCreate|HostRegister)\w*\s*\(")
    for path in _sources(os.path.join("paper_2605_02171_amd", "csrc"), (".hip", ".h")):
        code = re.sub(r"//[^\n]*", "", open(path).read())
        assert not allocating.search(code), path
    api = open(os.path.join(ROOT, "paper_2605_02171_amd", "csrc", "api.hip")).read()
    assert "static __device__ __align__(256) unsigned char scratch[QV_STATIC_SCRATCH_BYTES]" in api
    assert "hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))" in api
