"""Structural rules of this repository that can be checked without a GPU."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(*dirs, exts=(".py", ".hip", ".h", ".c")):
    for d in dirs:
        for base, _, files in os.walk(os.path.join(ROOT, d)):
            for f in files:
                if f.endswith(exts):
                    yield os.path.join(base, f)


def test_product_never_touches_the_oracle():
    for path in list(_sources("paper_2411_05309_amd", "include")):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), path
        assert "gpuvm_oracle" not in text and "oracle_" not in text, path


def test_oracle_never_touches_the_product():
    for path in _sources("oracle"):
        text = open(path).read()
        assert "paper_2411_05309_amd" not in text and "libgpuvm.so" not in text, path
        assert "hip_runtime" not in text and "gpuvm.h" not in text and "gpuvm_device.h" not in text, path


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    import paper_2411_05309_amd as gv
    monkeypatch.setattr(gv, "_lib", None)
    monkeypatch.setattr(gv, "LIB_PATH", str(tmp_path / "libgpuvm.so"))
    try:
        gv.load()
    except ImportError as e:
        assert "no CPU fallback" in str(e)
    else:
        raise AssertionError("load() must raise when the library is not built")


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_gpu_only_files_are_marked():
    for path in _sources("tests", exts=(".py",)):
        name = os.path.basename(path)
        if name.startswith("test_gpu_"):
            assert "pytestmark = pytest.mark.gpu" in open(path).read(), name
