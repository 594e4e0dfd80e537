"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_16864_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f


def test_measurement_aid_library_exports_both_probes():
    # bench_mfma_probe.so is built next to bench.py by build(); bench.py loads it with ctypes
    import ctypes
    path = os.path.join(ROOT, "bench_mfma_probe.so")
    if not os.path.exists(path):
        import pytest
        pytest.skip("bench_mfma_probe.so not built")
    lib = ctypes.CDLL(path)
    for name in ("bench_mfma_probe", "bench_valu_under_mfma"):
        assert hasattr(lib, name), name
