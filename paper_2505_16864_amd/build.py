"""Builds libjenga.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libjenga.so")
SOURCES = ["jenga_plan.cpp", "jenga_host.cpp", "jenga_permute.hip", "jenga_select.hip", "jenga_attn.hip", "jenga_prores.hip", "jenga_capi.hip"]


def build_library(verbose=False):
    """Compile every source for gfx950 and link libjenga.so; raises on failure."""
    cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
           # packed-FP32 VALU forms stay off for all device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "not a recognized feature" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libjenga.so")
    return LIB


def build_bench_probe():
    """bench.py's MFMA-only yardstick: its own shared object beside bench.py, not part of the library."""
    src = os.path.join(ROOT, "bench_mfma_probe.hip")
    out = os.path.join(ROOT, "bench_mfma_probe.so")
    cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", src, "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        print(res.stderr)
        raise RuntimeError("hipcc failed building bench_mfma_probe.so")
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_bench_probe())
