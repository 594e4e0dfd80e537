"""The host half of the library (curve, padding, adjacency bits, configuration checks, table export) built
with AddressSanitizer + UndefinedBehaviorSanitizer and run on the CPU: the same tables as the oracle, no
sanitizer report on valid, ragged, degenerate and invalid configurations."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import jenga_oracle as jo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_16864_amd", "csrc")


def _fnv(a):
    h = 1469598103934665603
    for byte in np.ascontiguousarray(a).tobytes():
        h = ((h ^ byte) * 1099511628211) & 0xFFFFFFFFFFFFFFFF
    return h


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path_factory.mktemp("asan") / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           os.path.join(ROOT, "tests", "host_sanitize_main.cpp"), os.path.join(CSRC, "jenga_plan.cpp"),
           os.path.join(CSRC, "jenga_host.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


VALID = [  # T H W n_text batch heads d m k p beta flags
    (1, 1, 1, 0, 1, 1, 64, 32, 0.3, 0.3, 0.0, 7), (1, 1, 1, 1, 2, 2, 128, 128, 1.0, 0.0, 0.0, 7),
    (3, 5, 7, 40, 2, 3, 64, 32, 0.3, 0.3, 0.25, 7), (7, 9, 13, 200, 1, 3, 128, 128, 0.25, 0.3, 0.0, 7),
    (5, 6, 11, 70, 1, 2, 128, 64, 0.3, 0.5, 0.0, 3), (2, 9, 3, 5, 1, 1, 64, 32, 0.5, 0.0, 0.0, 0),
    (13, 2, 5, 0, 1, 1, 64, 32, 0.5, 0.0, 0.0, 5), (9, 1, 4, 33, 1, 1, 64, 32, 0.05, 0.99, -1.0, 6),
    (8, 64, 127, 512, 1, 2, 64, 32, 0.05, 0.3, 0.0, 7),        # M = 2048, the largest block count taken
    (20, 30, 52, 512, 1, 12, 128, 128, 0.3, 0.9, 0.0, 7), (33, 24, 42, 256, 1, 24, 128, 128, 0.3, 0.3, 0.0, 7),
]
INVALID = [  # (config, expected status)
    ((0, 8, 8, 32, 1, 2, 64, 32, 0.25, 0.3, 0.0, 7), -1), ((4, 8, 8, -1, 1, 2, 64, 32, 0.25, 0.3, 0.0, 7), -1),
    ((4, 8, 8, 32, 1, 2, 64, 32, 0.0, 0.3, 0.0, 7), -1), ((4, 8, 8, 32, 1, 2, 64, 32, 0.25, 1.0, 0.0, 7), -1),
    ((4, 8, 8, 32, 1, 2, 64, 32, 0.25, 0.3, 0.0, 16), -1), ((4, 8, 8, 32, 1, 2, 96, 32, 0.25, 0.3, 0.0, 7), -2),
    ((4, 8, 8, 32, 1, 2, 64, 16, 0.25, 0.3, 0.0, 7), -2), ((400, 400, 400, 32, 1, 2, 64, 32, 0.25, 0.3, 0.0, 7), -2),
    ((8, 64, 128, 512, 1, 2, 64, 32, 0.05, 0.3, 0.0, 7), -2),   # M = 2064 > 2048
    ((2147483647, 2147483647, 2, 0, 1, 1, 64, 32, 0.5, 0.0, 0.0, 7), -2),   # products that overflow 32 bits
    ((16777216, 16777216, 16777216, 0, 1, 1, 64, 32, 0.5, 0.0, 0.0, 7), -2),
    ((4, 8, 8, 32, 70000, 1, 64, 32, 0.25, 0.3, 0.0, 7), -2),
]


def test_host_tables_under_sanitizers(driver):
    lines = "\n".join(" ".join(repr(x) for x in cfg) for cfg in VALID + [c for c, _ in INVALID]) + "\n"
    r = subprocess.run([driver], input=lines, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, "sanitizer report or crash:\n" + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    out = r.stdout.strip().split("\n")
    assert len(out) == 2 * (len(VALID) + len(INVALID)) + 1
    for n, cfg in enumerate(VALID):
        T, H, W, n_text, _, _, _, m, k, _, _, flags = cfg
        lay = jo.Layout(T, H, W, n_text, m, k, flags)
        got = [int(x) for x in out[2 * n].split()]
        assert got[:9] == [0, lay.N_v, lay.M_v, lay.M_c, lay.M, lay.N_pad, lay.pad_v, lay.pad_c, lay.K_top], cfg
        adja = jo.adjacency_mask(lay) if flags & jo.FLAG_ADJACENCY else np.zeros((lay.M_v, lay.M_v), dtype=bool)
        assert got[9:] == [_fnv(lay.perm.astype(np.int32)), _fnv(lay.inv.astype(np.int32)),
                           _fnv(adja.astype(np.uint8))], cfg
        assert out[2 * n + 1] == "ok"
    for n, (cfg, status) in enumerate(INVALID):
        line = out[2 * (len(VALID) + n)].split()
        assert int(line[0]) == status, cfg
        assert [int(x) for x in line[9:]] == [0, 0, 0]
    assert out[-1] == "null -1 -1 -1"
