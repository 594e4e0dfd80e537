"""Helpers for the GPU parity tests: run the HIP library through its binding, run the oracle on the
same seeded bits, compare."""
import numpy as np
import torch

import jenga_inputs as ji
from oracle import jenga_oracle as jo
from paper_2505_16864_amd.layer import CarveLayer

ATOL = 2e-2          # max |gpu - oracle|
RTOL_OF_MAX = 1e-2   # max |gpu - oracle| / max |oracle|, per (batch, head)


def oracle_layout(w, flags=None):
    # bit 3 of the library's flags (paced walk) only changes the order in which the kernel visits the blocks
    flags = w.get("flags", 7) if flags is None else flags
    return jo.Layout(w["T"], w["H"], w["W"], w["n_text"], w["block"], w["topk"], flags & 7)


def to_f64(t):
    return jo.bf16_bits_to_f64(ji.bits(t))


def check_output(got, want, what=""):
    """got, want: float64 arrays [B, heads, rows, d] (or any layout with heads on axis 1)."""
    err = np.abs(got - want)
    assert np.isfinite(got).all(), what + ": non-finite output"
    assert err.max() <= ATOL, "%s: max abs err %.4g" % (what, err.max())
    for b in range(want.shape[0]):
        for h in range(want.shape[1]):
            ref = np.abs(want[b, h]).max()
            if ref > 0:
                assert err[b, h].max() / ref <= RTOL_OF_MAX, "%s: head %d rel-to-max err %.4g" % (
                    what, h, err[b, h].max() / ref)
    return err.max()


def lists_from_gpu(layer):
    cnt = layer.sel_count.cpu().numpy()
    idx = layer.sel_index.cpu().numpy()
    return cnt, idx


def check_lists_against_mask(cnt, idx, mask):
    """Bit-exact: counts, ascending indices, and the dense mask they describe."""
    want_cnt, want_idx = jo.mask_to_lists(mask)
    assert np.array_equal(cnt, want_cnt)
    B, Hh, M, _ = mask.shape
    for b in range(B):
        for h in range(Hh):
            for i in range(M):
                n = cnt[b, h, i]
                assert np.array_equal(idx[b, h, i, :n], want_idx[b, h, i, :n]), (b, h, i)
