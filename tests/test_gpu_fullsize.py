"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The block masks and index lists of EVERY (head, query block) are compared bit for bit with the
oracle (the oracle's selection is cheap); the attention output is compared on sampled query blocks
the oracle computes one by one: the first and the ragged last vision block, both text blocks, and
seeded random ones, in the first, a middle and the last head."""
import numpy as np
import pytest
import torch

import jenga_inputs as ji
from oracle import jenga_oracle as jo
from paper_2505_16864_amd.layer import CarveLayer
from gpu_util import oracle_layout, to_f64, check_output

pytestmark = pytest.mark.gpu

_inputs = {}


def _qkv(name, seed):
    w = ji.WORKLOADS[name]
    key = (w["T"], w["H"], w["W"], w["n_text"], w["heads"], seed)
    if key not in _inputs:
        _inputs.clear()                     # keep one grid's tensors resident at a time
        _inputs[key] = ji.make_qkv(w, seed, device="cuda:0")
    return _inputs[key]


@pytest.mark.parametrize("name,seed", [("wan480p", 3000), ("hy_lowres", 4000), ("hy720p", 5000), ("hy720p_k10", 5000), ("hy720p_k20", 5000), ("wan480p_p90", 3100),
                                       ("max_blocks", 6000)])
def test_full_size(name, seed):
    w = ji.WORKLOADS[name]
    print("workload", name, "seed", seed, flush=True)
    q, k, v = _qkv(name, seed)
    layer = CarveLayer(w, "cuda:0", want_mask=True)
    out = layer.forward(q, k, v)
    torch.cuda.synchronize()
    lay = oracle_layout(w)
    info = layer.info
    assert (info.M_v, info.M, info.N_pad, info.K_top) == (lay.M_v, lay.M, lay.N_pad, lay.K_top)

    # permutation: the curve-side Q equals the oracle's gather, bit for bit (head 0 and last head)
    for h in (0, w["heads"] - 1):
        want = jo.permute(ji.bits(q[:, :, h:h + 1, :]), lay)
        assert np.array_equal(ji.bits(layer.q_c[:, h:h + 1]), want)

    got_mask = layer.mask.cpu().numpy().astype(bool)
    cnt = layer.sel_count.cpu().numpy()
    idx = layer.sel_index.cpu().numpy()
    rng = np.random.default_rng(seed)
    attn_heads = sorted({0, w["heads"] // 2, w["heads"] - 1})
    min_gap, min_c = np.inf, np.inf
    worst = 0.0
    for h in range(w["heads"]):
        qs, ks = [jo.permute(to_f64(x[:, :, h:h + 1, :]), lay) for x in (q, k)]
        want_mask, R = jo.build_mask(qs, ks, lay, w["p"], return_R=True)
        gap, cdist = jo.selection_margins(R, lay.K_top, w["p"])
        min_gap, min_c = min(min_gap, gap), min(min_c, cdist)
        assert np.array_equal(got_mask[:, h], want_mask[:, 0]), "mask differs in head %d" % h
        assert np.array_equal(cnt[:, h], want_mask[:, 0].sum(-1))
        for i in rng.integers(0, lay.M, 8):          # ascending lists on sampled rows
            n = cnt[0, h, i]
            assert np.array_equal(idx[0, h, i, :n], np.nonzero(want_mask[0, 0, i])[0])
        if h in attn_heads:
            vs = jo.permute(to_f64(v[:, :, h:h + 1, :]), lay)
            blocks = [0, lay.M_v - 1] + list(range(lay.M_v, lay.M)) + [int(x) for x in rng.integers(1, lay.M_v - 1, 4)]
            got = to_f64(layer.o_c[:, h:h + 1])
            for i in blocks:
                want = jo.attention_block(qs[0, 0], ks[0, 0], vs[0, 0], want_mask[0, 0, i], lay, i)
                sl = slice(i * lay.m, (i + 1) * lay.m)
                worst = max(worst, check_output(got[:, :, sl], want[None, None], "%s head %d block %d" % (name, h, i)))
        print("head", h, "ok", flush=True)
    # float64 leaves room to decide every row
    assert min_gap > 1e-11 and min_c > 1e-11, (min_gap, min_c)
    # un-permute: thw-side output equals the scatter of the curve-side output (sampled head)
    want_thw = jo.unpermute(ji.bits(layer.o_c[:, :1]), lay)
    assert np.array_equal(ji.bits(out[:, :, :1]), want_thw)
    print("%s: masks exact over %d rows, min rel gap %.3g, min |C-p| %.3g, worst abs err %.3g, density %.4f"
          % (name, w["heads"] * lay.M, min_gap, min_c, worst, got_mask.mean()), flush=True)
