"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Every output buffer is filled with a NaN bit pattern before the call; afterwards every valid row of
the whole tensor must be finite and every pad row exactly zero, so a row the work mapping skipped
cannot go unnoticed.  The block masks and index lists of EVERY (head, query block) are compared bit
for bit with the oracle.  The attention output is compared with the oracle on

  * whole heads (every query block): 2 heads at the 720p size, 3 heads at the smaller sizes;
  * in every other head: the first and the ragged last vision block, the text blocks, the blocks on
    both sides of each boundary between the eight runs the work mapping deals to the XCDs
    (i = c*ceil(M_v/8) - 1 and c*ceil(M_v/8)), and seeded random blocks up to 32 per head.

The heavy oracle work is split over several tests per workload so that none runs for minutes.
"""
import numpy as np
import pytest
import torch

import jenga_inputs as ji
from oracle import jenga_oracle as jo
from paper_2505_16864_amd.layer import CarveLayer
from gpu_util import oracle_layout, to_f64, check_output

pytestmark = pytest.mark.gpu

NAN_BITS = 0x7FC1

_state = {}


def _forward(name, seed):
    """Runs the whole path once per (workload, seed) and keeps the layer; one workload resident at a time."""
    key = (name, seed)
    if _state.get("key") != key:
        _state.clear()
        torch.cuda.empty_cache()
        w = ji.WORKLOADS[name]
        print("workload", name, "seed", seed, flush=True)
        q, k, v = ji.make_qkv(w, seed, device="cuda:0")
        layer = CarveLayer(w, "cuda:0", want_mask=True, want_lse=True)
        layer.o_c.view(torch.int16).fill_(NAN_BITS)
        layer.out_thw.view(torch.int16).fill_(NAN_BITS)
        layer.lse.fill_(float("nan"))
        out = layer.forward(q, k, v)
        torch.cuda.synchronize()
        _state.update(key=key, w=w, q=q, k=k, v=v, layer=layer, out=out, lay=oracle_layout(w), masks={})
    return _state


def _head_mask(st, h):
    """Oracle mask and probabilities of one head (cached)."""
    if h not in st["masks"]:
        lay = st["lay"]
        qs, ks = [jo.permute(to_f64(x[:, :, h:h + 1, :]), lay) for x in (st["q"], st["k"])]
        mask, R = jo.build_mask(qs, ks, lay, st["w"]["p"], return_R=True)
        st["masks"][h] = (mask[0, 0], R, qs[0, 0], ks[0, 0])
    return st["masks"][h]


def _check_blocks(st, h, blocks, what):
    lay, layer, w = st["lay"], st["layer"], st["w"]
    mask, _, qs, ks = _head_mask(st, h)
    vs = jo.permute(to_f64(st["v"][:, :, h:h + 1, :]), lay)[0, 0]
    got = to_f64(layer.o_c[:, h:h + 1])
    got_lse = layer.lse[0, h].cpu().numpy().astype(np.float64)
    beta = w.get("text_bias", 0.0)
    worst = 0.0
    for i in blocks:
        want, want_lse = jo.attention_block(qs, ks, vs, mask[i], lay, i, beta=beta, return_lse=True)
        sl = slice(i * lay.m, (i + 1) * lay.m)
        worst = max(worst, check_output(got[:, :, sl], want[None, None], "%s head %d block %d" % (what, h, i)))
        ok = lay.valid[sl]
        assert np.abs(got_lse[sl][ok] - want_lse[ok]).max() <= 1e-3, (what, h, i)
        assert np.isneginf(got_lse[sl][~ok]).all()
    return worst


def _boundary_blocks(lay):
    chunk = -(-lay.M_v // 8)
    b = {0, lay.M_v - 1}
    for c in range(1, 8):
        for i in (c * chunk - 1, c * chunk):
            if 0 <= i < lay.M_v:
                b.add(i)
    return b | set(range(lay.M_v, lay.M))


# (workload, seed, heads compared whole)
SIZES = [("wan480p", 3000, (0, 19, 39)), ("hy_lowres", 4000, (0, 11, 23)), ("hy_lowres_amp", 4000, (0, 12, 23)),
         ("wan13b", 3300, (0, 5, 11)), ("wan13b_paced", 3300, (7,)), ("hy720p", 5000, (0, 23)), ("hy720p_paced", 5000, (11,)), ("hy720p_k10", 5000, ()), ("hy720p_k20", 5000, ()),
         ("wan480p_p90", 3100, (7,)), ("max_blocks", 6000, (0, 1))]


@pytest.mark.parametrize("name,seed", [(n, s) for n, s, _ in SIZES])
def test_every_row_written_masks_and_lists_exact(name, seed):
    st = _forward(name, seed)
    w, lay, layer, out = st["w"], st["lay"], st["layer"], st["out"]
    info = layer.info
    assert (info.M_v, info.M, info.N_pad, info.K_top) == (lay.M_v, lay.M, lay.N_pad, lay.K_top)

    # no row left unwritten, over the whole tensors (checked on the device: these are test-side reductions)
    valid = torch.from_numpy(lay.valid).cuda()
    oc_bits = layer.o_c.view(torch.int16)
    assert torch.isfinite(layer.o_c[:, :, valid].float()).all(), "a valid curve-side row is not finite"
    assert not oc_bits[:, :, ~valid].any(), "a pad row is not zero"
    assert torch.isfinite(out.float()).all(), "a thw-side row is not finite"
    assert torch.isfinite(layer.lse[:, :, valid]).all() and torch.isneginf(layer.lse[:, :, ~valid]).all()

    # permutation: the curve-side Q equals the oracle's gather, bit for bit (head 0 and last head)
    for h in (0, w["heads"] - 1):
        want = jo.permute(ji.bits(st["q"][:, :, h:h + 1, :]), lay)
        assert np.array_equal(ji.bits(layer.q_c[:, h:h + 1]), want)

    got_mask = layer.mask.cpu().numpy().astype(bool)
    cnt = layer.sel_count.cpu().numpy()
    idx = layer.sel_index.cpu().numpy()
    rng = np.random.default_rng(seed)
    min_gap, min_c = np.inf, np.inf
    for h in range(w["heads"]):
        want_mask, R, _, _ = _head_mask(st, h)
        gap, cdist = jo.selection_margins(R, lay.K_top, w["p"])
        min_gap, min_c = min(min_gap, gap), min(min_c, cdist)
        assert np.array_equal(got_mask[0, h], want_mask), "mask differs in head %d" % h
        assert np.array_equal(cnt[0, h], want_mask.sum(-1))
        for i in list(rng.integers(0, lay.M, 8)) + sorted(_boundary_blocks(lay)):     # ascending lists
            n = cnt[0, h, i]
            assert np.array_equal(idx[0, h, i, :n], np.nonzero(want_mask[i])[0])
        if h not in (0, w["heads"] - 1):
            st["masks"].pop(h)              # keep the cache small; the attention tests rebuild what they need
    assert min_gap > 1e-11 and min_c > 1e-11, (min_gap, min_c)      # float64 leaves room to decide every row
    # un-permute: the thw-side output equals the scatter of the curve-side output (two heads)
    for h in (0, w["heads"] - 1):
        want_thw = jo.unpermute(ji.bits(layer.o_c[:, h:h + 1]), lay)
        assert np.array_equal(ji.bits(out[:, :, h:h + 1]), want_thw)
    print("%s: masks exact over %d rows, min rel gap %.3g, min |C-p| %.3g, density %.4f"
          % (name, w["heads"] * lay.M, min_gap, min_c, got_mask.mean()), flush=True)


@pytest.mark.parametrize("name,seed,h", [(n, s, h) for n, s, hs in SIZES for h in hs])
def test_whole_head_against_oracle(name, seed, h):
    st = _forward(name, seed)
    lay = st["lay"]
    worst = _check_blocks(st, h, range(lay.M), name)
    print("%s head %d: all %d query blocks within tolerance, worst abs err %.3g" % (name, h, lay.M, worst), flush=True)


@pytest.mark.parametrize("name,seed,part", [(n, s, part) for n, s, hs in SIZES if n != "max_blocks" for part in (0, 1)])
def test_sampled_blocks_in_every_other_head(name, seed, part):
    st = _forward(name, seed)
    w, lay = st["w"], st["lay"]
    whole = dict((n, hs) for n, _, hs in SIZES)[name]
    rng = np.random.default_rng(seed + 17)
    worst, n_blocks = 0.0, 0
    for h in range(w["heads"]):
        extra = [int(x) for x in rng.integers(1, max(2, lay.M_v - 1), 32)]
        if h in whole or h % 2 != part:
            continue
        blocks = sorted(_boundary_blocks(lay))
        blocks += [i for i in dict.fromkeys(extra) if i not in blocks][: max(0, 32 - len(blocks))]
        worst = max(worst, _check_blocks(st, h, blocks, name))
        n_blocks += len(blocks)
        st["masks"].pop(h, None)
    print("%s part %d: %d sampled query blocks within tolerance, worst abs err %.3g" % (name, part, n_blocks, worst),
          flush=True)
