"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded
inputs.  Permutation, masks and index lists bit-exact; attention within max-abs 2e-2 and 1e-2 of the
largest reference magnitude per head."""
import math

import numpy as np
import pytest
import torch

import jenga_inputs as ji
from oracle import jenga_oracle as jo
import paper_2505_16864_amd as J
from paper_2505_16864_amd.layer import CarveLayer
from gpu_util import oracle_layout, to_f64, check_output, lists_from_gpu, check_lists_against_mask

pytestmark = pytest.mark.gpu

# small enough for the oracle to finish in seconds, large enough for several tiles and ragged tails
CASES = {
    "tiny": ji.WORKLOADS["tiny"],
    "small": ji.WORKLOADS["small"],
    "ragged_m32_d64": dict(T=3, H=5, W=7, n_text=40, batch=2, heads=3, head_dim=64, block=32, topk=0.3, p=0.3),
    "ragged_m64_d128": dict(T=5, H=6, W=11, n_text=70, batch=1, heads=2, head_dim=128, block=64, topk=0.3, p=0.5),
    "ragged_m128_d128": dict(T=7, H=9, W=13, n_text=200, batch=1, heads=3, head_dim=128, block=128, topk=0.25, p=0.3),
    "m128_d64": dict(T=4, H=10, W=12, n_text=33, batch=1, heads=2, head_dim=64, block=128, topk=0.5, p=0.3),
    "m64_d64_notext": dict(T=4, H=6, W=9, n_text=0, batch=1, heads=2, head_dim=64, block=64, topk=0.4, p=0.2),
    "m32_d128": dict(T=2, H=7, W=9, n_text=5, batch=1, heads=2, head_dim=128, block=32, topk=0.2, p=0.6),
    "single_block": dict(T=1, H=2, W=3, n_text=0, batch=1, heads=1, head_dim=64, block=32, topk=0.3, p=0.3),
    "one_token_each": dict(T=1, H=1, W=1, n_text=1, batch=2, heads=2, head_dim=128, block=128, topk=1.0, p=0.0),
    "wide_M80": dict(T=6, H=20, W=21, n_text=40, batch=1, heads=2, head_dim=64, block=32, topk=0.1, p=0.9),
}


def _run(name, seed=11, flags=7, text_bias=0.0, w_override=None, want_lse=False):
    w = dict(CASES[name])
    if w_override:
        w.update(w_override)
    print("case", name, "seed", seed, "flags", flags, "text_bias", text_bias, flush=True)
    q, k, v = ji.make_qkv(w, seed)
    layer = CarveLayer(w, "cuda:0", text_bias=text_bias, flags=flags, want_mask=True, want_lse=want_lse)
    layer.o_c.view(torch.int16).fill_(0x7FC1)            # NaN pattern: every row must be overwritten
    layer.out_thw.view(torch.int16).fill_(0x7FC1)
    out = layer.forward(q.cuda(), k.cuda(), v.cuda())
    torch.cuda.synchronize()
    lay = oracle_layout(w, flags)
    return w, (q, k, v), layer, out, lay


@pytest.mark.parametrize("name", list(CASES))
def test_permute_and_unpermute_bit_exact(name):
    w = CASES[name]
    print("case", name, flush=True)
    q, _, _ = ji.make_qkv(w, 5)
    layer = CarveLayer(w, "cuda:0")
    lay = oracle_layout(w)
    qd = q.cuda()
    layer.o_c.fill_(7.0)                      # pads must be overwritten with zeros
    J.jenga_curve_permute(layer.plan, qd, layer.o_c)
    torch.cuda.synchronize()
    want = jo.permute(ji.bits(q), lay)
    assert np.array_equal(ji.bits(layer.o_c), want)
    layer.out_thw.fill_(3.0)
    J.jenga_unpermute(layer.plan, layer.o_c, layer.out_thw)
    torch.cuda.synchronize()
    assert np.array_equal(ji.bits(layer.out_thw), ji.bits(q))
    # exported tables equal the oracle's
    perm = np.zeros(lay.N_v, dtype=np.int32)
    inv = np.zeros(lay.N_v, dtype=np.int32)
    adja = np.zeros(lay.M_v * lay.M_v, dtype=np.uint8)
    J.jenga_plan_export(layer.plan, perm, inv, adja)
    assert np.array_equal(perm, lay.perm) and np.array_equal(inv, lay.inv)
    assert np.array_equal(adja.reshape(lay.M_v, lay.M_v).astype(bool), jo.adjacency_mask(lay))


@pytest.mark.parametrize("name", list(CASES))
def test_masks_lists_and_output(name):
    w, (q, k, v), layer, out, lay = _run(name)
    want_out, want_mask, want_oc = jo.carve_layer(ji.bits(q), ji.bits(k), ji.bits(v), lay, w["p"])
    got_mask = layer.mask.cpu().numpy().astype(bool)
    assert np.array_equal(got_mask, want_mask)
    cnt, idx = lists_from_gpu(layer)
    check_lists_against_mask(cnt, idx, want_mask)
    check_output(to_f64(layer.o_c), want_oc, name + " curve side")
    check_output(to_f64(out).transpose(0, 2, 1, 3), want_out.transpose(0, 2, 1, 3), name + " thw side")
    assert not ji.bits(layer.o_c)[:, :, ~lay.valid].any()       # pad query rows are exactly zero


@pytest.mark.parametrize("seed", list(range(100, 108)))
@pytest.mark.parametrize("name", ["ragged_m128_d128", "ragged_m32_d64"])
def test_more_seeds(name, seed):
    w, (q, k, v), layer, out, lay = _run(name, seed=seed)
    want_out, want_mask, _ = jo.carve_layer(ji.bits(q), ji.bits(k), ji.bits(v), lay, w["p"])
    assert np.array_equal(layer.mask.cpu().numpy().astype(bool), want_mask)
    check_output(to_f64(out).transpose(0, 2, 1, 3), want_out.transpose(0, 2, 1, 3), "%s seed %d" % (name, seed))


@pytest.mark.parametrize("flags", [0, 1, 2, 3, 4, 5, 6])
def test_mask_switches(flags):
    w, (q, k, v), layer, out, lay = _run("ragged_m32_d64", seed=12, flags=flags)
    want_out, want_mask, _ = jo.carve_layer(ji.bits(q), ji.bits(k), ji.bits(v), lay, w["p"])
    assert np.array_equal(layer.mask.cpu().numpy().astype(bool), want_mask)
    check_output(to_f64(out).transpose(0, 2, 1, 3), want_out.transpose(0, 2, 1, 3), "flags %d" % flags)


@pytest.mark.parametrize("topk,p", [(0.05, 0.0), (0.3, 0.0), (0.2, 0.5), (0.1, 0.9), (1.0, 0.3), (0.05, 0.99)])
def test_selection_knobs(topk, p):
    w, (q, k, v), layer, out, lay = _run("wide_M80", seed=13, w_override=dict(topk=topk, p=p))
    qc = jo.permute(to_f64(q), lay)
    kc = jo.permute(to_f64(k), lay)
    want_mask, R = jo.build_mask(qc, kc, lay, p, return_R=True)
    gap, cdist = jo.selection_margins(R, lay.K_top, p)
    assert gap > 1e-10 and cdist > 1e-10          # the inputs leave float64 room to decide
    assert np.array_equal(layer.mask.cpu().numpy().astype(bool), want_mask)
    cnt, idx = lists_from_gpu(layer)
    check_lists_against_mask(cnt, idx, want_mask)


def test_all_blocks_selected_equals_dense_attention():
    # p -> 1 selects every block: the kernel must reproduce Eq. 1
    w, (q, k, v), layer, out, lay = _run("ragged_m64_d128", seed=14, w_override=dict(p=0.9999999))
    assert layer.mask.cpu().numpy().all()
    want = jo.dense_attention(to_f64(q), to_f64(k), to_f64(v))
    check_output(to_f64(out).transpose(0, 2, 1, 3), want.transpose(0, 2, 1, 3), "dense")


# The text-attention amplifier (Sec. 3.2; the highlighted lines of Alg. 4) on every kernel shape.  The 128-token
# cases run the half-block kernel the paper's configurations use: ragged_m128_d128 has a last vision block with
# 51 valid tokens (its second half is all padding) and a ragged text block; m128_d64 has a text block with 33
# valid tokens (second half all padding); small has 64 text tokens (again an all-padding half) and no vision pads.
@pytest.mark.parametrize("beta", [-0.5 * math.log(0.5625), -1.5, 3.0])
@pytest.mark.parametrize("name", ["ragged_m32_d64", "ragged_m64_d128", "ragged_m128_d128", "m128_d64", "small"])
def test_text_bias(name, beta):
    w, (q, k, v), layer, out, lay = _run(name, seed=15, text_bias=beta)
    want_out, want_mask, want_oc = jo.carve_layer(ji.bits(q), ji.bits(k), ji.bits(v), lay, w["p"], beta=beta)
    base_out, _, _ = jo.carve_layer(ji.bits(q), ji.bits(k), ji.bits(v), lay, w["p"], beta=0.0)
    assert np.array_equal(layer.mask.cpu().numpy().astype(bool), want_mask)      # the bias plays no part in selection
    check_output(to_f64(layer.o_c), want_oc, "%s text bias %.3f curve side" % (name, beta))
    check_output(to_f64(out).transpose(0, 2, 1, 3), want_out.transpose(0, 2, 1, 3), "%s text bias %.3f" % (name, beta))
    assert not ji.bits(layer.o_c)[:, :, ~lay.valid].any()
    assert np.abs(want_out - base_out).max() > 2e-2      # the bias is visible at this tolerance


def test_text_bias_with_the_ragged_blocks_visited_first():
    # shuffled lists put the ragged vision block (second half all padding) and the ragged text block at the
    # front of some rows, so the running maximum starts from them
    beta = -0.5 * math.log(0.5625)
    w = dict(CASES["ragged_m128_d128"])
    q, k, v = ji.make_qkv(w, 21)
    layer = CarveLayer(w, "cuda:0", text_bias=beta)
    lay = oracle_layout(w)
    rng = np.random.default_rng(2)
    mask = rng.random((w["batch"], w["heads"], lay.M, lay.M)) < 0.5
    mask[:, :, :, lay.M_v - 1] = True
    mask[:, :, :, lay.M - 1] = True
    cnt, idx = jo.mask_to_lists(mask)
    for h in range(idx.shape[1]):
        for i in range(lay.M):
            n = cnt[0, h, i]
            rest = [j for j in idx[0, h, i, :n] if j not in (lay.M_v - 1, lay.M - 1)]
            first = [lay.M_v - 1, lay.M - 1] if i % 2 == 0 else [lay.M - 1, lay.M_v - 1]
            idx[0, h, i, :n] = first + list(rng.permutation(rest))
    layer.permute_in(q.cuda(), k.cuda(), v.cuda())
    layer.sel_count.copy_(torch.from_numpy(cnt))
    layer.sel_index.copy_(torch.from_numpy(idx))
    layer.o_c.view(torch.int16).fill_(0x7FC1)
    layer.attend()
    torch.cuda.synchronize()
    qc, kc, vc = [jo.permute(to_f64(x), lay) for x in (q, k, v)]
    check_output(to_f64(layer.o_c), jo.block_sparse_attention(qc, kc, vc, mask, lay, beta=beta), "ragged first")


# Log-sum-exp output: natural log of the sum of exp(logit) over the visited keys, -inf for pad rows.  float32
# online softmax in base 2 against the float64 oracle: 1e-3 absolute.
@pytest.mark.parametrize("name,beta", [("tiny", 0.0), ("small", 0.0), ("ragged_m32_d64", 0.3), ("ragged_m64_d128", 0.0),
                                       ("ragged_m128_d128", -0.5 * math.log(0.5625)), ("m128_d64", 0.0),
                                       ("one_token_each", 0.0), ("single_block", 0.0)])
def test_log_sum_exp(name, beta):
    w, (q, k, v), layer, out, lay = _run(name, seed=22, text_bias=beta, want_lse=True)
    qc, kc, vc = [jo.permute(to_f64(x), lay) for x in (q, k, v)]
    mask = jo.build_mask(qc, kc, lay, w["p"])
    want_o, want_lse = jo.block_sparse_attention(qc, kc, vc, mask, lay, beta=beta, return_lse=True)
    got = layer.lse.cpu().numpy().astype(np.float64)
    assert np.isneginf(got[:, :, ~lay.valid]).all()
    assert np.abs(got[:, :, lay.valid] - want_lse[:, :, lay.valid]).max() <= 1e-3
    check_output(to_f64(layer.o_c), want_o, name + " with lse")
    # an empty list gives -inf
    layer.sel_count.zero_()
    layer.attend()
    torch.cuda.synchronize()
    assert np.isneginf(layer.lse.cpu().numpy()).all()


# The time-paced walk (flag bit 3): same set of blocks, visited in an order that depends on a clock.  Same masks,
# outputs within the same tolerance, log-sum-exp within 1e-3; two runs agree within rounding, not bit for bit.
@pytest.mark.parametrize("name,beta", [("small", 0.0), ("ragged_m128_d128", 0.0), ("ragged_m128_d128", 0.5),
                                       ("m128_d64", -0.5 * math.log(0.5625)), ("one_token_each", 0.0)])
def test_paced_walk(name, beta):
    w, (q, k, v), layer, out, lay = _run(name, seed=23, flags=15, text_bias=beta, want_lse=True)
    qc, kc, vc = [jo.permute(to_f64(x), lay) for x in (q, k, v)]
    mask = jo.build_mask(qc, kc, lay, w["p"])
    assert np.array_equal(layer.mask.cpu().numpy().astype(bool), mask)
    want_o, want_lse = jo.block_sparse_attention(qc, kc, vc, mask, lay, beta=beta, return_lse=True)
    check_output(to_f64(layer.o_c), want_o, name + " paced walk")
    got_lse = layer.lse.cpu().numpy().astype(np.float64)
    assert np.isneginf(got_lse[:, :, ~lay.valid]).all()
    assert np.abs(got_lse[:, :, lay.valid] - want_lse[:, :, lay.valid]).max() <= 1e-3
    assert not ji.bits(layer.o_c)[:, :, ~lay.valid].any()
    first = to_f64(layer.o_c).copy()
    for _ in range(3):                      # the order may change from run to run, the result only within rounding
        layer.o_c.view(torch.int16).fill_(0x7FC1)
        layer.attend()
        torch.cuda.synchronize()
        again = to_f64(layer.o_c)
        assert np.abs(again - first).max() <= 2 ** -7 * max(1.0, np.abs(first).max())
        check_output(again, want_o, name + " paced walk, repeated")


def test_paced_walk_flag_is_ignored_for_other_block_sizes():
    # blocks of 32 and 64 tokens have the in-order walk only: with the flag the output is the same, bit for bit
    for name in ("ragged_m32_d64", "ragged_m64_d128"):
        w, (q, k, v), layer, out, lay = _run(name, seed=25, flags=15)
        paced = ji.bits(out).copy()
        w, (q, k, v), layer, out, lay = _run(name, seed=25, flags=7)
        assert np.array_equal(ji.bits(out), paced)


def test_paced_walk_with_given_lists_and_duplicates():
    # lists in random order with every block listed twice: the paced walk visits each block once
    w = dict(CASES["ragged_m128_d128"])
    q, k, v = ji.make_qkv(w, 24)
    layer = CarveLayer(w, "cuda:0", flags=15)
    lay = oracle_layout(w)
    rng = np.random.default_rng(3)
    mask = rng.random((w["batch"], w["heads"], lay.M, lay.M)) < 0.45
    mask[:, :, np.arange(lay.M), np.arange(lay.M)] = True
    cnt, idx = jo.mask_to_lists(mask)
    idx2 = np.full((w["batch"], w["heads"], lay.M, lay.M), -1, dtype=np.int32)
    cnt2 = np.zeros_like(cnt)
    for h in range(idx.shape[1]):
        for i in range(lay.M):
            n = cnt[0, h, i]
            twice = rng.permutation(np.concatenate([idx[0, h, i, :n], idx[0, h, i, :n]]))[: lay.M]
            keep = set(twice.tolist())
            mask[0, h, i] = False
            mask[0, h, i, list(keep)] = True
            idx2[0, h, i, : len(twice)] = twice
            cnt2[0, h, i] = len(twice)
    layer.permute_in(q.cuda(), k.cuda(), v.cuda())
    layer.sel_count.copy_(torch.from_numpy(cnt2))
    layer.sel_index.copy_(torch.from_numpy(idx2))
    layer.o_c.view(torch.int16).fill_(0x7FC1)
    layer.attend()
    torch.cuda.synchronize()
    qc, kc, vc = [jo.permute(to_f64(x), lay) for x in (q, k, v)]
    check_output(to_f64(layer.o_c), jo.block_sparse_attention(qc, kc, vc, mask, lay), "paced, duplicates")


def test_attention_with_given_lists_and_constant_values():
    # feed the oracle's lists of a random mask (not produced by selection) and a constant V
    w = dict(CASES["ragged_m128_d128"])
    q, k, v = ji.make_qkv(w, 16)
    v[:] = torch.tensor(np.linspace(-2, 2, w["head_dim"]), dtype=torch.bfloat16)
    layer = CarveLayer(w, "cuda:0")
    lay = oracle_layout(w)
    rng = np.random.default_rng(0)
    mask = rng.random((w["batch"], w["heads"], lay.M, lay.M)) < 0.4
    mask[:, :, np.arange(lay.M), np.arange(lay.M)] = True
    cnt, idx = jo.mask_to_lists(mask)
    layer.permute_in(q.cuda(), k.cuda(), v.cuda())
    layer.sel_count.copy_(torch.from_numpy(cnt))
    layer.sel_index.copy_(torch.from_numpy(idx))
    layer.attend()
    torch.cuda.synchronize()
    got = to_f64(layer.o_c)
    want_row = to_f64(v[0, 0, 0])
    assert np.abs(got[:, :, lay.valid] - want_row).max() <= 2e-2
    qc, kc, vc = [jo.permute(to_f64(x), lay) for x in (q, k, v)]
    check_output(got, jo.block_sparse_attention(qc, kc, vc, mask, lay), "given lists")


# Logits that climb by ~14 base-2 units per key block along the curve: with lists in ascending order the sums
# of probabilities taken against an old reference leave any fixed range every few blocks, so the reference has
# to move several times per row (Alg. 4's rescaling of l and O); descending lists never move it after the first
# block.  Curve-side tensors are written directly; the oracle gets the same bits.
@pytest.mark.parametrize("flags", [7, 15])
@pytest.mark.parametrize("order", ["ascending", "descending", "shuffled"])
@pytest.mark.parametrize("name", ["ragged_m128_d128", "ragged_m64_d128", "wide_M80"])
def test_reference_moves_when_logits_grow_along_the_list(name, order, flags):
    w = dict(CASES[name])
    lay = oracle_layout(w)
    B_, Hh, D = w["batch"], w["heads"], w["head_dim"]
    layer = CarveLayer(w, "cuda:0", flags=flags, want_lse=True)
    rng = np.random.default_rng(31)
    ramp = np.linspace(0.0, 8.0 * math.sqrt(128.0 / D), lay.N_pad)[None, None, :, None]
    qc = 1.0 + 0.25 * rng.standard_normal((B_, Hh, lay.N_pad, D))
    kc = ramp * (1.0 + 0.25 * rng.standard_normal((B_, Hh, lay.N_pad, D)))
    vc = rng.standard_normal((B_, Hh, lay.N_pad, D))
    for x in (qc, kc, vc):
        x[:, :, ~lay.valid] = 0.0
    tq, tk, tv = [torch.from_numpy(x).to(torch.bfloat16) for x in (qc, kc, vc)]
    layer.q_c.copy_(tq)
    layer.k_c.copy_(tk)
    layer.v_c.copy_(tv)
    mask = rng.random((B_, Hh, lay.M, lay.M)) < 0.7
    mask[:, :, np.arange(lay.M), np.arange(lay.M)] = True
    cnt, idx = jo.mask_to_lists(mask)
    for b in range(B_):
        for h in range(Hh):
            for i in range(lay.M):
                n = cnt[b, h, i]
                if order == "descending":
                    idx[b, h, i, :n] = idx[b, h, i, :n][::-1]
                elif order == "shuffled":
                    idx[b, h, i, :n] = rng.permutation(idx[b, h, i, :n])
    layer.sel_count.copy_(torch.from_numpy(cnt))
    layer.sel_index.copy_(torch.from_numpy(idx))
    layer.o_c.view(torch.int16).fill_(0x7FC1)
    layer.attend()
    torch.cuda.synchronize()
    f64 = [to_f64(t) for t in (tq, tk, tv)]
    want_o, want_lse = jo.block_sparse_attention(f64[0], f64[1], f64[2], mask, lay, return_lse=True)
    assert np.median(want_lse[:, :, lay.valid]) > 40.0   # a row's logits really span tens of e-folds above 0
    check_output(to_f64(layer.o_c), want_o, "%s %s flags %d" % (name, order, flags))
    got = layer.lse.cpu().numpy().astype(np.float64)
    assert np.abs(got[:, :, lay.valid] - want_lse[:, :, lay.valid]).max() <= 1e-3


@pytest.mark.parametrize("name", ["ragged_m128_d128", "ragged_m64_d128"])
def test_lists_in_any_order_give_the_same_attention(name):
    # Alg. 4 sums over a set of blocks: the order of the list must not matter beyond rounding
    w = dict(CASES[name])
    q, k, v = ji.make_qkv(w, 19)
    layer = CarveLayer(w, "cuda:0")
    lay = oracle_layout(w)
    rng = np.random.default_rng(1)
    mask = rng.random((w["batch"], w["heads"], lay.M, lay.M)) < 0.5
    mask[:, :, np.arange(lay.M), np.arange(lay.M)] = True
    cnt, idx = jo.mask_to_lists(mask)
    for b in range(idx.shape[0]):
        for h in range(idx.shape[1]):
            for i in range(lay.M):
                n = cnt[b, h, i]
                idx[b, h, i, :n] = rng.permutation(idx[b, h, i, :n])
    layer.permute_in(q.cuda(), k.cuda(), v.cuda())
    layer.sel_count.copy_(torch.from_numpy(cnt))
    layer.sel_index.copy_(torch.from_numpy(idx))
    layer.attend()
    torch.cuda.synchronize()
    qc, kc, vc = [jo.permute(to_f64(x), lay) for x in (q, k, v)]
    check_output(to_f64(layer.o_c), jo.block_sparse_attention(qc, kc, vc, mask, lay), "shuffled lists")


def test_malformed_lists_do_not_fault():
    w = dict(CASES["tiny"])
    q, k, v = ji.make_qkv(w, 17)
    layer = CarveLayer(w, "cuda:0")
    layer.permute_in(q.cuda(), k.cuda(), v.cuda())
    layer.sel_count.fill_(10 ** 6)            # clamped to M
    layer.sel_index.fill_(-5)                 # clamped to block 0
    layer.sel_index[:, :, :, 1] = 10 ** 6     # clamped to block M-1
    layer.attend()
    layer.sel_count.zero_()                   # no keys: zero rows
    layer.o_c.fill_(1.0)
    layer.attend()
    torch.cuda.synchronize()
    assert not ji.bits(layer.o_c).any()


def test_workspace_and_alignment_errors():
    w = dict(CASES["tiny"])
    layer = CarveLayer(w, "cuda:0")
    with pytest.raises(J.JengaError) as e:
        J.jenga_select_blocks(layer.plan, layer.q_c, layer.k_c, layer.sel_count, layer.sel_index, None,
                              layer.ws_select, layer.info.select_workspace_bytes - 1)
    assert e.value.status == -3
    with pytest.raises(J.JengaError) as e:
        J.jenga_block_sparse_attn(layer.plan, layer.q_c, layer.k_c, layer.v_c, layer.sel_count, layer.sel_index,
                                  layer.o_c, None, layer.ws_attn.data_ptr() + 16, layer.info.attn_workspace_bytes)
    assert e.value.status == -1


def test_deterministic():
    w, (q, k, v), layer, out, lay = _run("ragged_m128_d128", seed=18)
    first = ji.bits(out).copy()
    first_idx = layer.sel_index.cpu().numpy().copy()
    out2 = layer.forward(q.cuda(), k.cuda(), v.cuda())
    torch.cuda.synchronize()
    assert np.array_equal(ji.bits(out2), first)
    assert np.array_equal(layer.sel_index.cpu().numpy(), first_idx)
