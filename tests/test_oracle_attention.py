"""Pins for the oracle's attention (Eq. 1; Alg. 2; Alg. 4; the text-attention amplifier of Sec. 3.2)."""
import math
import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import jenga_oracle as jo


def _inputs(rng, lay, B=1, heads=2, d=8):
    n = lay.N_v + lay.n_text
    return [rng.standard_normal((B, n, heads, d)) for _ in range(3)]


def _loop_attention(q, k, v):
    """Eq. 1 with explicit loops on [N, d] arrays."""
    N, d = q.shape
    out = np.zeros_like(q)
    for r in range(N):
        logit = [sum(q[r, c] * k[s, c] for c in range(d)) / math.sqrt(d) for s in range(k.shape[0])]
        w = scipy_softmax(np.array(logit))
        for s in range(k.shape[0]):
            out[r] += w[s] * v[s]
    return out


def test_dense_attention_against_loops():
    rng = np.random.default_rng(0)
    q, k, v = [rng.standard_normal((2, 7, 2, 4)) for _ in range(3)]
    got = jo.dense_attention(q, k, v)
    for b in range(2):
        for h in range(2):
            assert np.allclose(got[b, :, h], _loop_attention(q[b, :, h], k[b, :, h], v[b, :, h]), atol=1e-13)


@pytest.mark.parametrize("g,n_text,m", [((2, 2, 2), 0, 4), ((4, 4, 4), 8, 8), ((3, 5, 7), 40, 32), ((4, 8, 8), 32, 32),
                                        ((2, 3, 5), 3, 8)])
def test_all_blocks_selected_equals_dense(g, n_text, m):
    # B = all ones must reproduce Eq. 1 exactly (up to rounding), pads and re-ordering included
    rng = np.random.default_rng(1)
    lay = jo.Layout(*g, n_text, m, 1.0)
    q, k, v = _inputs(rng, lay)
    want = jo.dense_attention(q, k, v)
    qc, kc, vc = [jo.permute(x, lay) for x in (q, k, v)]
    mask = jo.build_mask(qc, kc, lay, 0.3)
    if n_text == 0:
        assert mask.all()                   # k = 1 selects everything (K_top = M_v = M)
    # with text blocks K_top = k*M_v < M (Alg. 3 step 6), so force the all-ones mask
    mask = np.ones_like(mask)
    oc = jo.block_sparse_attention(qc, kc, vc, mask, lay)
    assert np.allclose(jo.unpermute(oc, lay), want, atol=1e-12)
    assert not oc[:, :, ~lay.valid].any()   # pad query rows are zero


def test_sparse_mask_equals_dense_restricted_to_selected_keys():
    rng = np.random.default_rng(2)
    lay = jo.Layout(3, 5, 7, 40, 32, 0.3)
    q, k, v = _inputs(rng, lay, heads=1)
    qc, kc, vc = [jo.permute(x, lay) for x in (q, k, v)]
    mask = rng.random((1, 1, lay.M, lay.M)) < 0.5
    mask[0, 0, np.arange(lay.M), np.arange(lay.M)] = True
    oc = jo.block_sparse_attention(qc, kc, vc, mask, lay)
    m = lay.m
    for i in range(lay.M):
        keys = [c for j in np.nonzero(mask[0, 0, i])[0] for c in range(j * m, (j + 1) * m) if lay.valid[c]]
        for r in range(i * m, (i + 1) * m):
            if not lay.valid[r]:
                assert not oc[0, 0, r].any()
                continue
            want = _loop_attention(qc[0, 0, r:r + 1], kc[0, 0, keys], vc[0, 0, keys])[0]
            assert np.allclose(oc[0, 0, r], want, atol=1e-12)


def test_block_diagonal_mask_is_independent_per_block():
    rng = np.random.default_rng(3)
    lay = jo.Layout(4, 4, 4, 0, 8, 0.5)
    q, k, v = _inputs(rng, lay, heads=1)
    qc, kc, vc = [jo.permute(x, lay) for x in (q, k, v)]
    mask = np.eye(lay.M, dtype=bool)[None, None]
    oc = jo.block_sparse_attention(qc, kc, vc, mask, lay)
    for i in range(lay.M):
        s = slice(i * 8, (i + 1) * 8)
        want = jo.dense_attention(qc[:, :, s].transpose(0, 2, 1, 3), kc[:, :, s].transpose(0, 2, 1, 3),
                                  vc[:, :, s].transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
        assert np.allclose(oc[:, :, s], want, atol=1e-13)


def test_constant_values_give_that_constant():
    rng = np.random.default_rng(4)
    lay = jo.Layout(2, 3, 5, 3, 8, 0.3)
    q, k, v = _inputs(rng, lay)
    v[:] = np.array([1.5, -2, 0, 3, 1, 1, 1, 7.0])
    qc, kc, vc = [jo.permute(x, lay) for x in (q, k, v)]
    mask = jo.build_mask(qc, kc, lay, 0.3)
    oc = jo.block_sparse_attention(qc, kc, vc, mask, lay)
    assert np.allclose(oc[:, :, lay.valid], v[0, 0, 0], atol=1e-13)


def test_text_bias_reweights_text_keys_for_vision_queries_only():
    # Sec. 3.2: score q_v k_c^T + beta.  Adding beta to a logit multiplies that key's weight by e^beta.
    rng = np.random.default_rng(5)
    lay = jo.Layout(2, 2, 4, 6, 8, 1.0)          # 2 vision blocks, 1 text block (6 valid)
    q, k, v = _inputs(rng, lay, heads=1)
    qc, kc, vc = [jo.permute(x, lay) for x in (q, k, v)]
    mask = np.ones((1, 1, 3, 3), dtype=bool)
    beta = -0.5 * math.log(0.5625)               # rho = 0.5, 0.75x resolution stage (Tab. 4)
    got = jo.block_sparse_attention(qc, kc, vc, mask, lay, beta=beta)
    base = jo.block_sparse_attention(qc, kc, vc, mask, lay, beta=0.0)
    valid = np.nonzero(lay.valid)[0]
    for r in valid:
        logit = kc[0, 0, valid] @ qc[0, 0, r] / math.sqrt(8)
        w = np.exp(logit - logit.max())
        if r < 16:                                # vision query: text keys (positions >= 16) amplified
            w[valid >= 16] *= math.exp(beta)
        w /= w.sum()
        assert np.allclose(got[0, 0, r], w @ vc[0, 0, valid], atol=1e-13)
    assert np.allclose(got[0, 0, 16:], base[0, 0, 16:], atol=0)        # text queries unbiased
    assert not np.allclose(got[0, 0, :16], base[0, 0, :16], atol=1e-6)


def test_bf16_helpers_roundtrip():
    x = np.array([0.0, 1.0, -1.5, 3.140625, 1e-3, 65280.0, -0.33203125])
    b = jo.f64_to_bf16_bits(x)
    y = jo.bf16_bits_to_f64(b)
    assert np.allclose(y, x, rtol=2 ** -8)
    assert np.array_equal(jo.f64_to_bf16_bits(y), b)
    assert jo.bf16_bits_to_f64(np.array([0x3F80, 0xC000, 0x3FC0], dtype=np.uint16)).tolist() == [1.0, -2.0, 1.5]
    # round to nearest even at the tie 1 + 2^-8
    assert jo.f64_to_bf16_bits(np.array([1.00390625]))[0] == 0x3F80
    assert jo.f64_to_bf16_bits(np.array([1.01171875]))[0] == 0x3F82


def test_whole_layer_on_tiny_workload_matches_dense_when_all_selected():
    import jenga_inputs as ji
    w = dict(ji.WORKLOADS["tiny"])
    q, k, v = ji.make_qkv(w, seed=7)
    lay = jo.Layout(w["T"], w["H"], w["W"], w["n_text"], w["block"], 1.0)
    out, mask, _ = jo.carve_layer(ji.bits(q), ji.bits(k), ji.bits(v), lay, 0.9999999)    # p -> 1 selects every block
    want = jo.dense_attention(*[jo.bf16_bits_to_f64(ji.bits(x)) for x in (q, k, v)])
    assert mask.all() and np.allclose(out, want, atol=1e-12)
    # and with the real top-k the output stays close to dense but is not equal to it
    lay2 = jo.Layout(w["T"], w["H"], w["W"], w["n_text"], w["block"], w["topk"])
    out2, mask2, _ = jo.carve_layer(ji.bits(q), ji.bits(k), ji.bits(v), lay2, w["p"])
    assert not mask2.all()
    assert np.abs(out2 - want).max() > 1e-6 and np.abs(out2 - want).mean() < np.abs(want).mean()


def test_lse_against_explicit_loops_and_library_logsumexp():
    # the normaliser of Eq. 1 over the visited keys: log sum exp(q.k/sqrt(d) + bias), natural log
    from scipy.special import logsumexp
    rng = np.random.default_rng(8)
    lay = jo.Layout(3, 5, 7, 40, 32, 0.3)        # ragged vision tail (9 valid) and ragged text tail (8 valid)
    q, k, v = _inputs(rng, lay, heads=1)
    qc, kc, vc = [jo.permute(x, lay) for x in (q, k, v)]
    mask = rng.random((1, 1, lay.M, lay.M)) < 0.5
    mask[0, 0, np.arange(lay.M), np.arange(lay.M)] = True
    beta = 0.4
    out, lse = jo.block_sparse_attention(qc, kc, vc, mask, lay, beta=beta, return_lse=True)
    assert np.array_equal(out, jo.block_sparse_attention(qc, kc, vc, mask, lay, beta=beta))
    m, d = lay.m, 8
    for i in range(lay.M):
        for r in range(i * m, (i + 1) * m):
            if not lay.valid[r]:
                assert lse[0, 0, r] == -np.inf
                continue
            logits = []
            for j in np.nonzero(mask[0, 0, i])[0]:
                for c in range(j * m, (j + 1) * m):
                    if lay.valid[c]:
                        s = sum(qc[0, 0, r, e] * kc[0, 0, c, e] for e in range(d)) / math.sqrt(d)
                        logits.append(s + (beta if (i < lay.M_v and j >= lay.M_v) else 0.0))
            assert lse[0, 0, r] == pytest.approx(logsumexp(np.array(logits)), abs=1e-12)
            assert lse[0, 0, r] == pytest.approx(math.log(sum(math.exp(x) for x in logits)), abs=1e-12)


def test_lse_merges_disjoint_key_sets():
    # two disjoint visited sets A and B: lse(A u B) = log(e^lse(A) + e^lse(B)) and the outputs
    # combine with those weights -- the identity that makes the value usable downstream
    rng = np.random.default_rng(9)
    lay = jo.Layout(2, 4, 4, 5, 8, 0.5)
    q, k, v = _inputs(rng, lay, heads=2)
    qc, kc, vc = [jo.permute(x, lay) for x in (q, k, v)]
    full = np.ones((1, 2, lay.M, lay.M), dtype=bool)
    a = np.zeros_like(full)
    a[..., : lay.M // 2] = True
    b = full & ~a
    o, l = jo.block_sparse_attention(qc, kc, vc, full, lay, return_lse=True)
    oa, la = jo.block_sparse_attention(qc, kc, vc, a, lay, return_lse=True)
    ob, lb = jo.block_sparse_attention(qc, kc, vc, b, lay, return_lse=True)
    ok = lay.valid
    assert np.allclose(l[:, :, ok], np.logaddexp(la[:, :, ok], lb[:, :, ok]), atol=1e-12)
    wa = np.exp(la[:, :, ok] - l[:, :, ok])[..., None]
    wb = np.exp(lb[:, :, ok] - l[:, :, ok])[..., None]
    assert np.allclose(o[:, :, ok], wa * oa[:, :, ok] + wb * ob[:, :, ok], atol=1e-12)
    # one key with logit exactly 0 (zero query): lse = log(number of keys)
    z = np.zeros_like(qc)
    _, l0 = jo.block_sparse_attention(z, kc, vc, full, lay, return_lse=True)
    assert np.allclose(l0[:, :, ok], math.log(ok.sum()), atol=1e-14)
    # a row list that is empty gives -inf and a zero row
    none = np.zeros_like(full)
    o_n, l_n = jo.block_sparse_attention(qc, kc, vc, none, lay, return_lse=True)
    assert not o_n.any() and np.isneginf(l_n).all()
