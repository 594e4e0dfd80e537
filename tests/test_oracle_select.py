"""Pins for the oracle's block selection (Sec. 3.1 Eq. 3; Alg. 3; appendix Eq. 5)."""
import itertools
import os
import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import jenga_oracle as jo

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand_curve_tensor(rng, lay, B=1, heads=2, d=8):
    x = rng.standard_normal((B, heads, lay.N_pad, d))
    x[:, :, ~lay.valid] = 0.0
    return x


def test_block_pool_constant_blocks_and_partial_mean():
    lay = jo.Layout(3, 5, 7, 40, 32, 0.3)        # last vision block has 9 valid tokens, last text block 8
    x = np.zeros((1, 1, lay.N_pad, 3))
    for j in range(lay.M):
        x[0, 0, j * 32:(j + 1) * 32] = [j + 1.0, -2.0 * j, 0.5]
    x[:, :, ~lay.valid] = 0.0                     # pads are zero, must not dilute the mean
    got = jo.block_pool(x, lay, lay.M)
    for j in range(lay.M):
        assert np.allclose(got[0, 0, j], [j + 1.0, -2.0 * j, 0.5], rtol=0, atol=1e-15)
    # a ramp inside the partial block: mean over the 9 valid rows only
    x[0, 0, 96:105, 0] = np.arange(9)
    assert jo.block_pool(x, lay, 4)[0, 0, 3, 0] == pytest.approx(4.0, abs=1e-15)


def test_relevance_is_scaled_softmax_of_pooled_products():
    rng = np.random.default_rng(1)
    qh = rng.standard_normal((2, 3, 5, 16))
    kh = rng.standard_normal((2, 3, 7, 16))
    R = jo.relevance(qh, kh)
    assert R.shape == (2, 3, 5, 7)
    assert np.allclose(R.sum(-1), 1.0, atol=1e-14)
    for b, h, i in itertools.product(range(2), range(3), range(5)):
        s = np.array([sum(qh[b, h, i, c] * kh[b, h, j, c] for c in range(16)) / 4.0 for j in range(7)])
        assert np.allclose(R[b, h, i], scipy_softmax(s), atol=1e-14)
    # zero queries -> uniform rows
    assert np.allclose(jo.relevance(np.zeros((1, 1, 2, 4)), kh[:1, :1, :, :4]), 1.0 / 7)
    # the 1/sqrt(d_k) matters: with d = 4 the logits are halved
    q1 = np.array([[[[2.0, 0, 0, 0]]]])
    k1 = np.array([[[[1.0, 0, 0, 0], [0, 0, 0, 0]]]])
    assert jo.relevance(q1, k1)[0, 0, 0, 0] == pytest.approx(np.e / (np.e + 1.0), abs=1e-15)


def test_importance_row_worked_examples():
    with open(os.path.join(GOLD, "selection_worked.txt")) as f:
        lines = [l for l in f if l.strip() and not l.startswith("#")]
    assert len(lines) >= 7
    for line in lines:
        k_top, p, r, want = [s.strip() for s in line.split(";")]
        r = np.array([float(x) for x in r.split()])
        row, n_k = jo.importance_row(r, int(k_top), float(p))
        assert np.array_equal(np.nonzero(row)[0], [int(x) for x in want.split()]), line
        assert n_k == row.sum()


def _brute_force_row(r, K_top, p):
    """Eq. 5 by exhaustive search: the smallest set with sum > p is a set of the largest values;
    rank every column by counting, then grow the prefix."""
    M = len(r)
    rank = [sum(1 for jj in range(M) if r[jj] > r[j] or (r[jj] == r[j] and jj < j)) for j in range(M)]
    by_rank = sorted(range(M), key=lambda j: rank[j])
    n, acc = 0, 0.0
    while True:
        acc += r[by_rank[n]]
        n += 1
        if acc > p or n == M:
            break
    n = min(M, max(n, K_top))
    return sorted(by_rank[:n])


def test_importance_against_brute_force_and_eq5_properties():
    rng = np.random.default_rng(2)
    for trial in range(200):
        M = int(rng.integers(1, 12))
        r = scipy_softmax(rng.standard_normal(M) * rng.uniform(0.1, 4))
        K_top = int(rng.integers(1, M + 1))
        p = float(rng.choice([0.0, 0.1, 0.3, 0.5, 0.9, 0.999]))
        row, n_k = jo.importance_row(r, K_top, p)
        sel = np.nonzero(row)[0]
        assert list(sel) == _brute_force_row(r, K_top, p)
        # properties fixed by Sec. 3.1 / Eq. 5
        assert len(sel) >= min(K_top, M)
        assert r[sel].sum() > p or len(sel) == M
        assert r[sel].min() >= r[~row].max() if len(sel) < M else True      # a prefix of the sorted order
        if len(sel) > K_top:                                                # minimal: dropping the smallest breaks > p
            assert r[sel].sum() - r[sel].min() <= p + 1e-15


def test_importance_special_cases():
    rng = np.random.default_rng(4)
    R = scipy_softmax(rng.standard_normal((1, 2, 6, 9)), axis=-1)
    assert (jo.importance_mask(R, 3, 0.0).sum(-1) == 3).all()         # p = 0 -> exactly K_top
    assert jo.importance_mask(R, 9, 0.3).all()                         # k = 1 -> every block
    assert jo.importance_mask(R, 1, 0.999999).sum(-1).min() >= 5       # large p -> nearly all
    # ties: lower index first
    row, _ = jo.importance_row(np.array([0.25, 0.25, 0.25, 0.25]), 2, 0.0)
    assert list(np.nonzero(row)[0]) == [0, 1]


@pytest.mark.parametrize("g,m", [((2, 3, 4), 4), ((3, 3, 3), 5), ((4, 4, 4), 8), ((1, 6, 5), 7), ((2, 2, 9), 6)])
def test_adjacency_against_token_pair_brute_force(g, m):
    T, H, W = g
    lay = jo.Layout(T, H, W, 0, m, 0.5)
    got = jo.adjacency_mask(lay)
    cells = np.stack(np.unravel_index(lay.perm, (T, H, W)), axis=1)     # cell of curve position i
    want = np.zeros((lay.M_v, lay.M_v), dtype=bool)
    for a in range(lay.N_v):
        for b in range(lay.N_v):
            if np.abs(cells[a] - cells[b]).max() <= 1:
                want[a // m, b // m] = True
    assert np.array_equal(got, want)
    assert np.array_equal(got, got.T) and got.diagonal().all()


def test_condition_mask_and_union():
    rng = np.random.default_rng(5)
    lay = jo.Layout(4, 4, 4, 20, 8, 0.25)           # 8 vision blocks, 3 text blocks (last one partial)
    q = _rand_curve_tensor(rng, lay)
    k = _rand_curve_tensor(rng, lay)
    cond = jo.condition_mask(lay)
    assert cond.shape == (8, 11) and cond[:, 8:].all() and not cond[:, :8].any()
    mask, R = jo.build_mask(q, k, lay, 0.3, return_R=True)
    assert mask.shape == (1, 2, 11, 11)
    assert mask[:, :, 8:, :].all()                  # text query blocks see every block (Alg. 2)
    assert mask[:, :, :8, 8:].all()                 # every text key block is on
    top = jo.importance_mask(R, lay.K_top, 0.3)
    adja = jo.adjacency_mask(lay)
    want = top.copy()
    want[:, :, :, 8:] = True
    want[:, :, :, :8] |= adja[None, None]
    assert np.array_equal(mask[:, :, :8], want)
    # switches
    lay_nc = jo.Layout(4, 4, 4, 20, 8, 0.25, flags=jo.FLAG_CURVE | jo.FLAG_ADJACENCY)
    m2 = jo.build_mask(q, k, lay_nc, 0.3)
    assert np.array_equal(m2[:, :, :8, :8], mask[:, :, :8, :8])
    assert np.array_equal(m2[:, :, :8, 8:], top[:, :, :, 8:])
    lay_na = jo.Layout(4, 4, 4, 20, 8, 0.25, flags=jo.FLAG_CURVE | jo.FLAG_CONDITION)
    m3 = jo.build_mask(q, k, lay_na, 0.3)
    assert np.array_equal(m3[:, :, :8, :8], top[:, :, :, :8])


def test_mask_to_lists():
    mask = np.zeros((1, 1, 3, 3), dtype=bool)
    mask[0, 0, 0, [0, 2]] = True
    mask[0, 0, 1, 1] = True
    mask[0, 0, 2] = True
    cnt, idx = jo.mask_to_lists(mask)
    assert cnt.tolist() == [[[2, 1, 3]]]
    assert idx[0, 0, 0, :2].tolist() == [0, 2] and idx[0, 0, 1, 0] == 1 and idx[0, 0, 2].tolist() == [0, 1, 2]


def test_selection_margins_on_hand_worked_rows():
    # dyadic rows: the sorted values, their running sums and therefore both margins are exact
    # row A: sorted .5 .25 .125 .0625 .0625, C = .5 .75 .875 .9375 1
    rA = np.array([0.5, 0.125, 0.25, 0.0625, 0.0625])
    R = rA[None, None, None, :]
    # K_top 1, p .6: n* = 2 -> N_k = 2; gap between 2nd (.25) and 3rd (.125) = .5 of .25; nearest C to p: .5 (|.1|)
    gap, c = jo.selection_margins(R, 1, 0.6)
    assert gap == 0.5 and c == pytest.approx(0.1, abs=1e-15)
    # K_top 3, p .25: N_k = 3; gap (.125 - .0625)/.125 = .5; |C - p| smallest at C_1 = .5 -> .25
    gap, c = jo.selection_margins(R, 3, 0.25)
    assert gap == 0.5 and c == 0.25
    # K_top 4: the 4th and 5th sorted values are equal -> zero gap (a tie the inputs must avoid)
    gap, c = jo.selection_margins(R, 4, 0.25)
    assert gap == 0.0
    # p exactly on a running sum -> zero distance (C_2 = .75)
    gap, c = jo.selection_margins(R, 1, 0.75)
    assert c == 0.0 and gap == 0.5             # n* = #{C <= .75} + 1 = 3, gap between .125 and .0625
    # every block kept: no gap to report
    gap, c = jo.selection_margins(R, 5, 0.0)
    assert gap == np.inf and c == 0.5
    # the minimum is taken over rows: add a row with a smaller gap
    rB = np.array([0.5, 0.25, 0.1875, 0.0625, 0.0])   # K_top 2: (.25 - .1875)/.25 = .25
    gap, c = jo.selection_margins(np.stack([rA, rB])[None, None], 2, 0.0)
    assert gap == 0.25 and c == 0.5
