"""Pins for the oracle's curve and partition (Sec. 3.1 Eq. 2; appendix on re-ordering and partition)."""
import itertools
import os
import numpy as np
import pytest

from oracle.curve import curve_cells, curve_perm, linear_index
from oracle import jenga_oracle as jo

GOLD = os.path.join(os.path.dirname(__file__), "golden")

GRIDS = [(1, 1, 1), (1, 1, 7), (1, 5, 1), (3, 1, 1), (1, 4, 6), (2, 2, 2), (4, 4, 4), (3, 5, 7), (4, 8, 8),
         (8, 16, 16), (5, 6, 11), (7, 7, 7), (2, 9, 3), (13, 2, 5), (6, 10, 15), (21, 30, 52), (33, 24, 42)]


@pytest.mark.parametrize("g", GRIDS)
def test_bijection_and_roundtrip(g):
    T, H, W = g
    perm, inv = curve_perm(T, H, W)
    n = T * H * W
    assert np.array_equal(np.sort(perm), np.arange(n))
    assert np.array_equal(inv[perm], np.arange(n))
    z = np.random.default_rng(0).standard_normal(n)
    z_blk = z[perm]                      # G
    back = np.empty_like(z)
    back[perm] = z_blk                   # G^-1
    assert np.array_equal(back, z)
    assert np.array_equal(z_blk[inv], z)


def test_every_small_grid_is_continuous():
    # consecutive curve positions are 3D neighbours (Chebyshev distance 1), on all grids up to 9^3
    for T, H, W in itertools.product(range(1, 10), repeat=3):
        c = curve_cells(T, H, W)
        assert len(np.unique(linear_index(c, T, H, W))) == T * H * W
        if len(c) > 1:
            assert np.abs(np.diff(c, axis=0)).max() == 1, (T, H, W)


@pytest.mark.parametrize("g", [(21, 30, 52), (33, 24, 42), (33, 45, 80), (32, 45, 80), (20, 30, 52)])
def test_workload_grids_continuous_mostly_unit_steps(g):
    c = curve_cells(*g)
    d = np.abs(np.diff(c, axis=0))
    assert d.max() == 1
    assert (d.sum(axis=1) > 1).mean() < 0.01      # diagonal steps are rare (odd sides only)
    assert tuple(c[0]) == (0, 0, 0)


def test_even_sides_only_unit_steps():
    for g in [(2, 2, 2), (4, 4, 4), (8, 8, 8), (4, 8, 8), (8, 16, 16), (2, 4, 6), (6, 10, 12), (20, 30, 52)]:
        d = np.abs(np.diff(curve_cells(*g), axis=0))
        assert d.sum(axis=1).max() == 1, g


def test_golden_2x2x2_is_the_hilbert_cell():
    want = np.loadtxt(os.path.join(GOLD, "curve_2x2x2.txt"), dtype=np.int64)
    got = curve_cells(2, 2, 2)
    assert np.array_equal(got, want)
    # Hamiltonian path between two adjacent corners
    assert np.abs(got[0] - got[-1]).sum() == 1


def test_power_of_two_cube_blocks_are_octants():
    # Fig. 3 toy: 4x4x4 latent, m = 8 -> 8 blocks; on a 2^n cube a Hilbert order makes every
    # aligned run of 8 cells a 2x2x2 cube, every run of 64 a 4x4x4 cube.
    c = curve_cells(4, 4, 4)
    lay = jo.Layout(4, 4, 4, 0, 8, 0.5)
    assert lay.M_v == 8 and lay.pad_v == 0
    for b in range(8):
        cells = c[b * 8:(b + 1) * 8]
        assert np.array_equal(cells.max(0) - cells.min(0), [1, 1, 1])
        assert np.all(cells.min(0) % 2 == 0)
    c8 = curve_cells(8, 8, 8)
    for b in range(8):
        cells = c8[b * 64:(b + 1) * 64]
        assert np.array_equal(cells.max(0) - cells.min(0), [3, 3, 3])


def test_locality_beats_linear_order():
    # Sec. 3.1: tokens close in 1D stay close in 3D; blocks of the curve order are compact clusters,
    # blocks of the linear thw order are row strips.
    T, H, W, m = 21, 30, 52, 128
    lay_c = jo.Layout(T, H, W, 0, m, 0.3, flags=7)
    lay_l = jo.Layout(T, H, W, 0, m, 0.3, flags=3)
    assert np.array_equal(lay_l.perm, np.arange(T * H * W))

    def bbox_stats(lay):
        cells = np.stack(np.unravel_index(lay.perm, (T, H, W)), axis=1)
        vol, ext = [], []
        for b in range(lay.M_v - 1):
            cc = cells[b * m:(b + 1) * m]
            e = cc.max(0) - cc.min(0) + 1
            vol.append(np.prod(e))
            ext.append(e.max())
        return np.mean(vol), np.mean(ext)

    vol_c, ext_c = bbox_stats(lay_c)
    vol_l, ext_l = bbox_stats(lay_l)
    assert vol_c < 0.6 * vol_l
    assert ext_c * 3 < ext_l


def test_adjacent_block_count_at_720p():
    # appendix: at 720p one block (no. 450) has 20 adjacent blocks; ours need not equal that curve,
    # but the count per block must be of that order.
    lay = jo.Layout(33, 45, 80, 0, 128, 0.3)
    cnt = jo.adjacency_mask(lay).sum(1)
    assert 12 < cnt.mean() < 28 and cnt.max() < 48 and cnt.min() >= 4


def test_partition_table_720p():
    T, H, W, m, blocks, pads = np.loadtxt(os.path.join(GOLD, "partition_720p.txt"), dtype=np.int64)
    lay = jo.Layout(T, H, W, 256, m, 0.3, flags=3)     # linear order: only sizes are needed here
    assert lay.N_v == 118800 and lay.M_v == blocks and lay.pad_v == pads
    assert lay.M_c == 2 and lay.M == 931 and lay.N_pad == 119168 and lay.K_top == 278
    assert abs(2 * pads / lay.N_v * 100 - 0.19) < 0.005


def test_k_top_rounding():
    assert jo.Layout(33, 24, 42, 256, 128, 0.3, flags=3).K_top == 78      # 0.3*260 must not floor to 77
    assert jo.Layout(21, 30, 52, 512, 128, 0.3, flags=3).K_top == 76
    assert jo.Layout(8, 16, 16, 64, 128, 0.3, flags=3).K_top == 4
    assert jo.Layout(4, 8, 8, 32, 32, 0.25, flags=3).K_top == 2
    assert jo.Layout(33, 45, 80, 256, 128, 0.1, flags=3).K_top == 92
    assert jo.Layout(2, 2, 2, 0, 8, 0.01, flags=3).K_top == 1


def test_layout_pads_and_text_placement():
    lay = jo.Layout(3, 5, 7, 40, 32, 0.3)       # 105 vision tokens -> 4 blocks, 23 pads; 40 text -> 2 blocks, 24 pads
    assert (lay.M_v, lay.pad_v, lay.M_c, lay.pad_c) == (4, 23, 2, 24)
    assert lay.valid[:105].all() and not lay.valid[105:128].any()
    assert lay.valid[128:168].all() and not lay.valid[168:].any()
    assert np.array_equal(lay.src_of_pos[128:168], 105 + np.arange(40))
    assert np.array_equal(lay.block_valid_counts(), [32, 32, 32, 9, 32, 8])


def test_permute_unpermute_roundtrip_and_definition():
    rng = np.random.default_rng(3)
    lay = jo.Layout(3, 5, 7, 40, 32, 0.3)
    x = rng.standard_normal((2, 145, 3, 4))
    y = jo.permute(x, lay)
    assert y.shape == (2, 3, lay.N_pad, 4)
    for i in (0, 17, 104):
        assert np.array_equal(y[1, 2, i], x[1, lay.perm[i], 2])
    assert np.array_equal(y[0, 1, 128 + 5], x[0, 105 + 5, 1])
    assert not y[:, :, 105:128].any() and not y[:, :, 168:].any()
    assert np.array_equal(jo.unpermute(y, lay), x)
