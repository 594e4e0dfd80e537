"""Pins of the stage-switch oracle (Sec. 3.2, Eq. 4) against what the mathematics and a library fix."""
import numpy as np
import pytest
import torch

from oracle import prores


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


@pytest.mark.parametrize("n_in,n_out", [(3, 4), (34, 45), (60, 80), (5, 5), (4, 8), (7, 3), (1, 6), (9, 2)])
def test_windows_cover_and_match_exact_fractions(n_in, n_out):
    from fractions import Fraction
    import math
    covered = set()
    for o in range(n_out):
        s, e = prores.area_window(o, n_in, n_out)
        assert s == math.floor(Fraction(o * n_in, n_out)) and e == math.ceil(Fraction((o + 1) * n_in, n_out))
        assert 0 <= s < e <= n_in
        covered.update(range(s, e))
    assert covered == set(range(n_in))


@pytest.mark.parametrize("shape,out", [((2, 3, 5, 7), (3, 8, 10)), ((3, 4, 6, 9), (4, 8, 12)), ((1, 2, 34, 60), (2, 45, 80)),
                                       ((2, 5, 7, 9), (3, 4, 5)), ((2, 3, 4, 5), (6, 8, 10))])
def test_upsample_matches_library_area_mode(shape, out):
    x = rnd(shape, 1)
    ref = torch.nn.functional.interpolate(torch.from_numpy(x)[None], size=out, mode="area")[0].numpy()
    np.testing.assert_allclose(prores.upsample_area(x, out), ref, rtol=0, atol=1e-13)


def test_integer_factor_is_replication():
    x = rnd((2, 2, 3, 4), 2)
    up = prores.upsample_area(x, (4, 6, 12))
    np.testing.assert_array_equal(up, x.repeat(2, 1).repeat(2, 2).repeat(3, 3))


def test_constant_field_and_mean_preservation():
    x = np.full((1, 3, 34, 60), 2.5)
    np.testing.assert_allclose(prores.upsample_area(x, (3, 45, 80)), 2.5, atol=1e-15)
    # same size: identity
    y = rnd((2, 3, 4, 5), 3)
    np.testing.assert_array_equal(prores.upsample_area(y, (3, 4, 5)), y)


def test_linear_ramp_hand_values():
    # 1D case written out by hand: 3 cells [0, 3, 6] to 4 cells; windows [0,1) [0,2) [1,3) [2,3)
    x = np.array([0.0, 3.0, 6.0]).reshape(1, 1, 1, 3)
    np.testing.assert_allclose(prores.upsample_area(x, (1, 1, 4)).ravel(), [0.0, 1.5, 4.5, 6.0], atol=0)


def test_stage_switch_limits_and_closed_form():
    x, e = rnd((2, 3, 5, 7), 4), rnd((2, 3, 5, 7), 5)
    n = rnd((2, 3, 8, 10), 6)
    out = (3, 8, 10)
    # sigma = 0: pure upsample of x_t; sigma = 1: pure noise
    np.testing.assert_array_equal(prores.stage_switch(x, e, n, 0.0, out), prores.upsample_area(x, out))
    np.testing.assert_allclose(prores.stage_switch(x, e, n, 1.0, out), n, atol=1e-15)
    # U is linear, so Eq. 4 expands to (1-s) U(x) - (1-s) s U(e) + s n
    s = 0.37
    want = (1 - s) * prores.upsample_area(x, out) - (1 - s) * s * prores.upsample_area(e, out) + s * n
    np.testing.assert_allclose(prores.stage_switch(x, e, n, s, out), want, atol=1e-13)
    # a flow-matching state x_t = (1-s) x0 + s eps with the exact eps as prediction recovers U(x0)
    x0 = rnd((2, 3, 5, 7), 7)
    xt = (1 - s) * x0 + s * e
    got = prores.stage_switch(xt, e, np.zeros_like(n), s, out)
    np.testing.assert_allclose(got, (1 - s) * (1 - s) * prores.upsample_area(x0, out), atol=1e-13)
