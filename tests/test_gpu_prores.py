"""GPU parity of jenga_stage_switch (Sec. 3.2, Eq. 4) against the float64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import jenga_inputs as ji
from oracle import prores

pytestmark = pytest.mark.gpu

# float32 window sums of at most 8 terms (upsampling) and two fused multiply-adds: a few ulp of the
# largest term.  |values| stay below ~8 for N(0,1) inputs, so 1e-5 absolute is about 10 float32 ulp there.
ATOL = 1e-5


def run(w, seed, sigma=None):
    from paper_2505_16864_amd import binding as jb
    sigma = w["sigma"] if sigma is None else sigma
    x, e, n = ji.make_latents(w, seed, device="cuda:0")
    out = torch.full((w["channels"],) + tuple(w["out"]), float("nan"), device="cuda:0", dtype=torch.float32)
    jb.jenga_stage_switch(x, e, n, out, w["channels"], w["in"], w["out"], sigma,
                          torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = prores.stage_switch(x.cpu().numpy(), e.cpu().numpy(), n.cpu().numpy(), float(np.float32(sigma)), w["out"])
    return out.cpu().numpy().astype(np.float64), want


@pytest.mark.parametrize("name", ["tiny", "ragged", "down", "down_w16", "up_w12", "up_wide"])
@pytest.mark.parametrize("seed", [0, 1])
def test_small_cases(name, seed):
    got, want = run(ji.STAGE_SWITCHES[name], 7000 + seed)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= ATOL


@pytest.mark.parametrize("sigma", [0.0, 1.0])
def test_sigma_limits(sigma):
    got, want = run(ji.STAGE_SWITCHES["ragged"], 7010, sigma)
    assert np.abs(got - want).max() <= ATOL


def test_same_size_is_elementwise():
    w = {"channels": 2, "in": (3, 6, 9), "out": (3, 6, 9), "sigma": 0.25}
    got, want = run(w, 7020)
    assert np.abs(got - want).max() <= ATOL


def test_full_size_540p_to_720p():
    w = ji.STAGE_SWITCHES["hy540to720"]
    got, want = run(w, 7030)
    assert got.shape == (16, 33, 90, 160)
    assert np.abs(got - want).max() <= ATOL


def test_invalid_arguments_launch_nothing():
    from paper_2505_16864_amd import binding as jb
    w = ji.STAGE_SWITCHES["tiny"]
    x, e, n = ji.make_latents(w, 7040, device="cuda:0")
    out = torch.zeros((w["channels"],) + tuple(w["out"]), device="cuda:0")
    for bad in (-0.1, 1.5, float("nan")):
        with pytest.raises(jb.JengaError) as err:
            jb.jenga_stage_switch(x, e, n, out, w["channels"], w["in"], w["out"], bad)
        assert err.value.status == -1
    with pytest.raises(jb.JengaError):
        jb.jenga_stage_switch(x, e, n, out, w["channels"], (0, 5, 7), w["out"], 0.5)
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
