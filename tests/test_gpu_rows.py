"""GPU parity of jenga_curve_permute_rows (f_blk = G(f), appendix "Frequency re-ordering"): bit-exact."""
import numpy as np
import pytest
import torch

import jenga_inputs as ji
from oracle import jenga_oracle as jo

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,cols", [("tiny", 4), ("tiny", 128), ("small", 32), ("hy_lowres", 128), ("small", 1024)])
def test_rows_follow_the_tokens(name, cols):
    from paper_2505_16864_amd import binding as jb
    w = ji.WORKLOADS[name]
    lay = jo.Layout(w["T"], w["H"], w["W"], w["n_text"], w["block"], w["topk"])
    n_src = lay.N_v + w["n_text"]
    g = torch.Generator().manual_seed(8100 + cols)
    table = torch.randn((n_src, cols), generator=g, dtype=torch.float32)
    cfg = jb.make_config(w["T"], w["H"], w["W"], w["n_text"], w["batch"], w["heads"], w["head_dim"], w["block"],
                         w["topk"], w["p"])
    plan = jb.jenga_plan_create(cfg)
    try:
        src = table.to("cuda:0")
        dst = torch.full((lay.N_pad, cols), float("nan"), device="cuda:0", dtype=torch.float32)
        jb.jenga_curve_permute_rows(plan, src, dst, cols * 4, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        got = dst.cpu().numpy()
    finally:
        jb.jenga_plan_destroy(plan)
    want = jo.permute(table.numpy().astype(np.float64)[None, :, None, :], lay)[0, 0]
    assert got.shape == want.shape
    assert np.array_equal(got.astype(np.float64), want)


def test_row_width_must_be_a_power_of_two():
    from paper_2505_16864_amd import binding as jb
    w = ji.WORKLOADS["tiny"]
    cfg = jb.make_config(w["T"], w["H"], w["W"], w["n_text"], w["batch"], w["heads"], w["head_dim"], w["block"],
                         w["topk"], w["p"])
    plan = jb.jenga_plan_create(cfg)
    try:
        buf = torch.zeros(1 << 16, device="cuda:0")
        for bad in (0, 8, 48, 8192):
            with pytest.raises(jb.JengaError) as err:
                jb.jenga_curve_permute_rows(plan, buf, buf, bad)
            assert err.value.status == -2
    finally:
        jb.jenga_plan_destroy(plan)
