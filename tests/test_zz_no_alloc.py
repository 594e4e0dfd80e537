"""The allocation-free selection entry point against jenga_select_blocks: same counts, lists and masks, bit
for bit, on two calls in a row that share the library's static scratch, the second with a smaller input."""
import numpy as np
import pytest
import torch

import jenga_inputs as ji
import paper_2505_16864_amd as J
from paper_2505_16864_amd.layer import CarveLayer

pytestmark = pytest.mark.gpu

BIG = dict(T=9, H=20, W=28, n_text=300, batch=2, heads=5, head_dim=128, block=32, topk=0.2, p=0.4)    # M = 168
SMALL = dict(T=3, H=5, W=7, n_text=40, batch=1, heads=3, head_dim=64, block=32, topk=0.3, p=0.3)      # M = 6


def _both(w, seed):
    print("no-alloc case", w, "seed", seed, flush=True)
    q, k, v = ji.make_qkv(w, seed, device="cuda:0")
    layer = CarveLayer(w, "cuda:0", want_mask=True)
    assert layer.info.select_workspace_bytes <= 64 << 20
    layer.permute_in(q, k, v)
    layer.select()
    torch.cuda.synchronize()
    want = (layer.sel_count.clone(), layer.sel_index.clone(), layer.mask.clone())
    layer.sel_count.fill_(-7)
    layer.sel_index.fill_(-1)
    layer.mask.fill_(9)
    J.jenga_select_blocks_static(layer.plan, layer.q_c, layer.k_c, layer.sel_count, layer.sel_index, layer.mask,
                                 torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(layer.sel_count, want[0])
    assert torch.equal(layer.mask, want[2])
    cnt = want[0].cpu().numpy()
    got_idx, want_idx = layer.sel_index.cpu().numpy(), want[1].cpu().numpy()
    for b, h, i in np.ndindex(cnt.shape):
        assert np.array_equal(got_idx[b, h, i, :cnt[b, h, i]], want_idx[b, h, i, :cnt[b, h, i]])
    assert cnt.min() >= 1
    return layer


def test_static_scratch_two_calls_second_smaller():
    big = _both(BIG, 41)
    small = _both(SMALL, 42)          # the scratch still holds the bigger call's scores
    again = _both(BIG, 43)
    del big, small, again


def test_static_scratch_rejects_what_does_not_fit():
    w = ji.WORKLOADS["hy720p"]
    layer = CarveLayer(w, "cuda:0")
    assert layer.info.select_workspace_bytes > 64 << 20
    with pytest.raises(J.JengaError) as e:
        J.jenga_select_blocks_static(layer.plan, layer.q_c, layer.k_c, layer.sel_count, layer.sel_index, None)
    assert e.value.status == -3
    assert J.raw().jenga_select_blocks_static(None, None, None, None, None, None, None) == -1
