"""CPU tests of the C-ABI library: it loads, exports every declared symbol, validates arguments,
and its host-side tables (curve, padding, adjacency) equal the oracle's bit for bit."""
import ctypes
import os
import re
import numpy as np
import pytest

import paper_2505_16864_amd as J
from oracle import jenga_oracle as jo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "jenga.h")).read()
    declared = set(re.findall(r"\b(jenga_[a-z_]+)\s*\(", header))
    assert declared == set(J.EXPORTS)
    lib = J.raw()
    for name in declared:
        assert getattr(lib, name) is not None
    assert b"ok" == lib.jenga_strerror(0)
    assert b"workspace" in lib.jenga_strerror(-3)


def test_struct_layout_matches_header():
    assert ctypes.sizeof(J.jenga_config) == 56
    assert J.jenga_config.topk_ratio.offset == 32 and J.jenga_config.flags.offset == 52
    assert ctypes.sizeof(J.jenga_plan_info_t) == 48


GRIDS = [(1, 1, 1), (1, 1, 9), (2, 2, 2), (4, 4, 4), (3, 5, 7), (4, 8, 8), (8, 16, 16), (5, 6, 11), (7, 7, 7),
         (2, 9, 3), (13, 2, 5), (6, 10, 15), (9, 1, 4), (21, 30, 52), (33, 24, 42), (33, 45, 80), (20, 30, 52)]


@pytest.mark.parametrize("g", GRIDS)
def test_host_tables_equal_oracle(g):
    T, H, W = g
    n_text = 40
    for m in (32, 128):
        cfg = J.make_config(T, H, W, n_text, 1, 2, 64, m, 0.3, 0.3)
        lay = jo.Layout(T, H, W, n_text, m, 0.3)
        if lay.M > 2048:        # beyond what the selection kernel is built for: must be refused
            with pytest.raises(J.JengaError) as e:
                J.jenga_plan_tables(cfg)
            assert e.value.status == -2
            continue
        perm = np.zeros(lay.N_v, dtype=np.int32)
        inv = np.zeros(lay.N_v, dtype=np.int32)
        adja = np.zeros(lay.M_v * lay.M_v, dtype=np.uint8)
        info = J.jenga_plan_tables(cfg, perm, inv, adja)
        assert (info.N_v, info.M_v, info.M_c, info.M, info.N_pad, info.pad_v, info.pad_c, info.K_top) == \
               (lay.N_v, lay.M_v, lay.M_c, lay.M, lay.N_pad, lay.pad_v, lay.pad_c, lay.K_top)
        assert np.array_equal(perm, lay.perm)
        assert np.array_equal(inv, lay.inv)
        assert np.array_equal(adja.reshape(lay.M_v, lay.M_v).astype(bool), jo.adjacency_mask(lay))


def test_many_small_grids_equal_oracle():
    import itertools
    for T, H, W in itertools.product(range(1, 7), repeat=3):
        cfg = J.make_config(T, H, W, 0, 1, 1, 64, 32, 0.5, 0.0)
        lay = jo.Layout(T, H, W, 0, 32, 0.5)
        perm = np.zeros(lay.N_v, dtype=np.int32)
        J.jenga_plan_tables(cfg, perm)
        assert np.array_equal(perm, lay.perm), (T, H, W)


def test_flags_linear_order_and_no_adjacency():
    cfg = J.make_config(3, 5, 7, 0, 1, 1, 64, 32, 0.5, 0.0, flags=J.JENGA_FLAG_CONDITION)
    perm = np.zeros(105, dtype=np.int32)
    adja = np.ones(16, dtype=np.uint8)
    J.jenga_plan_tables(cfg, perm, None, adja)
    assert np.array_equal(perm, np.arange(105)) and not adja.any()


def test_k_top_and_workspace_sizes():
    info = J.jenga_plan_tables(J.make_config(33, 24, 42, 256, 1, 24, 128, 128, 0.3, 0.3))
    assert info.K_top == 78 and info.M == 262
    info = J.jenga_plan_tables(J.make_config(33, 45, 80, 256, 1, 24, 128, 128, 0.3, 0.3))
    assert (info.M_v, info.pad_v, info.M, info.N_pad, info.K_top) == (929, 112, 931, 119168, 278)
    assert info.attn_workspace_bytes == 2 * 24 * 119168 * 128 * 2 + 256
    assert info.select_workspace_bytes >= 24 * (929 + 931) * 128 * 8 + 24 * 929 * 931 * 8


@pytest.mark.parametrize("bad,status", [
    (dict(T=0), -1), (dict(n_text=-1), -1), (dict(batch=0), -1), (dict(heads=0), -1),
    (dict(topk=0.0), -1), (dict(topk=1.5), -1), (dict(p=1.0), -1), (dict(p=-0.1), -1), (dict(flags=16), -1),
    (dict(text_bias=float("nan")), -1), (dict(text_bias=float("inf")), -1), (dict(text_bias=float("-inf")), -1),
    # Alg. 2's text-only branch (no vision tokens) is plain dense attention and is not taken by this library
    (dict(T=0, H=0, W=0), -1), (dict(W=0), -1),
    (dict(head_dim=96), -2), (dict(block=16), -2), (dict(block=256), -2), (dict(T=400, H=400, W=400), -2),
])
def test_invalid_configs_are_rejected(bad, status):
    args = dict(T=4, H=8, W=8, n_text=32, batch=1, heads=2, head_dim=64, block=32, topk=0.25, p=0.3,
                text_bias=0.0, flags=7)
    args.update(bad)
    cfg = J.make_config(**args)
    with pytest.raises(J.JengaError) as e:
        J.jenga_plan_tables(cfg)
    assert e.value.status == status
    plan = ctypes.c_void_p()
    assert J.raw().jenga_plan_create(ctypes.byref(cfg), ctypes.byref(plan)) == status
    assert not plan.value


def test_null_arguments_return_einval_without_a_device():
    lib = J.raw()
    assert lib.jenga_plan_create(None, None) == -1
    assert lib.jenga_plan_info(None, None) == -1
    assert lib.jenga_plan_export(None, None, None, None) == -1
    assert lib.jenga_curve_permute(None, None, None, None) == -1
    assert lib.jenga_unpermute(None, None, None, None) == -1
    assert lib.jenga_curve_permute_rows(None, None, None, 512, None) == -1
    assert lib.jenga_select_blocks(None, None, None, None, None, None, None, 0, None) == -1
    assert lib.jenga_block_sparse_attn(None, None, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.jenga_pack_kv(None, None, None, None, 0, None) == -1
    assert lib.jenga_block_sparse_attn_packed(None, None, None, 0, None, None, None, None, None) == -1
    assert lib.jenga_stage_switch(None, None, None, None, 1, 1, 1, 1, 1, 1, 1, 0.5, None) == -1
    assert lib.jenga_plan_destroy(None) == 0
