"""ctypes binding of libjenga.so: the same names as the C ABI, argument marshalling only.

Every step of the path runs in the library's HIP kernels.  If the library has not been built the
import of this module fails: there is no fallback.
"""
import ctypes
import os

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libjenga.so")

JENGA_FLAG_ADJACENCY = 1
JENGA_FLAG_CONDITION = 2
JENGA_FLAG_CURVE = 4
JENGA_FLAG_PACED_WALK = 8

EXPORTS = ["jenga_plan_create", "jenga_plan_destroy", "jenga_plan_info", "jenga_plan_export", "jenga_plan_tables",
           "jenga_curve_permute", "jenga_curve_permute_rows", "jenga_select_blocks", "jenga_select_blocks_static",
           "jenga_block_sparse_attn", "jenga_pack_kv",
           "jenga_block_sparse_attn_packed", "jenga_unpermute", "jenga_stage_switch", "jenga_strerror"]


class jenga_config(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("n_text", ctypes.c_int32), ("batch", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("block", ctypes.c_int32),
                ("topk_ratio", ctypes.c_double), ("cum_prob", ctypes.c_double),
                ("text_bias", ctypes.c_float), ("flags", ctypes.c_uint32)]


class jenga_plan_info_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("N_v", "M_v", "M_c", "M", "N_pad", "pad_v", "pad_c", "K_top")] + \
               [("select_workspace_bytes", ctypes.c_uint64), ("attn_workspace_bytes", ctypes.c_uint64)]


class JengaError(RuntimeError):
    def __init__(self, status, what):
        super().__init__("%s: %s (%d)" % (what, _lib.jenga_strerror(status).decode(), status))
        self.status = status


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libjenga.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "or `python paper_2505_16864_amd/build.py` (needs hipcc)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
    lib.jenga_plan_create.argtypes = [ctypes.POINTER(jenga_config), ctypes.POINTER(vp)]
    lib.jenga_plan_destroy.argtypes = [vp]
    lib.jenga_plan_info.argtypes = [vp, ctypes.POINTER(jenga_plan_info_t)]
    lib.jenga_plan_export.argtypes = [vp, vp, vp, vp]
    lib.jenga_plan_tables.argtypes = [ctypes.POINTER(jenga_config), ctypes.POINTER(jenga_plan_info_t), vp, vp, vp]
    lib.jenga_curve_permute.argtypes = [vp, vp, vp, vp]
    lib.jenga_unpermute.argtypes = [vp, vp, vp, vp]
    lib.jenga_curve_permute_rows.argtypes = [vp, vp, vp, ctypes.c_int32, vp]
    lib.jenga_select_blocks.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.jenga_select_blocks_static.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.jenga_block_sparse_attn.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.jenga_pack_kv.argtypes = [vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.jenga_block_sparse_attn_packed.argtypes = [vp, vp, vp, ctypes.c_size_t, vp, vp, vp, vp, vp]
    lib.jenga_stage_switch.argtypes = [vp, vp, vp, vp] + [ctypes.c_int32] * 7 + [ctypes.c_float, vp]
    lib.jenga_strerror.argtypes = [ctypes.c_int]
    lib.jenga_strerror.restype = ctypes.c_char_p
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()


def _check(status, what):
    if status != 0:
        raise JengaError(status, what)


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / None / int."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def make_config(T, H, W, n_text, batch, heads, head_dim, block, topk, p, text_bias=0.0, flags=7):
    return jenga_config(T, H, W, n_text, batch, heads, head_dim, block, float(topk), float(p),
                        float(text_bias), flags)


def jenga_plan_create(cfg):
    plan = ctypes.c_void_p()
    _check(_lib.jenga_plan_create(ctypes.byref(cfg), ctypes.byref(plan)), "jenga_plan_create")
    return plan


def jenga_plan_destroy(plan):
    _check(_lib.jenga_plan_destroy(plan), "jenga_plan_destroy")


def jenga_plan_info(plan):
    info = jenga_plan_info_t()
    _check(_lib.jenga_plan_info(plan, ctypes.byref(info)), "jenga_plan_info")
    return info


def jenga_plan_export(plan, perm=None, inv_perm=None, adja=None):
    """perm, inv_perm: int32 numpy arrays [N_v]; adja: uint8 numpy array [M_v*M_v] (host)."""
    _check(_lib.jenga_plan_export(plan, _ptr(perm), _ptr(inv_perm), _ptr(adja)), "jenga_plan_export")


def jenga_plan_tables(cfg, perm=None, inv_perm=None, adja=None):
    """Host-only tables of a config (no device): returns the info struct, fills the given host arrays."""
    info = jenga_plan_info_t()
    _check(_lib.jenga_plan_tables(ctypes.byref(cfg), ctypes.byref(info), _ptr(perm), _ptr(inv_perm), _ptr(adja)),
           "jenga_plan_tables")
    return info


def jenga_curve_permute(plan, src_thw, dst_curve, stream=None):
    _check(_lib.jenga_curve_permute(plan, _ptr(src_thw), _ptr(dst_curve), stream), "jenga_curve_permute")


def jenga_curve_permute_rows(plan, src_rows, dst_rows, row_bytes, stream=None):
    _check(_lib.jenga_curve_permute_rows(plan, _ptr(src_rows), _ptr(dst_rows), row_bytes, stream),
           "jenga_curve_permute_rows")


def jenga_unpermute(plan, src_curve, dst_thw, stream=None):
    _check(_lib.jenga_unpermute(plan, _ptr(src_curve), _ptr(dst_thw), stream), "jenga_unpermute")


def jenga_select_blocks(plan, q_curve, k_curve, sel_count, sel_index, mask, workspace, workspace_bytes,
                        stream=None):
    _check(_lib.jenga_select_blocks(plan, _ptr(q_curve), _ptr(k_curve), _ptr(sel_count), _ptr(sel_index),
                                    _ptr(mask), _ptr(workspace), workspace_bytes, stream), "jenga_select_blocks")


def jenga_select_blocks_static(plan, q_curve, k_curve, sel_count, sel_index, mask, stream=None):
    _check(_lib.jenga_select_blocks_static(plan, _ptr(q_curve), _ptr(k_curve), _ptr(sel_count), _ptr(sel_index),
                                           _ptr(mask), stream), "jenga_select_blocks_static")


def jenga_block_sparse_attn(plan, q, k, v, sel_count, sel_index, out_curve, lse, workspace, workspace_bytes,
                            stream=None):
    """lse: float32 device tensor [batch, heads, N_pad] or None."""
    _check(_lib.jenga_block_sparse_attn(plan, _ptr(q), _ptr(k), _ptr(v), _ptr(sel_count), _ptr(sel_index),
                                        _ptr(out_curve), _ptr(lse), _ptr(workspace), workspace_bytes, stream),
           "jenga_block_sparse_attn")


def jenga_pack_kv(plan, k, v, workspace, workspace_bytes, stream=None):
    _check(_lib.jenga_pack_kv(plan, _ptr(k), _ptr(v), _ptr(workspace), workspace_bytes, stream), "jenga_pack_kv")


def jenga_block_sparse_attn_packed(plan, q, workspace, workspace_bytes, sel_count, sel_index, out_curve, lse=None,
                                   stream=None):
    _check(_lib.jenga_block_sparse_attn_packed(plan, _ptr(q), _ptr(workspace), workspace_bytes, _ptr(sel_count),
                                               _ptr(sel_index), _ptr(out_curve), _ptr(lse), stream),
           "jenga_block_sparse_attn_packed")


def jenga_stage_switch(x_t, eps_t, eps_tilde, x_out, channels, in_shape, out_shape, sigma_t, stream=None):
    """in_shape = (T_in, H_in, W_in), out_shape = (T_out, H_out, W_out); float32 device tensors."""
    _check(_lib.jenga_stage_switch(_ptr(x_t), _ptr(eps_t), _ptr(eps_tilde), _ptr(x_out), channels,
                                   *[int(v) for v in in_shape], *[int(v) for v in out_shape], float(sigma_t), stream),
           "jenga_stage_switch")


def raw():
    """The ctypes library object, for tests of the error paths."""
    return _lib
