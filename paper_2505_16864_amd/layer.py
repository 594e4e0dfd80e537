"""Buffers for one attention layer: torch owns the device memory and the stream, the library does the work."""
import torch

from . import binding as B


class CarveLayer:
    """Allocates the curve-side tensors, index lists and workspaces of one configuration once and
    runs the four calls on torch's current stream."""

    def __init__(self, w, device="cuda:0", text_bias=None, flags=None, want_mask=False, want_lse=False):
        self.w = dict(w)
        if text_bias is None:
            text_bias = w.get("text_bias", 0.0)
        if flags is None:
            flags = w.get("flags", 7)
        self.device = torch.device(device)
        self.cfg = B.make_config(w["T"], w["H"], w["W"], w["n_text"], w["batch"], w["heads"], w["head_dim"],
                                 w["block"], w["topk"], w["p"], text_bias, flags)
        with torch.cuda.device(self.device):
            self.plan = B.jenga_plan_create(self.cfg)
        self.info = B.jenga_plan_info(self.plan)
        i, dev = self.info, self.device
        shape_c = (w["batch"], w["heads"], i.N_pad, w["head_dim"])
        self.q_c, self.k_c, self.v_c, self.o_c = [torch.empty(shape_c, dtype=torch.bfloat16, device=dev)
                                                  for _ in range(4)]
        self.sel_count = torch.empty((w["batch"], w["heads"], i.M), dtype=torch.int32, device=dev)
        self.sel_index = torch.full((w["batch"], w["heads"], i.M, i.M), -1, dtype=torch.int32, device=dev)
        self.mask = torch.zeros((w["batch"], w["heads"], i.M, i.M), dtype=torch.uint8, device=dev) if want_mask else None
        self.lse = torch.empty((w["batch"], w["heads"], i.N_pad), dtype=torch.float32, device=dev) if want_lse else None
        self.ws_select = torch.empty(max(1, i.select_workspace_bytes), dtype=torch.uint8, device=dev)
        self.ws_attn = torch.empty(max(1, i.attn_workspace_bytes), dtype=torch.uint8, device=dev)
        self.out_thw = torch.empty((w["batch"], i.N_v + w["n_text"], w["heads"], w["head_dim"]),
                                   dtype=torch.bfloat16, device=dev)

    def _stream(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    def permute_in(self, q, k, v):
        s = self._stream()
        B.jenga_curve_permute(self.plan, q, self.q_c, s)
        B.jenga_curve_permute(self.plan, k, self.k_c, s)
        B.jenga_curve_permute(self.plan, v, self.v_c, s)

    def select(self):
        B.jenga_select_blocks(self.plan, self.q_c, self.k_c, self.sel_count, self.sel_index, self.mask,
                              self.ws_select, self.ws_select.numel(), self._stream())

    def attend(self):
        B.jenga_block_sparse_attn(self.plan, self.q_c, self.k_c, self.v_c, self.sel_count, self.sel_index,
                                  self.o_c, self.lse, self.ws_attn, self.ws_attn.numel(), self._stream())

    def pack(self):
        B.jenga_pack_kv(self.plan, self.k_c, self.v_c, self.ws_attn, self.ws_attn.numel(), self._stream())

    def attend_packed(self):
        B.jenga_block_sparse_attn_packed(self.plan, self.q_c, self.ws_attn, self.ws_attn.numel(), self.sel_count,
                                         self.sel_index, self.o_c, self.lse, self._stream())

    def permute_out(self):
        B.jenga_unpermute(self.plan, self.o_c, self.out_thw, self._stream())

    def forward(self, q, k, v):
        """Whole path on thw-side bf16 tensors [batch, N_v+N_c, heads, d]; returns the thw-side output."""
        self.permute_in(q, k, v)
        self.select()
        self.attend()
        self.permute_out()
        return self.out_thw

    def close(self):
        if self.plan is not None:
            B.jenga_plan_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
