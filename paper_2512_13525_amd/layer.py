"""Buffer plumbing for one MoE-instance layer step: allocates the device buffers the C ABI
asks the caller to own and queues route -> schedule -> permute -> grouped FFN -> combine on
one stream.  No arithmetic happens here."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B
from .workloads import MoEConfig, bf16_bits


def to_device_bf16(x_f32: np.ndarray, device="cuda") -> torch.Tensor:
    """float32 array holding bf16-representable values -> bf16 tensor on the device."""
    bits = torch.from_numpy(bf16_bits(x_f32).view(np.int16))
    return bits.view(torch.bfloat16).to(device)


class LayerStep:
    """Device buffers for one (config, g_self) and the calls of one layer step."""

    def __init__(self, cfg: MoEConfig, slot_to_expert, g_self: int, device="cuda"):
        self.cfg, self.g_self, self.dev = cfg, g_self, device
        self.pl = B.Placement(slot_to_expert, cfg.E, cfg.n_inst, cfg.C)
        T, k, C = cfg.T, cfg.k, cfg.C
        i32 = dict(dtype=torch.int32, device=device)
        self.dtype = B.MOE_DTYPE_BF16 if cfg.dtype == "bf16" else B.MOE_DTYPE_F32
        self.tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.topk_ids = torch.empty((T, k), **i32)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, device=device)
        self.rid = torch.empty((T, k), **i32)
        self.act_rep = torch.empty((cfg.E,), **i32)
        self.load = torch.empty((cfg.n_inst,), **i32)
        self.slot_count = torch.empty((C,), **i32)
        self.slot_off = torch.empty((C + 1,), **i32)
        self.perm = torch.empty((T * k,), **i32)
        self.pos = torch.empty((T * k,), **i32)
        self.blocks = torch.empty((B.moe_block_list_len(T, k, C),), **i32)
        self.Yp = torch.empty((T * k, cfg.d_h), dtype=torch.float32, device=device)
        self.Y = torch.empty((T, cfg.d_h), dtype=self.tdtype, device=device)
        ws = B.moe_workspace_bytes(T, k, C, cfg.d_h, cfg.d_e, self.dtype)
        self.workspace = torch.empty((ws,), dtype=torch.uint8, device=device)
        B.moe_workspace_init(self.workspace)
        self.sync = torch.zeros((B.moe_front_sync_len(self.pl, T, k),), **i32)
        self.gate_sync = torch.zeros((B.moe_gate_sync_len(T),), **i32)
        self.gate_logits = torch.empty((T, cfg.E), dtype=torch.float32, device=device)
        self.W13 = None
        self.W2 = None

    # -- weights -------------------------------------------------------------------------
    def set_weights(self, W13_canonical: torch.Tensor, W2_canonical: torch.Tensor):
        """Canonical [C,2*d_e,d_h] / [C,d_h,d_e] device tensors; bf16 weights are packed once."""
        cfg = self.cfg
        if self.dtype == B.MOE_DTYPE_BF16:
            self.W13 = torch.empty_like(W13_canonical)
            self.W2 = torch.empty_like(W2_canonical)
            B.moe_pack_weights_bf16(W13_canonical, W2_canonical, cfg.C, cfg.d_h, cfg.d_e, self.W13, self.W2)
        else:
            self.W13, self.W2 = W13_canonical, W2_canonical

    def set_packed_weights(self, W13, W2):
        self.W13, self.W2 = W13, W2

    # -- steps ---------------------------------------------------------------------------
    def route(self, logits, stream=None):
        c = self.cfg
        if c.route == "softmax":
            B.moe_route(logits, c.k, self.topk_ids, self.topk_w, B.MOE_ROUTE_SOFTMAX, True, stream=stream)
        else:
            B.moe_route(logits, c.k, self.topk_ids, self.topk_w, B.MOE_ROUTE_SIGMOID_GROUP, True,
                        c.n_group, c.topk_group, 1.0, stream=stream)

    def schedule(self, stream=None):
        c = self.cfg
        B.moe_schedule(self.pl, self.topk_ids, c.T, c.k, self.rid, self.act_rep, self.load, stream=stream)

    def permute(self, stream=None):
        c = self.cfg
        B.moe_permute(self.pl, self.g_self, self.rid, c.T, c.k, self.slot_count, self.slot_off,
                      self.perm, self.pos, self.blocks, stream=stream)

    def front(self, logits, stream=None):
        """route + schedule + permute in one launch."""
        c = self.cfg
        group = c.route != "softmax"
        B.moe_route_schedule_permute(self.pl, self.g_self, logits, c.k, self.topk_ids, self.topk_w, self.rid,
                                     self.act_rep, self.load, self.slot_count, self.slot_off, self.perm, self.pos,
                                     self.blocks, self.sync, B.MOE_ROUTE_SIGMOID_GROUP if group else B.MOE_ROUTE_SOFTMAX, True,
                                     c.n_group if group else 1, c.topk_group if group else 1, 1.0, stream=stream)

    def front_gate(self, X, Wr, bias=None, stream=None):
        """gate (X * Wr^T + bias) + route + schedule + permute in one launch; returns the logits."""
        c = self.cfg
        group = c.route != "softmax"
        B.moe_gate_route_schedule_permute(self.pl, self.g_self, X, Wr, bias, c.k, self.gate_logits, self.topk_ids,
                                          self.topk_w, self.rid, self.act_rep, self.load, self.slot_count,
                                          self.slot_off, self.perm, self.pos, self.blocks, self.gate_sync,
                                          B.MOE_ROUTE_SIGMOID_GROUP if group else B.MOE_ROUTE_SOFTMAX, True,
                                          c.n_group if group else 1, c.topk_group if group else 1, 1.0, stream=stream)
        return self.gate_logits

    def ffn(self, X, stream=None, W13=None, W2=None):
        c = self.cfg
        B.moe_grouped_ffn(X, self.W13 if W13 is None else W13, self.W2 if W2 is None else W2,
                          c.T, c.k, c.C, c.d_h, c.d_e, self.dtype, self.slot_off, self.perm, self.blocks,
                          self.Yp, self.workspace, stream=stream)

    def combine(self, stream=None):
        c = self.cfg
        B.moe_combine(self.Yp, self.pos, self.topk_w, c.T, c.k, c.d_h, self.dtype, self.Y, stream=stream)

    def step(self, logits, X, stream=None, W13=None, W2=None):
        """The layer step through the four separate entry points (five launches)."""
        self.route(logits, stream)
        self.schedule(stream)
        self.permute(stream)
        self.ffn(X, stream, W13, W2)
        self.combine(stream)
        return self.Y

    def step_fused(self, logits, X, stream=None, W13=None, W2=None):
        """The same step in three launches: front (a0-a4), FFN, combine."""
        self.front(logits, stream)
        self.ffn(X, stream, W13, W2)
        self.combine(stream)
        return self.Y

    # -- shared expert (option) ----------------------------------------------------------
    def enable_shared(self, W13_shared: torch.Tensor, W2_shared: torch.Tensor):
        """Canonical [2*d_s, d_h] / [d_h, d_s] device tensors of a shared expert: one more slot
        that every token visits, run by the same FFN kernel through a dispatch of its own."""
        c = self.cfg
        d_s = W2_shared.shape[1]
        i32 = dict(dtype=torch.int32, device=self.dev)
        self.d_s = d_s
        self.s_slot_off = torch.empty((2,), **i32)
        self.s_perm = torch.empty((max(c.T, 1),), **i32)
        self.s_blocks = torch.empty((B.moe_block_list_len(c.T, 1, 1),), **i32)
        self.s_Yp = torch.empty((c.T, c.d_h), dtype=torch.float32, device=self.dev)
        ws = B.moe_workspace_bytes(c.T, 1, 1, c.d_h, d_s, self.dtype)
        self.s_workspace = torch.empty((ws,), dtype=torch.uint8, device=self.dev)
        B.moe_workspace_init(self.s_workspace)
        w13, w2 = W13_shared.reshape(1, 2 * d_s, c.d_h), W2_shared.reshape(1, c.d_h, d_s)
        if self.dtype == B.MOE_DTYPE_BF16:
            self.s_W13, self.s_W2 = torch.empty_like(w13), torch.empty_like(w2)
            B.moe_pack_weights_bf16(w13, w2, 1, c.d_h, d_s, self.s_W13, self.s_W2)
        else:
            self.s_W13, self.s_W2 = w13.contiguous(), w2.contiguous()
        B.moe_shared_dispatch(c.T, self.s_slot_off, self.s_perm, self.s_blocks)

    def step_fused_shared(self, logits, X, stream=None, W13=None, W2=None):
        """front, routed FFN, shared-expert FFN, combine of both (four launches)."""
        c = self.cfg
        self.front(logits, stream)
        self.ffn(X, stream, W13, W2)
        B.moe_grouped_ffn(X, self.s_W13, self.s_W2, c.T, 1, 1, c.d_h, self.d_s, self.dtype, self.s_slot_off,
                          self.s_perm, self.s_blocks, self.s_Yp, self.s_workspace, stream=stream)
        B.moe_combine_shared(self.Yp, self.pos, self.topk_w, self.s_Yp, c.T, c.k, c.d_h, self.dtype, self.Y, stream=stream)
        return self.Y
