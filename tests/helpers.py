"""Shared plumbing of the GPU parity tests: run the oracle and the HIP path on the same
seeded inputs.  Holds no arithmetic of its own."""
from __future__ import annotations

import numpy as np

from oracle import dispatch, ffn, routing, scheduling
from paper_2512_13525_amd import workloads as W


def oracle_route(cfg, logits):
    if cfg.route == "softmax":
        ids, w = routing.route_softmax(logits, cfg.k)
        return ids, w, None
    ids, w, info = routing.route_sigmoid_group(logits, cfg.k, cfg.n_group, cfg.topk_group)
    return ids, w, info


class OracleRun:
    """Everything the oracle computes for (cfg, g_self) on the seeded inputs."""

    def __init__(self, cfg, g_self=None, with_ffn=True, weights=None, only_activated=False):
        self.cfg = cfg
        self.lay = W.build_placement(cfg)
        self.pl = scheduling.make_placement(self.lay, cfg.E, cfg.n_inst, cfg.C)
        self.logits = W.router_logits(cfg)
        self.X = W.activations(cfg)
        self.ids, self.w, self.route_info = oracle_route(cfg, self.logits)
        self.O, self.act_rep, self.load = scheduling.aebs(self.ids, self.pl)
        if g_self is None:
            g_self = int(np.argmax(self.load))          # the straggler instance sets layer latency
        self.g_self = g_self
        self.slot_count, self.slot_off, self.perm = dispatch.permute(self.O, g_self, cfg.C)
        self.pos = np.full(cfg.T * cfg.k, -1, dtype=np.int32)
        self.pos[self.perm] = np.arange(len(self.perm), dtype=np.int32)
        if with_ffn:
            if weights is None:
                if only_activated:
                    # slots without a request hold NaN: the HIP path must never read them
                    W13 = np.full((cfg.C, 2 * cfg.d_e, cfg.d_h), np.nan, dtype=np.float32)
                    W2 = np.full((cfg.C, cfg.d_h, cfg.d_e), np.nan, dtype=np.float32)
                    for s in np.nonzero(self.slot_count > 0)[0]:
                        W13[s], W2[s] = W.expert_weights(cfg, int(self.lay[g_self * cfg.C + s]))
                    weights = (W13, W2)
                else:
                    weights = W.instance_weights(cfg, self.lay, g_self)
            self.W13, self.W2 = weights
            self.Yp = ffn.grouped_ffn(self.X, self.W13, self.W2, self.slot_off, self.perm, cfg.k)
            self.Y = dispatch.combine(self.Yp, self.perm, self.w, cfg.T, cfg.k)


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def expected_blocks(slot_off, block_rows, heavy_rows=16):
    """The FFN work list that follows from slot_off: every slot's rows cut into blocks of at
    most `block_rows` rows; slots with more than `heavy_rows` requests first, ascending slot
    order within each class; [n_blocks, block_rows, n_wide, n_wide128] then [slot, first row, slot end, slot
    start] per block (flattened int32); n_wide / n_wide128 = number of 64-row / 128-row blocks of the slots
    with more than 64 requests."""
    out = []
    for heavy in (True, False):
        for s in range(len(slot_off) - 1):
            lo, hi = int(slot_off[s]), int(slot_off[s + 1])
            if (hi - lo > heavy_rows) != heavy:
                continue
            for r in range(lo, hi, block_rows):
                out.append([s, r, hi, lo])
    rows = np.diff(np.asarray(slot_off, dtype=np.int64))
    n_wide = int(sum((int(v) + 63) // 64 for v in rows if v > 64))
    n_wide128 = int(sum((int(v) + 127) // 128 for v in rows if v > 64))
    return np.array([[len(out), block_rows, n_wide, n_wide128]] + out, dtype=np.int32).reshape(-1)
