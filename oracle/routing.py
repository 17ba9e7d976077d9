"""Oracle: gating selection on the MoE side (Sec. 3.3 "Gating on the MoE side";
Sec. 3.4 workflow, the step before Step 1: "gating produces the top-k logical
expert ids").  The paper fixes no score function; the two used here are the
softmax top-k of the DeepSeek-V2 / Qwen3 families and the sigmoid,
group-limited top-k of DeepSeek-V3, which the workload list names.

Test infrastructure only.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np


def _topk_desc(values: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries per row, largest first; equal values: lower index first."""
    order = np.argsort(-values, axis=1, kind="stable")
    return order[:, :k]


def route_softmax(logits: np.ndarray, k: int, renormalize: bool = True
                  ) -> Tuple[np.ndarray, np.ndarray]:
    """ids [T,k] int32 (j-th column = j-th largest logit), w [T,k] float64.

    Softmax is monotone, so the selection is taken on the logits themselves (no
    rounding can enter the integer result).  w = softmax over all E experts,
    gathered at ids; with ``renormalize`` the k weights are rescaled to sum to 1.
    """
    logits = np.asarray(logits, dtype=np.float32)
    T, E = logits.shape
    assert 1 <= k <= E
    ids = _topk_desc(logits, k)
    z = logits.astype(np.float64)
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z)
    p /= p.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, ids, axis=1)
    if renormalize:
        w = w / w.sum(axis=1, keepdims=True)
    return ids.astype(np.int32), w


def route_sigmoid_group(logits: np.ndarray, k: int, n_group: int, topk_group: int,
                        scale: float = 1.0) -> Tuple[np.ndarray, np.ndarray, Dict[str, np.ndarray]]:
    """Sigmoid scores with group-limited top-k.

    s = sigmoid(logit).  Experts form n_group contiguous groups; a group's score is the
    sum of its two largest s; the topk_group best groups survive (lower group id on
    ties); the k largest s among surviving experts are selected (lower id on ties);
    w = s / sum(selected s) * scale.

    sigmoid is monotone, so "largest s" is decided on the logits.  Only the group score
    needs sigmoid numerically; that decision is taken in fp32, the precision of the
    kernel, and its fp64 margin (gap between the last kept and the first dropped group
    score) is returned so a caller can tell a genuine decision from a rounding tie.

    Returns ids [T,k] int32, w [T,k] float64, info {"group_margin": [T] float64,
    "kept_groups": [T,topk_group] int64}.
    """
    logits = np.asarray(logits, dtype=np.float32)
    T, E = logits.shape
    assert E % n_group == 0 and 1 <= topk_group <= n_group
    per = E // n_group
    assert per >= 2 and k <= topk_group * per
    lg = logits.reshape(T, n_group, per)
    top2 = -np.sort(-lg, axis=2)[:, :, :2]                       # two largest logits per group
    one = np.float32(1.0)
    s32 = one / (one + np.exp(-top2, dtype=np.float32))           # fp32 sigmoid
    gscore32 = (s32[:, :, 0] + s32[:, :, 1]).astype(np.float32)
    kept = _topk_desc(gscore32, topk_group)                       # [T, topk_group]
    # fp64 margin of the group decision
    s64 = 1.0 / (1.0 + np.exp(-top2.astype(np.float64)))
    g64 = s64.sum(axis=2)
    g_sorted = -np.sort(-g64, axis=1)
    if topk_group < n_group:
        margin = g_sorted[:, topk_group - 1] - g_sorted[:, topk_group]
    else:
        margin = np.full(T, np.inf)
    mask = np.zeros((T, n_group), dtype=bool)
    np.put_along_axis(mask, kept, True, axis=1)
    emask = np.repeat(mask, per, axis=1)
    masked = np.where(emask, logits, -np.inf).astype(np.float32)
    ids = _topk_desc(masked, k)
    s_all = 1.0 / (1.0 + np.exp(-logits.astype(np.float64)))
    w = np.take_along_axis(s_all, ids, axis=1)
    w = w / w.sum(axis=1, keepdims=True) * scale
    return ids.astype(np.int32), w, {"group_margin": margin, "kept_groups": np.sort(kept, axis=1)}
