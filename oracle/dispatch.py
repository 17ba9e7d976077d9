"""Oracle: this instance's share of Step 4 (Sec. 3.4 workflow: each instance processes
the activation requests whose replica it hosts) and the weighted top-k combine whose
per-instance partial result enters the reverse-path all-reduce (Sec. 3.3, last
paragraph).

Readings: a request is the pair p = i*k + j; requests inside one slot's segment are
kept in ascending p (a stable grouping), so the index output is unique.

Test infrastructure only.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def permute(O: np.ndarray, g_self: int, C: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """O [T,k] replica ids -> (slot_count [C], slot_off [C+1], perm [n_local]).

    perm lists the pair ids p = i*k + j routed to instance g_self, grouped by local
    slot (rid - g_self*C), ascending p inside a group; slot_off is the exclusive scan
    of slot_count."""
    O = np.asarray(O)
    flat = O.reshape(-1)
    slot_count = np.zeros(C, dtype=np.int32)
    buckets = [[] for _ in range(C)]
    for p in range(flat.shape[0]):
        rid = int(flat[p])
        if rid // C == g_self:
            s = rid - g_self * C
            buckets[s].append(p)
            slot_count[s] += 1
    slot_off = np.zeros(C + 1, dtype=np.int32)
    for s in range(C):
        slot_off[s + 1] = slot_off[s] + slot_count[s]
    perm = np.array([p for b in buckets for p in b], dtype=np.int32)
    return slot_count, slot_off, perm


def combine(Yp: np.ndarray, perm: np.ndarray, w: np.ndarray, T: int, k: int) -> np.ndarray:
    """Y[i,:] = sum over this instance's requests (i,j) of w[i,j] * Yp[pos(i,j),:], the
    sum taken in ascending j; tokens with no local request get zeros.  float64."""
    d_h = Yp.shape[1]
    Y = np.zeros((T, d_h), dtype=np.float64)
    pos_of = {int(p): r for r, p in enumerate(perm)}
    for i in range(T):
        for j in range(k):
            r = pos_of.get(i * k + j)
            if r is not None:
                Y[i] += float(w[i, j]) * Yp[r].astype(np.float64)
    return Y
