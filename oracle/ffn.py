"""Oracle: the expert FFN over activated experts (Sec. 2.2, "Performance bottleneck of
MoE layers": each expert is two GEMMs, gate/up fused as one and down; the activation
between them is SiLU(gate) * up, fixed by the workload list, not by the paper).

``grouped_ffn`` is the definition applied per non-empty slot with a library matmul;
``dense_layer`` is an independent per-token, per-choice statement of the whole layer
that knows nothing of replicas, slots or permutations.

fp64 throughout, no intermediate rounding.  Test infrastructure only.
"""
from __future__ import annotations

import numpy as np


def silu(h: np.ndarray) -> np.ndarray:
    return h / (1.0 + np.exp(-h))


def expert_ffn(x: np.ndarray, w13: np.ndarray, w2: np.ndarray) -> np.ndarray:
    """x [m,d_h]; w13 [2*d_e,d_h] (gate rows first, then up rows); w2 [d_h,d_e] -> [m,d_h]."""
    d_e = w13.shape[0] // 2
    x = x.astype(np.float64)
    h = x @ w13[:d_e].astype(np.float64).T
    u = x @ w13[d_e:].astype(np.float64).T
    a = silu(h) * u
    return a @ w2.astype(np.float64).T


def grouped_ffn(X: np.ndarray, W13: np.ndarray, W2: np.ndarray, slot_off: np.ndarray,
                perm: np.ndarray, k: int) -> np.ndarray:
    """X [T,d_h]; W13 [C,2*d_e,d_h]; W2 [C,d_h,d_e] (physical slots of this instance).
    Row r of the result is FFN_slot(x_token) for request perm[r] (token = perm[r] // k).
    Slots with no request are not touched."""
    n_local = int(slot_off[-1])
    Yp = np.zeros((n_local, X.shape[1]), dtype=np.float64)
    for s in range(len(slot_off) - 1):
        lo, hi = int(slot_off[s]), int(slot_off[s + 1])
        if hi == lo:
            continue
        tok = np.asarray(perm[lo:hi]) // k
        Yp[lo:hi] = expert_ffn(X[tok], W13[s], W2[s])
    return Yp


def dense_layer(X: np.ndarray, ids: np.ndarray, w: np.ndarray, weights_of) -> np.ndarray:
    """Y[i] = sum_j w[i,j] * FFN_{ids[i,j]}(x_i), one token and one choice at a time with
    the *logical* expert's weights (``weights_of(e) -> (w13, w2)``)."""
    T, k = ids.shape
    Y = np.zeros((T, X.shape[1]), dtype=np.float64)
    for i in range(T):
        x = X[i].astype(np.float64)
        for j in range(k):
            w13, w2 = weights_of(int(ids[i, j]))
            d_e = w13.shape[0] // 2
            y = np.zeros(X.shape[1], dtype=np.float64)
            for c in range(d_e):
                h = float(np.dot(w13[c].astype(np.float64), x))
                u = float(np.dot(w13[d_e + c].astype(np.float64), x))
                a = h / (1.0 + np.exp(-h)) * u
                y += a * w2[:, c].astype(np.float64)
            Y[i] += float(w[i, j]) * y
    return Y


def add_shared_expert(Y_routed: np.ndarray, X: np.ndarray, w13_shared: np.ndarray, w2_shared: np.ndarray) -> np.ndarray:
    """Layer output with a shared expert (an expert every token visits with weight 1; Sec. 4
    notes that the paper itself runs it on the attention side): Y[i] = Y_routed[i] + FFN_shared(x_i)."""
    return np.asarray(Y_routed, dtype=np.float64) + expert_ffn(np.asarray(X), w13_shared, w2_shared)
