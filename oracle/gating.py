"""Oracle: the router's linear layer on the MoE side (Sec. 3.3 "Gating on the MoE side": the MoE
instance receives the complete activations and runs the gate itself, so the gate's logits are
computed where the experts are; Sec. 3.4 workflow, the step before Step 1).

The gate is the plain linear map logits[i, e] = sum_c X[i, c] * W_r[e, c] (+ bias[e]); the paper
fixes nothing else about it.  The selection that follows (routing.py) is an integer decision
taken on these logits in fp32, the precision the kernel holds them in, so `gate_logits_f32`
rounds the fp64 sums once.  `selection_margin` tells a test how far a token's selection is from
flipping under a perturbation of the logits (summation order on the GPU differs).

Test infrastructure only.
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def gate_logits(X: np.ndarray, Wr: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """fp64 logits [T,E] of activations X [T,d_h] under router weights W_r [E,d_h]."""
    X = np.asarray(X, dtype=np.float64)
    Wr = np.asarray(Wr, dtype=np.float64)
    assert X.ndim == 2 and Wr.ndim == 2 and X.shape[1] == Wr.shape[1]
    z = np.matmul(X, Wr.T)
    if bias is not None:
        bias = np.asarray(bias, dtype=np.float64)
        assert bias.shape == (Wr.shape[0],)
        z = z + bias[None, :]
    return z


def gate_logits_f32(X: np.ndarray, Wr: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """The same logits rounded once to fp32: the values the selection is taken on."""
    return gate_logits(X, Wr, bias).astype(np.float32)


def selection_margin(logits: np.ndarray, k: int) -> np.ndarray:
    """Per token, the smallest gap between neighbours among the k+1 largest logits (fp64).

    If every logit moves by less than half of this, neither the selected set nor the order of
    the k selected experts changes.  With k == E the (k+1)-th value does not exist and only the
    order inside the selection counts."""
    z = -np.sort(-np.asarray(logits, dtype=np.float64), axis=1)
    top = z[:, : min(k + 1, z.shape[1])]
    if top.shape[1] < 2:
        return np.full(z.shape[0], np.inf)
    return (top[:, :-1] - top[:, 1:]).min(axis=1)
