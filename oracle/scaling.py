"""Oracle: SLO-aware resource scaling (Sec. 3.5 "Fine-Grained Scaling under SLOs": the
layer-wise latency model of Eq. 1a-1c, the steady-state batch of Eq. 2 (Little's law), the
problem of Eq. 3 and the enumeration of Alg. 2).  Control plane of the method.

Readings where the section is silent:
  * all L layers share one set of coefficients (the paper's are per layer; a sum of L equal terms);
  * the communication term is a profiled cost model the paper does not print: linear in the
    batch, comm0 + comm1 * B per layer;
  * attention memory M_a(b, S_ctx) = mem_fixed + mem_per_token * b * S_ctx;
  * a_max(n_e, B) comes from a table on a grid of n_e and B (the Monte-Carlo estimate);
    linear interpolation in B between grid points, clamped at the ends; an n_e that is not on the
    grid is not a candidate;
  * B* is real-valued; the residual f(B) = B - lambda * TPOT(B) is bisected 60 times on
    [1, B_max] after the two boundary cases the section names;
  * ties in n_a + n_e keep the first candidate in the enumeration order of Alg. 2 (n_a outer,
    n_e inner, both ascending).

Test infrastructure only.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np


@dataclass
class Model:
    L: int
    c_a: float
    alpha: float
    c_kv: float
    beta: float
    c_e: float
    comm0: float
    comm1: float
    S_ctx: float
    mem_budget: float
    mem_fixed: float
    mem_per_token: float


def a_max_lookup(table: np.ndarray, ne_values: Sequence[int], B_values: Sequence[float], n_e: int, B: float
                 ) -> Optional[float]:
    if n_e not in list(ne_values):
        return None
    row = np.asarray(table, dtype=np.float64)[list(ne_values).index(n_e)]
    Bs = [float(x) for x in B_values]
    if B <= Bs[0]:
        return float(row[0])
    if B >= Bs[-1]:
        return float(row[-1])
    for i in range(len(Bs) - 1):
        if Bs[i] <= B <= Bs[i + 1]:
            t = (B - Bs[i]) / (Bs[i + 1] - Bs[i])
            return float(row[i] + t * (row[i + 1] - row[i]))
    raise AssertionError


def tpot(m: Model, a_max: float, B: float, n_a: int) -> float:
    """Eq. 1a-1c for one batch size and one configuration (seconds or any one time unit)."""
    b = B / n_a
    t_attn = max(m.c_a, m.alpha * b + m.c_kv * b * m.S_ctx)
    t_moe = m.beta * a_max + m.c_e
    t_comm = m.comm0 + m.comm1 * B
    return m.L * (t_attn + t_moe + t_comm)


def steady_batch(m: Model, table, ne_values, B_values, lam: float, n_a: int, n_e: int, B_max: float
                 ) -> Optional[float]:
    """Eq. 2: B* = lambda * TPOT(B*), or None when even B_max cannot sustain the demand."""
    def f(B):
        return B - lam * tpot(m, a_max_lookup(table, ne_values, B_values, n_e, B), B, n_a)
    if f(1.0) >= 0.0:
        return 1.0
    if f(B_max) < 0.0:
        return None
    lo, hi = 1.0, float(B_max)
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if f(mid) < 0.0:
            lo = mid
        else:
            hi = mid
    return hi


def solve(m: Model, table, ne_values, B_values, lam: float, slo: float, n_max: int, ne_min: int, B_max: float
          ) -> Optional[Tuple[int, int, float, float]]:
    """Alg. 2.  Returns (n_a, n_e, B*, TPOT) of the feasible configuration with the fewest GPUs."""
    opt, best = None, None
    for n_a in range(1, n_max + 1):
        for n_e in range(ne_min, n_max + 1):
            if n_e not in list(ne_values):
                continue
            Bs = steady_batch(m, table, ne_values, B_values, lam, n_a, n_e, B_max)
            if Bs is None:
                continue
            T = tpot(m, a_max_lookup(table, ne_values, B_values, n_e, Bs), Bs, n_a)
            if T > slo:
                continue
            if m.mem_fixed + m.mem_per_token * (Bs / n_a) * m.S_ctx > m.mem_budget:
                continue
            if best is None or n_a + n_e < best:
                opt, best = (n_a, n_e, Bs, T), n_a + n_e
    return opt
