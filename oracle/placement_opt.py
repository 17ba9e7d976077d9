"""Oracle: activation-aware replica management (Appendix B, "Activation-Aware Replica
Placement": the replica-count rule, the co-activation load of Eq. 6 and the greedy placement of
Alg. 3).  Control plane of the method: it produces the replica layout that Alg. 1 schedules over.

Readings where the appendix is silent:
  * statistics: c(e) = number of batches of the window that activate e; a(e, e') = number of
    batches that activate both (what raises the concurrent activations of an instance is being
    activated in the same batch);
  * an expert never gets more replicas than there are instances (two replicas on one instance
    are useless: Alg. 3 keeps x[e, g] in {0, 1}); the replica-count rule then grants the slot to
    the next best expert;
  * ties: largest c(e)/R(e) -> lower expert id; replica order -> decreasing load, then expert
    id, then copy number; arg min over instances -> lowest instance; arg min over swaps -> lowest
    (g, position of j in P(g), h);
  * the penalty of a swap is the change of the summed co-activation load:
    Delta I(i -> g, j -> h) = sum_{m in P(g)\\{j}} [a(e_i, e_m) - a(e_j, e_m)] + sum_{m in P(h)} a(e_j, e_m).
Sums are fp64 in placement order (the order replicas were put on the instance).

Test infrastructure only.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np


def coactivation_counts(ids: np.ndarray, E: int) -> Tuple[np.ndarray, np.ndarray]:
    """ids [n_batches, B, k] expert ids of a window of batches -> c [E], a [E,E] (fp64 counts;
    a symmetric with zero diagonal)."""
    ids = np.asarray(ids)
    c = np.zeros(E, dtype=np.float64)
    a = np.zeros((E, E), dtype=np.float64)
    for batch in ids:
        act = sorted(set(int(x) for x in batch.reshape(-1)))
        for x in act:
            c[x] += 1.0
        for i, x in enumerate(act):
            for y in act[i + 1:]:
                a[x, y] += 1.0
                a[y, x] += 1.0
    return c, a


def replica_counts(c: np.ndarray, n_inst: int, C: int) -> np.ndarray:
    """One replica each, then the n_inst*C - E spare slots one at a time to the expert with the
    largest load per replica c(e)/R(e) among those with fewer than n_inst replicas."""
    c = np.asarray(c, dtype=np.float64)
    E = len(c)
    S = n_inst * C
    if S < E:
        raise ValueError("fewer slots than experts")
    R = np.ones(E, dtype=np.int64)
    for _ in range(S - E):
        best = -1
        for e in range(E):
            if R[e] >= n_inst:
                continue
            if best < 0 or c[e] / R[e] > c[best] / R[best]:
                best = e
        if best < 0:
            break                      # every expert is on every instance
        R[best] += 1
    return R


def coactivation_load(P_g: List[int], a: np.ndarray) -> float:
    """Eq. 6: I(g) = sum over unordered pairs of experts on the instance of a(e, e')."""
    tot = 0.0
    for i in range(len(P_g)):
        for j in range(i + 1, len(P_g)):
            tot += float(a[P_g[i], P_g[j]])
    return tot


def _penalty(e: int, members: List[int], a: np.ndarray, skip: int = -1) -> float:
    s = 0.0
    for pos, m in enumerate(members):
        if pos != skip:
            s += float(a[e, m])
    return s


def place_replicas(n_inst: int, C: int, R: np.ndarray, c: np.ndarray, a: np.ndarray) -> np.ndarray:
    """Alg. 3.  Returns slot_to_expert [n_inst*C] int32 (-1 = empty), instance g's slots in
    the order its replicas were placed."""
    R = np.asarray(R, dtype=np.int64)
    c = np.asarray(c, dtype=np.float64)
    a = np.asarray(a, dtype=np.float64)
    E = len(R)
    if (R < 1).any() or (R > n_inst).any() or int(R.sum()) > n_inst * C:
        raise ValueError("replica counts do not fit")
    P: List[List[int]] = [[] for _ in range(n_inst)]
    slots = [C] * n_inst
    x = np.zeros((E, n_inst), dtype=bool)
    replicas = [(e, r) for e in range(E) for r in range(int(R[e]))]
    replicas.sort(key=lambda t: (-(c[t[0]] / R[t[0]]), t[0], t[1]))
    for e, _ in replicas:
        feasible = [g for g in range(n_inst) if slots[g] > 0 and not x[e, g]]
        if feasible:
            best_g, best_p = -1, 0.0
            for g in feasible:
                p = _penalty(e, P[g], a)
                if best_g < 0 or p < best_p:
                    best_g, best_p = g, p
            P[best_g].append(e)
            slots[best_g] -= 1
            x[e, best_g] = True
            continue
        best = None
        for g in range(n_inst):
            if x[e, g]:
                continue
            for pos, ej in enumerate(P[g]):
                for h in range(n_inst):
                    if slots[h] <= 0 or x[ej, h] or h == g:
                        continue
                    d = (_penalty(e, P[g], a, skip=pos) - _penalty(ej, P[g], a, skip=pos)) + _penalty(ej, P[h], a)
                    if best is None or d < best[0]:
                        best = (d, g, pos, h)
        if best is None:
            raise ValueError("no feasible swap")
        _, g, pos, h = best
        ej = P[g][pos]
        P[g][pos] = e
        P[h].append(ej)
        slots[h] -= 1
        x[ej, g] = False
        x[ej, h] = True
        x[e, g] = True
    lay = np.full((n_inst, C), -1, dtype=np.int32)
    for g in range(n_inst):
        lay[g, :len(P[g])] = P[g]
    return lay.reshape(-1)
