"""Oracle: exact optimum of the scheduling problem Alg. 1 approximates (Sec. 3.4:
map activation requests to replicas so that the maximum number of activated
experts on any instance is minimal).

Sending two requests for the same expert to two different replicas activates the
expert twice and can only raise a count, so an optimal schedule seats every
activated expert on exactly one of its hosts: a restricted-assignment problem with
unit jobs.  Two independent solvers:

  * ``optimum_brute``  enumerates every host choice (tiny inputs only);
  * ``optimum_matching`` tries caps M = lower bound, lower bound + 1, ... and tests each
    by growing a capacitated bipartite matching with augmenting paths.

Test infrastructure only; used to grade schedule quality, never for parity of the
schedule itself (Alg. 1 is a heuristic and need not reach the optimum).
"""
from __future__ import annotations

import itertools
from typing import List, Sequence

import numpy as np

from .scheduling import Placement


def _split(activated: Sequence[int], pl: Placement):
    base = np.zeros(pl.n_inst, dtype=np.int64)
    multi: List[int] = []
    for e in activated:
        if pl.R[e] == 1:
            base[pl.hosts[e][0]] += 1
        else:
            multi.append(e)
    return base, multi


def optimum_brute(activated: Sequence[int], pl: Placement, limit: int = 2_000_000) -> int:
    base, multi = _split(sorted(set(int(e) for e in activated)), pl)
    n_comb = 1
    for e in multi:
        n_comb *= len(pl.hosts[e])
        if n_comb > limit:
            raise ValueError("too many combinations for exhaustive search")
    best = None
    for choice in itertools.product(*[pl.hosts[e] for e in multi]):
        load = base.copy()
        for g in choice:
            load[g] += 1
        m = int(load.max()) if len(load) else 0
        if best is None or m < best:
            best = m
    return int(best)


def _feasible(cap: np.ndarray, multi: List[int], pl: Placement) -> bool:
    """Can every expert in ``multi`` be matched to one of its hosts with at most cap[g]
    experts on instance g?  Augmenting-path matching with capacities."""
    if (cap < 0).any():
        return False
    seated: List[List[int]] = [[] for _ in range(pl.n_inst)]   # experts per instance

    def try_seat(e: int, seen: set) -> bool:
        for g in pl.hosts[e]:
            if g in seen:
                continue
            seen.add(g)
            if len(seated[g]) < cap[g]:
                seated[g].append(e)
                return True
            for idx, other in enumerate(seated[g]):
                if try_seat(other, seen):
                    seated[g][idx] = e
                    return True
        return False

    for e in multi:
        if not try_seat(e, set()):
            return False
    return True


def optimum_matching(activated: Sequence[int], pl: Placement) -> int:
    act = sorted(set(int(e) for e in activated))
    base, multi = _split(act, pl)
    lo = max(int(base.max()) if len(act) else 0, -(-len(act) // pl.n_inst))
    M = lo
    while True:
        if _feasible(M - base, multi, pl):
            return M
        M += 1
