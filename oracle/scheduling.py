"""Oracle: replica layout tables and Activated-Expert-Balanced Scheduling
(Sec. 3.4, Alg. 1), taken step by step in the paper's notation.

Readings where Alg. 1 is silent:
  * the multi-replica loop visits activated experts in ascending logical id;
  * arg min over G(e) breaks ties towards the lowest instance index;
  * single-replica experts are seated first (the prose after Alg. 1 says so; the
    comment above the first loop in the listing is a misprint);
  * the physical replica id of slot s on instance g is g*C + s;
  * an expert may not have two replicas on one instance (Alg. 3 keeps a bitmap
    x[e,g] for exactly that), and every expert needs at least one replica.

Also the two comparison policies the evaluation describes in words (Sec. 5,
baselines): replicas chosen at random per activation request, and a static
"home replica only" mapping.  They are used for a_max context, never for parity.

Test infrastructure only.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


class PlacementError(ValueError):
    pass


@dataclass
class Placement:
    E: int
    n_inst: int
    C: int
    slot_to_expert: np.ndarray          # [n_inst*C] int, -1 = empty
    R: np.ndarray                       # [E] replica counts
    hosts: List[List[int]]              # G(e): hosting instances, ascending
    rids: List[List[int]]               # P(e,g) aligned with hosts[e]

    def instance_of(self, rid: int) -> int:
        return rid // self.C


def make_placement(slot_to_expert, E: int, n_inst: int, C: int) -> Placement:
    lay = np.asarray(slot_to_expert, dtype=np.int64)
    if E < 1 or n_inst < 1 or C < 1:
        raise PlacementError("non-positive dimension")
    if lay.shape != (n_inst * C,):
        raise PlacementError("slot_to_expert must have n_inst*C entries")
    hosts: List[List[int]] = [[] for _ in range(E)]
    rids: List[List[int]] = [[] for _ in range(E)]
    for g in range(n_inst):
        for s in range(C):
            e = int(lay[g * C + s])
            if e == -1:
                continue
            if e < 0 or e >= E:
                raise PlacementError(f"slot ({g},{s}) names expert {e} outside [0,{E})")
            if hosts[e] and hosts[e][-1] == g:
                raise PlacementError(f"expert {e} has two replicas on instance {g}")
            hosts[e].append(g)
            rids[e].append(g * C + s)
    for e in range(E):
        if not hosts[e]:
            raise PlacementError(f"expert {e} has no replica")
    R = np.array([len(h) for h in hosts], dtype=np.int64)
    return Placement(E, n_inst, C, lay.astype(np.int32), R, hosts, rids)


def aebs(L: np.ndarray, pl: Placement) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Alg. 1.  L [T,k] logical ids -> (O [T,k] replica ids, actRep [E] (-1 = not activated),
    load [n_inst] = number of activated experts seated on each instance)."""
    L = np.asarray(L)
    # collect: the set of activated experts (Step 1)
    activated = sorted(set(int(e) for e in L.reshape(-1)))
    # initialise actRep and load
    act_rep = np.full(pl.E, -1, dtype=np.int32)
    load = np.zeros(pl.n_inst, dtype=np.int32)
    # single-replica experts go to their only host (Step 2, first loop)
    for e in activated:
        if pl.R[e] == 1:
            g = pl.hosts[e][0]
            act_rep[e] = pl.rids[e][0]
            load[g] += 1
    # multi-replica experts go to the least-loaded host (Step 2, second loop)
    for e in activated:
        if pl.R[e] > 1:
            best = 0
            for idx in range(1, len(pl.hosts[e])):
                if load[pl.hosts[e][idx]] < load[pl.hosts[e][best]]:
                    best = idx
            act_rep[e] = pl.rids[e][best]
            load[pl.hosts[e][best]] += 1
    # rewrite every activation request (Step 3)
    O = np.empty(L.shape, dtype=np.int32)
    for i in range(L.shape[0]):
        for j in range(L.shape[1]):
            O[i, j] = act_rep[L[i, j]]
    return O, act_rep, load


def loads_of(O: np.ndarray, pl: Placement) -> np.ndarray:
    """Distinct activated replicas per instance for an arbitrary rewrite O (any policy)."""
    load = np.zeros(pl.n_inst, dtype=np.int64)
    for rid in set(int(r) for r in np.asarray(O).reshape(-1)):
        load[rid // pl.C] += 1
    return load


def home_only(L: np.ndarray, pl: Placement) -> np.ndarray:
    """Static policy: every request goes to the first replica (lowest instance) of its expert."""
    first = np.array([r[0] for r in pl.rids], dtype=np.int32)
    return first[np.asarray(L)]


def random_replica_from_draws(L: np.ndarray, pl: Placement, U: np.ndarray) -> np.ndarray:
    """Per-request random replica (the token-balancing baselines of Sec. 5: each (token, choice)
    independently picks one replica of its expert uniformly; balances tokens, not activated
    experts).  The draws are inputs: request (i, j) takes replica number U[i, j] mod R(e) of its
    expert e, replicas counted in ascending instance order."""
    L = np.asarray(L)
    U = np.asarray(U, dtype=np.uint64)
    O = np.empty(L.shape, dtype=np.int32)
    for i in range(L.shape[0]):
        for j in range(L.shape[1]):
            r = pl.rids[int(L[i, j])]
            O[i, j] = r[int(U[i, j] % np.uint64(len(r)))]
    return O


def random_replica(L: np.ndarray, pl: Placement, rng: np.random.Generator) -> np.ndarray:
    """random_replica_from_draws with 32-bit draws taken from `rng`."""
    L = np.asarray(L)
    return random_replica_from_draws(L, pl, rng.integers(0, 1 << 32, size=L.shape, dtype=np.uint64))
