"""Pins for the oracle's routing, Alg. 1, exact optimum and activation-count closed forms.
CPU only.  Each pin is something other than the oracle's own formula: hand-worked
fixtures, brute force, a library routine, an invariant or a closed form of Appendix A."""
import itertools
import json
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import bounds, optimum, routing, scheduling
from paper_2512_13525_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def gold(name):
    with open(os.path.join(GOLD, name)) as f:
        return json.load(f)


# ----------------------------------------------------------------------------- routing

def brute_topk(row, k):
    idx = list(range(len(row)))
    idx.sort(key=lambda e: (-float(row[e]), e))
    return idx[:k]


@pytest.mark.parametrize("cfg", [W.tiny(), W.dsv2lite(), W.qwen3(32), W.stress(64, 1.25, 1.5)],
                         ids=lambda c: c.name)
def test_softmax_topk_matches_full_sort_and_scipy(cfg):
    z = W.router_logits(cfg)
    ids, w = routing.route_softmax(z, cfg.k)
    p = scipy.special.softmax(z.astype(np.float64), axis=1)
    for i in range(cfg.T):
        assert list(ids[i]) == brute_topk(z[i], cfg.k)
        ref = p[i, ids[i]]
        np.testing.assert_allclose(w[i], ref / ref.sum(), rtol=1e-12)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=1e-12)
    assert (w > 0).all()
    # weights ordered like the logits they come from
    assert (np.diff(w, axis=1) <= 1e-15).all()
    # un-normalised variant is the plain softmax probability
    _, w_raw = routing.route_softmax(z, cfg.k, renormalize=False)
    np.testing.assert_allclose(w_raw, np.take_along_axis(p, ids.astype(np.int64), axis=1), rtol=1e-12)


def test_softmax_topk_ties_go_to_lower_id():
    z = np.array([[1.0, 3.0, 3.0, 0.0, 3.0], [0.0, 0.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    ids, w = routing.route_softmax(z, 2)
    assert ids.tolist() == [[1, 2], [0, 1]]
    np.testing.assert_allclose(w, 0.5)


def test_sigmoid_group_hand_example():
    g = gold("route_sigmoid_group_tiny.json")
    ids, w, info = routing.route_sigmoid_group(np.array(g["logits"], dtype=np.float32), g["k"],
                                               g["n_group"], g["topk_group"])
    assert ids.tolist() == g["ids"]
    np.testing.assert_allclose(w, np.array(g["w"]), atol=2e-6)
    assert info["kept_groups"].tolist() == [[0, 1], [0, 1]]
    assert info["group_margin"][0] == pytest.approx(1.380797 - 1.244919, abs=1e-5)
    assert info["group_margin"][1] == 0.0


def test_sigmoid_group_brute_force():
    cfg = W.dsv3(64)
    z = W.router_logits(cfg)
    ids, w, info = routing.route_sigmoid_group(z, cfg.k, cfg.n_group, cfg.topk_group, scale=2.5)
    per = cfg.E // cfg.n_group
    for i in range(cfg.T):
        s = [1.0 / (1.0 + math.exp(-float(v))) for v in z[i]]
        gs = []
        for g in range(cfg.n_group):
            top = sorted(s[g * per:(g + 1) * per], reverse=True)
            gs.append(top[0] + top[1])
        keep = sorted(range(cfg.n_group), key=lambda g: (-gs[g], g))[:cfg.topk_group]
        if info["group_margin"][i] > 1e-6:
            assert sorted(keep) == info["kept_groups"][i].tolist()
        cand = [e for e in range(cfg.E) if e // per in info["kept_groups"][i]]
        cand.sort(key=lambda e: (-float(z[i, e]), e))
        assert ids[i].tolist() == cand[:cfg.k]
        tot = sum(s[e] for e in cand[:cfg.k])
        np.testing.assert_allclose(w[i], [2.5 * s[e] / tot for e in cand[:cfg.k]], rtol=1e-12)
    np.testing.assert_allclose(w.sum(axis=1), 2.5, rtol=1e-12)
    # the seeded workload has no rounding-level group ties
    assert info["group_margin"].min() > 1e-5


# ----------------------------------------------------------------------------- placement

def test_placement_tables_and_validation():
    g = gold("aebs_order_and_ties.json")["layout"]
    pl = scheduling.make_placement(g["slot_to_expert"], g["E"], g["n_inst"], g["C"])
    assert pl.hosts == [[0, 1], [0, 2], [1], [2]]
    assert pl.rids == [[0, 2], [1, 4], [3], [5]]
    assert pl.R.tolist() == [2, 2, 1, 1]
    with pytest.raises(scheduling.PlacementError):      # expert 3 missing
        scheduling.make_placement([0, 1, 0, 2, 1, -1], 4, 3, 2)
    with pytest.raises(scheduling.PlacementError):      # two replicas on one instance
        scheduling.make_placement([0, 0, 1, 2, 1, 3], 4, 3, 2)
    with pytest.raises(scheduling.PlacementError):      # id out of range
        scheduling.make_placement([0, 1, 0, 2, 1, 4], 4, 3, 2)
    with pytest.raises(scheduling.PlacementError):      # wrong length
        scheduling.make_placement([0, 1, 2, 3], 4, 3, 2)


@pytest.mark.parametrize("cfg", [W.tiny(), W.dsv2lite(), W.qwen3(), W.dsv3(), W.stress(64, 1.0),
                                 W.stress(64, 1.125, 0.8), W.stress(64, 1.25, 1.5)], ids=lambda c: c.name)
def test_generated_layouts_are_valid(cfg):
    lay = W.build_placement(cfg)
    pl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    assert (lay >= 0).sum() == cfg.S - (1 if cfg.name == "tiny" else 0)
    assert pl.R.sum() == (lay >= 0).sum()
    if cfg.zipf_s > 0:
        # hotter experts never have fewer replicas than colder ones under the count rule
        p = W.expert_popularity(cfg)
        R = W.replica_counts(p, cfg.S)
        order = np.argsort(-p)
        assert (np.diff(R[order]) <= 0).all()
        assert R.sum() == cfg.S


# ----------------------------------------------------------------------------- Alg. 1

@pytest.mark.parametrize("name", ["aebs_tiny_layout.json", "aebs_order_and_ties.json"])
def test_aebs_hand_examples(name):
    g = gold(name)
    lay = g["layout"]
    pl = scheduling.make_placement(lay["slot_to_expert"], lay["E"], lay["n_inst"], lay["C"])
    O, act_rep, load = scheduling.aebs(np.array(g["L"]), pl)
    assert act_rep.tolist() == g["act_rep"]
    assert load.tolist() == g["load"]
    assert O.tolist() == g["O"]
    act = sorted(set(np.array(g["L"]).reshape(-1).tolist()))
    assert optimum.optimum_brute(act, pl) == g["optimum"]
    assert optimum.optimum_matching(act, pl) == g["optimum"]


def check_schedule_invariants(L, O, act_rep, load, pl):
    T, k = L.shape
    lay = pl.slot_to_expert
    # every request lands on a slot that holds a replica of its expert
    assert (lay[O.reshape(-1)] == L.reshape(-1)).all()
    act = sorted(set(L.reshape(-1).tolist()))
    # one replica per activated expert, none for the others
    for e in range(pl.E):
        if e in act:
            assert act_rep[e] in pl.rids[e]
        else:
            assert act_rep[e] == -1
    assert load.sum() == len(act)
    for g in range(pl.n_inst):
        assert load[g] == sum(1 for e in act if act_rep[e] // pl.C == g)
    for e in act:
        if pl.R[e] == 1:
            assert act_rep[e] == pl.rids[e][0]
    # per-expert request counts sum to T*k
    cnt = np.bincount(lay[O.reshape(-1)], minlength=pl.E)
    assert cnt.sum() == T * k
    assert (loads_match := scheduling.loads_of(O, pl).tolist()) == load.tolist(), loads_match


CFGS = [W.tiny(), W.dsv2lite(), W.qwen3(32), W.qwen3(256), W.dsv3(128),
        W.stress(64, 1.0, 0.0), W.stress(64, 1.125, 0.8), W.stress(512, 1.25, 1.5)]


def route(cfg, z):
    if cfg.route == "softmax":
        return routing.route_softmax(z, cfg.k)[:2]
    return routing.route_sigmoid_group(z, cfg.k, cfg.n_group, cfg.topk_group)[:2]


@pytest.mark.parametrize("cfg", CFGS, ids=lambda c: f"{c.name}-T{c.T}")
def test_aebs_invariants_and_bounds(cfg):
    lay = W.build_placement(cfg)
    pl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    ids, _ = route(cfg, W.router_logits(cfg))
    O, act_rep, load = scheduling.aebs(ids, pl)
    check_schedule_invariants(ids, O, act_rep, load, pl)
    act = sorted(set(ids.reshape(-1).tolist()))
    a_max = int(load.max())
    single = np.zeros(cfg.n_inst, dtype=int)
    for e in act:
        if pl.R[e] == 1:
            single[pl.hosts[e][0]] += 1
    opt = optimum.optimum_matching(act, pl)
    assert a_max >= opt >= max(single.max(), -(-len(act) // cfg.n_inst))
    assert a_max <= cfg.C
    # the static policy can never beat the optimum either, and AEBS is no worse than it here
    assert scheduling.loads_of(scheduling.home_only(ids, pl), pl).max() >= opt
    # result depends only on the set of activated experts: shuffle and duplicate tokens
    rng = np.random.default_rng(7)
    sel = rng.permutation(np.concatenate([np.arange(cfg.T), rng.integers(0, cfg.T, cfg.T // 2)]))
    ids2 = ids[sel][:, rng.permutation(cfg.k)]
    O2, act_rep2, load2 = scheduling.aebs(ids2, pl)
    assert act_rep2.tolist() == act_rep.tolist() and load2.tolist() == load.tolist()
    assert (O2 == act_rep[ids2]).all()


def test_aebs_without_replication_is_forced():
    cfg = W.stress(128, 1.0, 0.8)
    lay = W.build_placement(cfg)
    pl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    assert (pl.R == 1).all()
    ids, _ = route(cfg, W.router_logits(cfg))
    O, act_rep, load = scheduling.aebs(ids, pl)
    per = cfg.E // cfg.n_inst
    act = set(ids.reshape(-1).tolist())
    for g in range(cfg.n_inst):
        assert load[g] == len([e for e in act if e // per == g])
    assert (O == ids).all()          # contiguous home layout with C = E/n_inst: rid == expert id


def random_instance(rng, E, n_inst, C, n_act):
    """Random valid layout with S - E extra replicas, and a random activated set."""
    while True:
        lay = np.full((n_inst, C), -1, dtype=np.int64)
        used = np.zeros(n_inst, dtype=int)
        ok = True
        for e in rng.permutation(E):
            free = [g for g in range(n_inst) if used[g] < C]
            if not free:
                ok = False
                break
            g = int(rng.choice(free))
            lay[g, used[g]] = e
            used[g] += 1
        if not ok:
            continue
        for g in range(n_inst):
            while used[g] < C and rng.random() < 0.8:
                cand = [e for e in range(E) if e not in lay[g]]
                lay[g, used[g]] = int(rng.choice(cand))
                used[g] += 1
        break
    act = sorted(rng.choice(E, size=n_act, replace=False).tolist())
    return lay.reshape(-1), act


def test_optimum_matching_equals_brute_force_and_bounds_greedy():
    rng = np.random.default_rng(123)
    worse = 0
    for trial in range(300):
        E = int(rng.integers(4, 13))
        n_inst = int(rng.integers(2, 5))
        C = int(-(-E // n_inst) + rng.integers(0, 3))
        n_act = int(rng.integers(1, E + 1))
        lay, act = random_instance(rng, E, n_inst, C, n_act)
        pl = scheduling.make_placement(lay, E, n_inst, C)
        L = np.array(act, dtype=np.int32).reshape(-1, 1)
        O, act_rep, load = scheduling.aebs(L, pl)
        check_schedule_invariants(L, O, act_rep, load, pl)
        b = optimum.optimum_brute(act, pl)
        assert optimum.optimum_matching(act, pl) == b
        assert load.max() >= b
        worse += int(load.max() > b)
        # no policy beats the optimum
        assert scheduling.loads_of(scheduling.home_only(L, pl), pl).max() >= b
        assert scheduling.loads_of(scheduling.random_replica(L, pl, rng), pl).max() >= b
    assert worse < 150          # the greedy is usually optimal on such small cases


def test_greedy_picks_least_loaded_host_stepwise():
    """Replay Alg. 1's second loop from act_rep alone: at the moment an expert was seated,
    no other host of it had a strictly smaller load, and among equals it took the lowest."""
    cfg = W.stress(256, 1.25, 0.8)
    lay = W.build_placement(cfg)
    pl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    ids, _ = route(cfg, W.router_logits(cfg))
    _, act_rep, load = scheduling.aebs(ids, pl)
    act = sorted(set(ids.reshape(-1).tolist()))
    cur = np.zeros(cfg.n_inst, dtype=int)
    for e in act:
        if pl.R[e] == 1:
            cur[pl.hosts[e][0]] += 1
    for e in act:
        if pl.R[e] > 1:
            g = act_rep[e] // cfg.C
            loads = [(cur[h], h) for h in pl.hosts[e]]
            assert (cur[g], g) == min(loads)
            cur[g] += 1
    assert cur.tolist() == load.tolist()


# ----------------------------------------------------------------------------- Appendix A closed forms

def test_expected_activated_closed_form_uniform():
    # Eq. 4 holds with equality without replication; uniform routing: (E/n)*(1-(1-k/E)^B)
    assert bounds.expected_activated(np.full(256, 8 / 256), range(16), 64) == pytest.approx(
        16 * (1 - (1 - 8 / 256) ** 64))
    assert 16 * (1 - (1 - 8 / 256) ** 64) == pytest.approx(13.90, abs=0.01)
    E, k, n_inst, B, N = 64, 6, 4, 16, 1500
    per = E // n_inst
    lay = np.arange(E)
    pl = scheduling.make_placement(lay, E, n_inst, per)
    rng = np.random.default_rng(11)
    tot = np.zeros(n_inst)
    amax = []
    for _ in range(N):
        ids = W.uniform_topk_ids(E, k, B, rng)
        _, _, load = scheduling.aebs(ids, pl)
        tot += load
        amax.append(load.max())
    expect = bounds.expected_activated(np.full(E, k / E), range(per), B)
    assert expect == pytest.approx(per * (1 - (1 - k / E) ** B))
    sigma_mean = math.sqrt(expect / N)      # Var(a_g) <= E[a_g] (negative association)
    assert np.abs(tot / N - expect).max() < 4 * sigma_mean
    # Eq. 5 is an upper bound on a_max (checked on the mean and as a high quantile)
    bound = bounds.a_max_bound(expect, per, n_inst)
    assert np.mean(amax) <= bound
    assert np.mean(np.array(amax) <= bound) > 0.95


def test_a_max_bound_formula_values():
    assert bounds.a_max_bound(10.0, 27, 8) == math.floor(10 + math.sqrt(20 * math.log(8)) + 1)
    assert bounds.a_max_bound(26.5, 27, 16) == 28      # capped at C, then +1


def test_random_replica_draws_pick_the_stated_replica():
    """The token-balancing baseline with its draws as inputs: draw 0 is the first replica (the
    home-only policy), draw R(e)-1 the last, every choice hosts the expert, and the loads are the
    distinct replicas per instance."""
    cfg = W.stress(64, 1.25, 0.8)
    lay = W.build_placement(cfg)
    pl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    rng = np.random.default_rng(11)
    L = np.stack([rng.choice(cfg.E, size=cfg.k, replace=False) for _ in range(40)]).astype(np.int32)
    zero = scheduling.random_replica_from_draws(L, pl, np.zeros(L.shape, dtype=np.uint32))
    np.testing.assert_array_equal(zero, scheduling.home_only(L, pl))
    lastd = np.array([[pl.R[e] - 1 for e in row] for row in L], dtype=np.uint32)
    last = scheduling.random_replica_from_draws(L, pl, lastd)
    assert all(last[i, j] == pl.rids[int(L[i, j])][-1] for i in range(L.shape[0]) for j in range(L.shape[1]))
    U = rng.integers(0, 1 << 32, size=L.shape, dtype=np.uint64)
    O = scheduling.random_replica_from_draws(L, pl, U)
    lay64 = np.asarray(lay)
    assert (lay64[O] == L).all()                                  # the chosen slot holds the requested expert
    # wrap-around of the modulus: draw + R(e) picks the same replica
    shifted = U + np.array([[pl.R[e] for e in row] for row in L], dtype=np.uint64)
    np.testing.assert_array_equal(scheduling.random_replica_from_draws(L, pl, shifted), O)
    load = scheduling.loads_of(O, pl)
    assert load.sum() == len(set(O.reshape(-1).tolist()))
    assert load.max() >= optimum.optimum_matching(sorted(set(L.reshape(-1).tolist())), pl)   # no policy beats the optimum
