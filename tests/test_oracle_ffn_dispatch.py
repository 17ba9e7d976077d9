"""Pins for the oracle's permutation, grouped FFN, combine and whole-layer result.  CPU only."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import dispatch, ffn, routing, scheduling
from paper_2512_13525_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def small_cfg(**kw):
    base = dict(name="small", E=8, k=2, d_h=32, d_e=48, T=24, n_inst=2, C=5, dtype="f32", seed=3,
                fixed_layout=(0, 1, 2, 3, -1, 4, 5, 6, 7, 0))
    base.update(kw)
    return W.MoEConfig(**base)


def setup(cfg):
    lay = W.build_placement(cfg)
    pl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    ids, w = routing.route_softmax(W.router_logits(cfg), cfg.k)
    X = W.activations(cfg)
    return lay, pl, ids, w, X


# ----------------------------------------------------------------------------- permutation

@pytest.mark.parametrize("cfg", [W.tiny(), W.qwen3(256), W.stress(512, 1.25, 0.8)], ids=lambda c: c.name)
def test_permute_is_a_stable_grouping(cfg):
    lay, pl, ids, w, _ = setup(cfg)
    O, _, load = scheduling.aebs(ids, pl)
    seen = []
    total = 0
    for g in range(cfg.n_inst):
        cnt, off, perm = dispatch.permute(O, g, cfg.C)
        flat = O.reshape(-1)
        local = np.nonzero(flat // cfg.C == g)[0]
        # library statement: stable argsort of the local pairs by slot
        key = flat[local] - g * cfg.C
        np.testing.assert_array_equal(perm, local[np.argsort(key, kind="stable")])
        np.testing.assert_array_equal(off, np.concatenate([[0], np.cumsum(cnt)]))
        np.testing.assert_array_equal(cnt, np.bincount(key, minlength=cfg.C))
        assert cnt.sum() == len(perm) == off[-1]
        assert (cnt > 0).sum() == load[g]          # activated slots == scheduler's load
        for s in range(cfg.C):
            seg = perm[off[s]:off[s + 1]]
            assert (np.diff(seg) > 0).all()
            assert (flat[seg] == g * cfg.C + s).all()
        seen.extend(perm.tolist())
        total += len(perm)
    assert total == cfg.T * cfg.k and sorted(seen) == list(range(cfg.T * cfg.k))


def test_permute_empty_instance():
    O = np.array([[5, 6], [7, 5]], dtype=np.int32)
    cnt, off, perm = dispatch.permute(O, 0, 5)
    assert cnt.tolist() == [0] * 5 and off.tolist() == [0] * 6 and perm.size == 0


# ----------------------------------------------------------------------------- FFN

def test_swiglu_hand_example():
    with open(os.path.join(GOLD, "swiglu_tiny.json")) as f:
        g = json.load(f)
    y = ffn.expert_ffn(np.array(g["x"]), np.array(g["w13"]), np.array(g["w2"]))
    np.testing.assert_allclose(y, np.array(g["y"]), rtol=1e-9)


def test_expert_ffn_equals_library_mlp():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 40))
    w13 = rng.standard_normal((2 * 24, 40)) * 0.2
    w2 = rng.standard_normal((40, 24)) * 0.2
    tx, t13, t2 = (torch.from_numpy(a) for a in (x, w13, w2))
    ref = (torch.nn.functional.silu(tx @ t13[:24].T) * (tx @ t13[24:].T)) @ t2.T
    np.testing.assert_allclose(ffn.expert_ffn(x, w13, w2), ref.numpy(), rtol=1e-11, atol=1e-13)
    # zero down-projection gives zero; the map is linear in W2
    assert not ffn.expert_ffn(x, w13, np.zeros_like(w2)).any()
    w2b = rng.standard_normal((40, 24))
    np.testing.assert_allclose(ffn.expert_ffn(x, w13, w2 + 3 * w2b),
                               ffn.expert_ffn(x, w13, w2) + 3 * ffn.expert_ffn(x, w13, w2b), rtol=1e-9, atol=1e-11)


def test_grouped_ffn_single_expert_k1_is_plain_mlp():
    cfg = small_cfg(E=1, k=1, n_inst=1, C=1, fixed_layout=(0,), T=9)
    X = W.activations(cfg)
    w13, w2 = W.expert_weights(cfg, 0)
    off = np.array([0, cfg.T], dtype=np.int32)
    perm = np.arange(cfg.T, dtype=np.int32)
    Yp = ffn.grouped_ffn(X, w13[None], w2[None], off, perm, 1)
    tx, t13, t2 = (torch.from_numpy(a.astype(np.float64)) for a in (X, w13, w2))
    ref = (torch.nn.functional.silu(tx @ t13[:cfg.d_e].T) * (tx @ t13[cfg.d_e:].T)) @ t2.T
    np.testing.assert_allclose(Yp, ref.numpy(), rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("policy", ["aebs", "home", "random"])
def test_layer_is_schedule_independent_and_matches_dense_loop(policy):
    """Sum over instances of (permute -> grouped FFN -> combine) equals the dense per-token
    layer for any valid schedule: replicas hold identical weights."""
    cfg = small_cfg()
    lay, pl, ids, w, X = setup(cfg)
    if policy == "aebs":
        O = scheduling.aebs(ids, pl)[0]
    elif policy == "home":
        O = scheduling.home_only(ids, pl)
    else:
        O = scheduling.random_replica(ids, pl, np.random.default_rng(5))
    cache = {}
    Y = np.zeros((cfg.T, cfg.d_h))
    untouched_ok = True
    for g in range(cfg.n_inst):
        W13, W2 = W.instance_weights(cfg, lay, g, cache)
        cnt, off, perm = dispatch.permute(O, g, cfg.C)
        # poison the weights of slots with no request: they must not be touched
        for s in range(cfg.C):
            if cnt[s] == 0:
                W13[s] = np.nan
                W2[s] = np.nan
        Yp = ffn.grouped_ffn(X, W13, W2, off, perm, cfg.k)
        untouched_ok &= bool(np.isfinite(Yp).all())
        Y += dispatch.combine(Yp, perm, w, cfg.T, cfg.k)
    assert untouched_ok
    dense = ffn.dense_layer(X, ids, w, lambda e: W.expert_weights(cfg, e))
    np.testing.assert_allclose(Y, dense, rtol=1e-9, atol=1e-12)


def test_combine_with_identity_ffn():
    cfg = small_cfg()
    lay, pl, ids, w, X = setup(cfg)
    O = scheduling.aebs(ids, pl)[0]
    tot = np.zeros((cfg.T, cfg.d_h))
    for g in range(cfg.n_inst):
        cnt, off, perm = dispatch.permute(O, g, cfg.C)
        Yp = X[perm // cfg.k].astype(np.float64)        # "FFN" = identity
        Y = dispatch.combine(Yp, perm, w, cfg.T, cfg.k)
        local_w = np.where(O // cfg.C == g, w, 0.0).sum(axis=1)
        np.testing.assert_allclose(Y, X * local_w[:, None], rtol=1e-12, atol=1e-15)
        tot += Y
    np.testing.assert_allclose(tot, X, rtol=1e-12, atol=1e-14)   # weights sum to 1


def test_bf16_rounding_helper():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.3895313892515355e38, 1e-40], dtype=np.float32)
    r = W.round_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, ref)
    rng = np.random.default_rng(1)
    y = rng.standard_normal(100000).astype(np.float32) * 3
    np.testing.assert_array_equal(W.round_to_bf16(y), torch.from_numpy(y).to(torch.bfloat16).to(torch.float32).numpy())
    np.testing.assert_array_equal(W.bf16_bits_to_f32(W.bf16_bits(W.round_to_bf16(y))), W.round_to_bf16(y))


def test_shared_expert_is_one_more_choice_with_weight_one():
    """Adding a shared expert equals the dense per-token loop run with one extra choice per token
    (the shared expert, weight 1); with all routed weights zero it is a plain MLP."""
    import torch
    cfg = W.MoEConfig("sh", E=6, k=2, d_h=16, d_e=8, T=5, n_inst=2, C=4, zipf_s=0.5, dtype="f32", seed=2)
    X = W.activations(cfg)
    z = W.router_logits(cfg)
    from oracle import routing
    ids, w = routing.route_softmax(z, cfg.k)
    ws13, ws2 = W.shared_expert_weights(cfg, 12)
    weights_of = lambda e: (ws13, ws2) if e == cfg.E else W.expert_weights(cfg, e)
    routed = ffn.dense_layer(X, ids, w, weights_of)
    want = ffn.dense_layer(X, np.concatenate([ids, np.full((cfg.T, 1), cfg.E, dtype=ids.dtype)], axis=1),
                           np.concatenate([w, np.ones((cfg.T, 1))], axis=1), weights_of)
    np.testing.assert_allclose(ffn.add_shared_expert(routed, X, ws13, ws2), want, rtol=1e-12, atol=1e-15)
    x = torch.from_numpy(X.astype(np.float64))
    h = x @ torch.from_numpy(ws13[:12].astype(np.float64)).T
    u = x @ torch.from_numpy(ws13[12:].astype(np.float64)).T
    mlp = (torch.nn.functional.silu(h) * u) @ torch.from_numpy(ws2.astype(np.float64)).T
    np.testing.assert_allclose(ffn.add_shared_expert(np.zeros_like(routed), X, ws13, ws2), mlp.numpy(), rtol=1e-10, atol=1e-14)
