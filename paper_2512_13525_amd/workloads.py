"""Seeded synthetic inputs for the MoE-instance layer step.

This module only *draws inputs*: router logits, activations, expert weights and
a replica layout (the table the paper's control plane would hand to every MoE
instance).  It holds none of the hot path's arithmetic (no routing, no
scheduling, no FFN) and is the one module the CPU oracle's tests and the HIP
path's tests both feed from.

Shapes and skew stand in for the models and request traces the paper measured
on (Sec. 5, "Models and workloads"), which are not available here: only layer
dimensions, top-k, expert counts and a Zipf popularity skew are kept.

Replica counts follow the rule of Appendix B ("Replica count"): one replica per
logical expert, then every spare slot goes to the expert with the largest
activation count per replica.  The co-activation-aware placement of Alg. 3 is
replaced by a simpler deterministic rule (see ``build_placement``).
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class MoEConfig:
    name: str
    E: int                 # logical experts
    k: int                 # experts per token
    d_h: int               # hidden size
    d_e: int               # expert intermediate size
    T: int                 # tokens in the decode batch
    n_inst: int            # MoE instances (n_e in the paper)
    C: int                 # replica slots per instance
    route: str = "softmax"         # "softmax" | "sigmoid_group"
    n_group: int = 1
    topk_group: int = 1
    zipf_s: float = 0.0
    dtype: str = "bf16"            # "bf16" | "f32"
    seed: int = 0
    fixed_layout: Optional[Tuple[int, ...]] = None   # slot_to_expert if prescribed

    @property
    def S(self) -> int:
        return self.n_inst * self.C

    @property
    def bytes_per_expert(self) -> int:
        return 3 * self.d_h * self.d_e * (2 if self.dtype == "bf16" else 4)

    def with_(self, **kw) -> "MoEConfig":
        return dataclasses.replace(self, **kw)


def tiny() -> MoEConfig:
    # instance 0 = {0,1,2,3,empty}; instance 1 = {4,5,6,7,replica of 0}
    return MoEConfig("tiny", E=8, k=2, d_h=256, d_e=512, T=64, n_inst=2, C=5,
                     dtype="f32", seed=0,
                     fixed_layout=(0, 1, 2, 3, -1, 4, 5, 6, 7, 0))


def dsv2lite(T: int = 128) -> MoEConfig:
    return MoEConfig("dsv2lite", E=64, k=6, d_h=2048, d_e=1408, T=T, n_inst=4, C=17,
                     zipf_s=1.1, seed=0)


def qwen3(T: int = 256) -> MoEConfig:
    return MoEConfig("qwen3_30b_a3b", E=128, k=8, d_h=2048, d_e=768, T=T, n_inst=8, C=17,
                     zipf_s=1.0, seed=0)


def dsv3(T: int = 512) -> MoEConfig:
    return MoEConfig("dsv3", E=256, k=8, d_h=7168, d_e=2048, T=T, n_inst=8, C=36,
                     route="sigmoid_group", n_group=8, topk_group=4, zipf_s=1.2, seed=0)


def stress(T: int = 64, r: float = 1.0, s: float = 0.0) -> MoEConfig:
    C = int(round(16 * r))
    return MoEConfig(f"stress_r{r}_s{s}", E=256, k=8, d_h=4096, d_e=1536, T=T, n_inst=16, C=C,
                     zipf_s=s, seed=0)


NAMED = {"tiny": tiny, "dsv2lite": dsv2lite, "qwen3": qwen3, "dsv3": dsv3, "stress": stress}


# --------------------------------------------------------------------------- bf16 helpers

def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> float32 holding the nearest bf16 value (ties to even)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 holding bf16-representable values -> uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- popularity / logits

def _rng(cfg: MoEConfig, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.default_rng([cfg.seed, stream, sub])


def expert_popularity(cfg: MoEConfig) -> np.ndarray:
    """p_e proportional to rank(e)^-s, rank = seeded random permutation; sums to 1."""
    rank = _rng(cfg, 1).permutation(cfg.E) + 1
    p = rank.astype(np.float64) ** (-cfg.zipf_s)
    return p / p.sum()


def router_logits(cfg: MoEConfig, T: Optional[int] = None, sub: int = 0) -> np.ndarray:
    """N(0,1) logits plus the per-expert bias ln(E*p_e); float32 [T,E]."""
    T = cfg.T if T is None else T
    z = _rng(cfg, 2, sub).standard_normal((T, cfg.E), dtype=np.float32)
    if cfg.zipf_s != 0.0:
        bias = np.log(cfg.E * expert_popularity(cfg)).astype(np.float32)
        z = z + bias[None, :]
    return np.ascontiguousarray(z, dtype=np.float32)


def router_weights(cfg: MoEConfig) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Router (gate) matrix W_r [E,d_h] ~ N(0, 1/d_h), so that logits of N(0,1) activations are
    ~N(0,1) like `router_logits`, and the per-expert bias ln(E*p_e) of the Zipf skew (None when
    zipf_s == 0).  W_r is bf16-representable when cfg.dtype == 'bf16'; the bias stays float32."""
    wr = _rng(cfg, 5).standard_normal((cfg.E, cfg.d_h), dtype=np.float32) * np.float32(cfg.d_h ** -0.5)
    if cfg.dtype == "bf16":
        wr = round_to_bf16(wr)
    bias = None
    if cfg.zipf_s != 0.0:
        bias = np.log(cfg.E * expert_popularity(cfg)).astype(np.float32)
    return np.ascontiguousarray(wr), bias


def topic_bias(cfg: MoEConfig, n_topics: int, boost: float, contiguous: bool) -> np.ndarray:
    """Per-topic logit bias [n_topics, E] of a synthetic trace with co-activation structure (a
    stand-in for the request traces of Sec. 5: batches of one topic prefer one cluster of
    experts).  Topic t boosts E/n_topics experts by `boost`: a contiguous id range, or a seeded
    random subset.  Added to the Zipf bias of `router_logits`; float32."""
    E = cfg.E
    per = E // n_topics
    order = np.arange(E) if contiguous else _rng(cfg, 6).permutation(E)
    bias = np.zeros((n_topics, E), dtype=np.float32)
    for t in range(n_topics):
        bias[t, order[t * per:(t + 1) * per]] = boost
    if cfg.zipf_s != 0.0:
        bias += np.log(E * expert_popularity(cfg)).astype(np.float32)[None, :]
    return bias


def activations(cfg: MoEConfig, T: Optional[int] = None, sub: int = 0) -> np.ndarray:
    """N(0,1) activations, float32 [T,d_h]; bf16-representable when cfg.dtype == 'bf16'."""
    T = cfg.T if T is None else T
    x = _rng(cfg, 3, sub).standard_normal((T, cfg.d_h), dtype=np.float32)
    return round_to_bf16(x) if cfg.dtype == "bf16" else x


def expert_weights(cfg: MoEConfig, e: int) -> Tuple[np.ndarray, np.ndarray]:
    """Weights of logical expert e, N(0, 0.02): W13 [2*d_e, d_h] (gate rows, then up rows)
    and W2 [d_h, d_e]; float32, bf16-representable when cfg.dtype == 'bf16'.
    Every replica of e holds a copy of exactly these values."""
    g = _rng(cfg, 4, e)
    w13 = g.standard_normal((2 * cfg.d_e, cfg.d_h), dtype=np.float32) * np.float32(0.02)
    w2 = g.standard_normal((cfg.d_h, cfg.d_e), dtype=np.float32) * np.float32(0.02)
    if cfg.dtype == "bf16":
        w13, w2 = round_to_bf16(w13), round_to_bf16(w2)
    return w13, w2


def shared_expert_weights(cfg: MoEConfig, d_e_shared: int) -> Tuple[np.ndarray, np.ndarray]:
    """Weights of a shared expert of width d_e_shared, N(0, 0.02) like the routed experts:
    W13 [2*d_e_shared, d_h], W2 [d_h, d_e_shared]."""
    g = _rng(cfg, 7)
    w13 = g.standard_normal((2 * d_e_shared, cfg.d_h), dtype=np.float32) * np.float32(0.02)
    w2 = g.standard_normal((cfg.d_h, d_e_shared), dtype=np.float32) * np.float32(0.02)
    if cfg.dtype == "bf16":
        w13, w2 = round_to_bf16(w13), round_to_bf16(w2)
    return w13, w2


def instance_weights(cfg: MoEConfig, slot_to_expert: np.ndarray, g: int,
                     cache: Optional[Dict[int, Tuple[np.ndarray, np.ndarray]]] = None
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """Physical weights of instance g: W13 [C, 2*d_e, d_h], W2 [C, d_h, d_e] (float32).
    Empty slots are zero-filled."""
    W13 = np.zeros((cfg.C, 2 * cfg.d_e, cfg.d_h), dtype=np.float32)
    W2 = np.zeros((cfg.C, cfg.d_h, cfg.d_e), dtype=np.float32)
    for s in range(cfg.C):
        e = int(slot_to_expert[g * cfg.C + s])
        if e < 0:
            continue
        if cache is not None and e in cache:
            w13, w2 = cache[e]
        else:
            w13, w2 = expert_weights(cfg, e)
            if cache is not None:
                cache[e] = (w13, w2)
        W13[s], W2[s] = w13, w2
    return W13, W2


# --------------------------------------------------------------------------- replica layout

def replica_counts(c: np.ndarray, S: int) -> np.ndarray:
    """Appendix B, 'Replica count': one replica each, then the S-E spare slots go one at a
    time to the expert with the largest c(e)/R(e) (lower id on ties)."""
    E = len(c)
    if S < E:
        raise ValueError("fewer slots than experts")
    R = np.ones(E, dtype=np.int64)
    for _ in range(S - E):
        R[int(np.argmax(c / R))] += 1
    return R


def build_placement(cfg: MoEConfig) -> np.ndarray:
    """slot_to_expert [n_inst*C] (int32, -1 = empty slot).

    Home replicas are contiguous (expert e lives on instance e // (E/n_inst)).  Spare
    slots receive the extra replicas chosen by ``replica_counts`` with c(e) = Zipf
    popularity; each extra replica goes to the instance that still has a free slot,
    does not host that expert yet, and has the smallest summed popularity so far
    (lowest instance id on ties).  Experts are seated hottest first.
    """
    if cfg.fixed_layout is not None:
        lay = np.asarray(cfg.fixed_layout, dtype=np.int32)
        assert lay.shape == (cfg.S,)
        return lay
    E, n, C = cfg.E, cfg.n_inst, cfg.C
    if E % n != 0 or C < E // n:
        raise ValueError("layout needs E divisible by n_inst and C >= E/n_inst")
    per = E // n
    lay = np.full((n, C), -1, dtype=np.int32)
    for e in range(E):
        lay[e // per, e % per] = e
    p = expert_popularity(cfg)
    R = replica_counts(p, n * C)
    used = np.full(n, per, dtype=np.int64)
    heat = np.array([p[g * per:(g + 1) * per].sum() for g in range(n)])
    hosts: List[set] = [{e // per} for e in range(E)]
    extras = [(e, r) for e in range(E) for r in range(int(R[e]) - 1)]
    extras.sort(key=lambda t: (-p[t[0]], t[0], t[1]))
    for e, _ in extras:
        cand = [g for g in range(n) if used[g] < C and g not in hosts[e]]
        if not cand:
            continue            # every instance with a free slot already hosts e
        g = min(cand, key=lambda q: (heat[q], q))
        lay[g, used[g]] = e
        used[g] += 1
        heat[g] += p[e]
        hosts[e].add(g)
    # slots an extra replica could not take go to the expert with the largest
    # popularity per replica among those the instance does not host yet
    for g in range(n):
        while used[g] < C:
            cand = [e for e in range(E) if g not in hosts[e]]
            if not cand:
                break
            e = min(cand, key=lambda q: (-p[q] / len(hosts[q]), q))
            lay[g, used[g]] = e
            used[g] += 1
            heat[g] += p[e]
            hosts[e].add(g)
    return lay.reshape(-1)


def uniform_topk_ids(E: int, k: int, T: int, rng: np.random.Generator) -> np.ndarray:
    """T independent uniformly random k-subsets of range(E) (int32 [T,k])."""
    keys = rng.random((T, E))
    return np.argsort(keys, axis=1)[:, :k].astype(np.int32)
