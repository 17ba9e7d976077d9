"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integers bit-exact; fp32 weights to rtol 1e-5; FFN / layer output within a
relative Frobenius error of 2e-2 (bf16 path, the bar the task states) or 1e-5 (fp32 path:
K <= 512 fp32 accumulations, error ~ sqrt(K)*2^-24 ~ 1.3e-6, with margin)."""
import numpy as np
import pytest
import torch

from paper_2512_13525_amd import binding as B
from paper_2512_13525_amd import workloads as W
from paper_2512_13525_amd.layer import LayerStep, to_device_bf16
from oracle import dispatch, ffn, scheduling

from helpers import OracleRun, expected_blocks, oracle_route, rel_fro

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
TOL_F32 = 1e-5


def small(name="small", **kw):
    base = dict(name=name, E=18, k=3, d_h=64, d_e=96, T=37, n_inst=3, C=7, zipf_s=0.9, seed=5)
    base.update(kw)
    return W.MoEConfig(**base)


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def upload_weights(step, cfg, W13, W2):
    if cfg.dtype == "bf16":
        step.set_weights(to_device_bf16(W13), to_device_bf16(W2))
    else:
        step.set_weights(torch.from_numpy(W13).cuda(), torch.from_numpy(W2).cuda())


def upload_x(cfg, X):
    return to_device_bf16(X) if cfg.dtype == "bf16" else torch.from_numpy(X).cuda()


ROUTE_CFGS = [W.tiny(), W.dsv2lite(), W.qwen3(32), W.qwen3(1024), W.dsv3(512), W.stress(8192, 1.25, 1.5),
              small(), small("odd", E=70, k=5, T=3), small("e1024", E=1024, k=32, T=9)]


@pytest.mark.parametrize("cfg", ROUTE_CFGS, ids=lambda c: f"{c.name}-T{c.T}")
def test_route_parity(cfg):
    logits = W.router_logits(cfg)
    ids, w, info = oracle_route(cfg, logits)
    d_logits = torch.from_numpy(logits).cuda()
    d_ids = torch.full((cfg.T, cfg.k), -7, dtype=torch.int32, device="cuda")
    d_w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
    if cfg.route == "softmax":
        B.moe_route(d_logits, cfg.k, d_ids, d_w)
    else:
        B.moe_route(d_logits, cfg.k, d_ids, d_w, B.MOE_ROUTE_SIGMOID_GROUP, True, cfg.n_group, cfg.topk_group, 1.0)
    torch.cuda.synchronize()
    g_ids, g_w = d_ids.cpu().numpy(), d_w.cpu().numpy()
    if info is None:
        np.testing.assert_array_equal(g_ids, ids)
        np.testing.assert_allclose(g_w, w, rtol=1e-5)
    else:
        sure = info["group_margin"] > 1e-5            # a genuine group decision, not a rounding tie
        assert sure.mean() > 0.99
        np.testing.assert_array_equal(g_ids[sure], ids[sure])
        np.testing.assert_allclose(g_w[sure], w[sure], rtol=1e-5)
        per = cfg.E // cfg.n_group                    # near-ties: still a valid group-limited selection
        for i in np.nonzero(~sure)[0]:
            assert len(set(g_ids[i] // per)) <= cfg.topk_group and len(set(g_ids[i])) == cfg.k
    if cfg.route == "softmax":
        # un-normalised variant
        B.moe_route(d_logits, cfg.k, d_ids, d_w, B.MOE_ROUTE_SOFTMAX, False)
        torch.cuda.synchronize()
        from oracle import routing
        _, w_raw = routing.route_softmax(logits, cfg.k, renormalize=False)
        np.testing.assert_array_equal(d_ids.cpu().numpy(), ids)
        np.testing.assert_allclose(d_w.cpu().numpy(), w_raw, rtol=2e-5)


def test_route_ties_lower_id():
    z = np.zeros((5, 64), dtype=np.float32)
    z[1, [3, 9, 40]] = 2.0
    z[2, :] = -1.5
    z[3, 63] = 1.0
    d_ids = torch.empty((5, 4), dtype=torch.int32, device="cuda")
    d_w = torch.empty((5, 4), dtype=torch.float32, device="cuda")
    B.moe_route(torch.from_numpy(z).cuda(), 4, d_ids, d_w)
    torch.cuda.synchronize()
    from oracle import routing
    ids, w = routing.route_softmax(z, 4)
    np.testing.assert_array_equal(d_ids.cpu().numpy(), ids)
    np.testing.assert_allclose(d_w.cpu().numpy(), w, rtol=1e-5)


SCHED_CFGS = ([W.tiny(), W.dsv2lite(), W.qwen3(32), W.qwen3(256), W.qwen3(1024), W.dsv3(512), small(),
               small("k1", k=1, T=1), small("ragged", k=5, T=77),
               # more than 64 slots per instance: the slot scan takes two rounds of 64 lanes
               small("many_slots", E=150, n_inst=2, C=80, k=4, T=200)] +
              [W.stress(T, r, s) for (T, r, s) in [(64, 1.0, 0.0), (64, 1.125, 0.8), (64, 1.25, 1.5),
                                                   (1000, 1.25, 0.8), (8192, 1.125, 1.5), (8192, 1.25, 0.0)]])


def gpu_schedule(cfg, lay, ids):
    pl = B.Placement(lay, cfg.E, cfg.n_inst, cfg.C)
    T = ids.shape[0]
    d_rid = torch.full((T, cfg.k), -9, dtype=torch.int32, device="cuda")
    d_rep = torch.full((cfg.E,), -9, dtype=torch.int32, device="cuda")
    d_load = torch.full((cfg.n_inst,), -9, dtype=torch.int32, device="cuda")
    B.moe_schedule(pl, dev_i32(ids) if T else None, T, cfg.k, d_rid if T else None, d_rep, d_load)
    torch.cuda.synchronize()
    return pl, d_rid, d_rep.cpu().numpy(), d_load.cpu().numpy()


@pytest.mark.parametrize("cfg", SCHED_CFGS, ids=lambda c: f"{c.name}-T{c.T}")
def test_schedule_and_permute_parity(cfg):
    lay = W.build_placement(cfg)
    opl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    ids, _, _ = oracle_route(cfg, W.router_logits(cfg))
    O, act_rep, load = scheduling.aebs(ids, opl)
    pl, d_rid, g_rep, g_load = gpu_schedule(cfg, lay, ids)
    np.testing.assert_array_equal(g_rep, act_rep)
    np.testing.assert_array_equal(g_load, load)
    np.testing.assert_array_equal(d_rid.cpu().numpy(), O)
    # determinism: a second run gives the same bits
    _, d_rid2, g_rep2, g_load2 = gpu_schedule(cfg, lay, ids)
    assert torch.equal(d_rid, d_rid2) and (g_rep2 == g_rep).all() and (g_load2 == g_load).all()
    # permute for every instance (or a spread of them when there are many)
    n = cfg.T * cfg.k
    for g in sorted(set([0, cfg.n_inst - 1, int(np.argmax(load)), int(np.argmin(load))])):
        cnt, off, perm = dispatch.permute(O, g, cfg.C)
        d_cnt = torch.full((cfg.C,), -9, dtype=torch.int32, device="cuda")
        d_off = torch.full((cfg.C + 1,), -9, dtype=torch.int32, device="cuda")
        d_perm = torch.full((n,), -9, dtype=torch.int32, device="cuda")
        d_pos = torch.full((n,), -9, dtype=torch.int32, device="cuda")
        d_blk = torch.full((B.moe_block_list_len(cfg.T, cfg.k, cfg.C),), -9, dtype=torch.int32, device="cuda")
        B.moe_permute(pl, g, d_rid, cfg.T, cfg.k, d_cnt, d_off, d_perm, d_pos, d_blk)
        torch.cuda.synchronize()
        blk = expected_blocks(off, B.moe_block_rows(cfg.T))
        assert blk[0] <= B.moe_max_blocks(cfg.T, cfg.k, cfg.C)
        g_blk = d_blk.cpu().numpy()
        np.testing.assert_array_equal(g_blk[:len(blk)], blk)
        assert (g_blk[len(blk):] == -9).all()                   # entries past the last block untouched
        np.testing.assert_array_equal(d_cnt.cpu().numpy(), cnt)
        np.testing.assert_array_equal(d_off.cpu().numpy(), off)
        g_perm = d_perm.cpu().numpy()
        np.testing.assert_array_equal(g_perm[:len(perm)], perm)
        assert (g_perm[len(perm):] == -9).all()                 # capacity tail untouched
        pos = np.full(n, -1, dtype=np.int32)
        pos[perm] = np.arange(len(perm))
        np.testing.assert_array_equal(d_pos.cpu().numpy(), pos)


@pytest.mark.parametrize("cfg", [W.tiny(), W.dsv2lite(), W.qwen3(256), W.dsv3(512), small("ragged", k=5, T=77),
                                 W.stress(1000, 1.25, 0.8), W.stress(8192, 1.125, 1.5)],
                         ids=lambda c: f"{c.name}-T{c.T}")
def test_baseline_policies_parity(cfg):
    """moe_schedule_baseline: the home-only and the random-replica policy, bit for bit."""
    lay = W.build_placement(cfg)
    opl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    pl = B.Placement(lay, cfg.E, cfg.n_inst, cfg.C)
    ids, _, _ = oracle_route(cfg, W.router_logits(cfg))
    U = np.random.default_rng(cfg.seed + 17).integers(0, 1 << 32, size=ids.shape, dtype=np.uint64)
    d_draws = torch.from_numpy(U.astype(np.uint32).view(np.int32)).cuda()
    for policy, O in ((B.MOE_POLICY_HOME, scheduling.home_only(ids, opl)),
                      (B.MOE_POLICY_RANDOM, scheduling.random_replica_from_draws(ids, opl, U))):
        d_rid = torch.full(ids.shape, -9, dtype=torch.int32, device="cuda")
        d_load = torch.full((cfg.n_inst,), -9, dtype=torch.int32, device="cuda")
        B.moe_schedule_baseline(pl, dev_i32(ids), cfg.T, cfg.k, policy,
                                d_draws if policy == B.MOE_POLICY_RANDOM else None, d_rid, d_load)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_rid.cpu().numpy(), O)
        np.testing.assert_array_equal(d_load.cpu().numpy(), scheduling.loads_of(O, opl))


def test_schedule_empty_batch_and_layout_swap():
    cfg = W.tiny()
    lay = W.build_placement(cfg)
    pl, _, rep, load = gpu_schedule(cfg, lay, np.zeros((0, cfg.k), dtype=np.int32))
    assert (rep == -1).all() and (load == 0).all()
    # a new layout between two steps is followed with no stale state
    ids = np.array([[0, 1], [2, 3], [4, 0], [1, 4]], dtype=np.int32)
    _, d_rid, rep1, load1 = gpu_schedule(cfg, lay, ids)
    assert rep1.tolist() == [9, 1, 2, 3, 5, -1, -1, -1] and load1.tolist() == [3, 2]
    lay2 = np.array([4, 5, 6, 7, 0, 0, 1, 2, 3, -1], dtype=np.int32)        # instances swapped
    O2, rep2, load2 = scheduling.aebs(ids, scheduling.make_placement(lay2, 8, 2, 5))
    _, d_rid2, g_rep2, g_load2 = gpu_schedule(cfg, lay2, ids)
    np.testing.assert_array_equal(g_rep2, rep2)
    np.testing.assert_array_equal(g_load2, load2)
    np.testing.assert_array_equal(d_rid2.cpu().numpy(), O2)
    with pytest.raises(B.MoeError):
        B.Placement([0, 1, 2, 3, -1, 4, 5, 6, -1, 0], 8, 2, 5)                  # expert 7 missing


FFN_CFGS = [W.tiny(), small(), small("multi_tile", T=300, k=4, E=8, n_inst=2, C=5, d_h=128, d_e=160, zipf_s=1.5),
            small("f32_ragged", dtype="f32", T=21, d_h=36, d_e=20),
            W.dsv2lite(), W.qwen3(32), W.qwen3(256), W.qwen3(1024), W.stress(64, 1.25, 0.8),
            W.stress(2048, 1.25, 0.8), W.dsv3(512),
            # token-heavy points of the stress sweep: the tiled-GEMM launches (taken by the rule) next to the
            # streaming launch on a list that wraps around
            W.stress(4096, 1.25, 0.8), W.stress(8192, 1.25, 0.8)]


@pytest.mark.parametrize("cfg", FFN_CFGS, ids=lambda c: f"{c.name}-T{c.T}")
def test_layer_parity(cfg):
    """route -> schedule -> permute -> grouped FFN -> combine for the straggler instance."""
    big = cfg.C * cfg.d_h * cfg.d_e > (1 << 26)
    orc = OracleRun(cfg, only_activated=big)      # big layers: unread slots hold NaN instead of weights
    print(f"  oracle ready: g_self={orc.g_self} n_local={len(orc.perm)} a_g={int((orc.slot_count > 0).sum())}", flush=True)
    step = LayerStep(cfg, orc.lay, orc.g_self)
    upload_weights(step, cfg, orc.W13, orc.W2)
    print("  weights uploaded", flush=True)
    # poison rows beyond n_local so that "left untouched" is visible
    step.Yp.fill_(123.0)
    Y = step.step(torch.from_numpy(orc.logits).cuda(), upload_x(cfg, orc.X))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(step.topk_ids.cpu().numpy(), orc.ids)
    np.testing.assert_array_equal(step.rid.cpu().numpy(), orc.O)
    np.testing.assert_array_equal(step.slot_off.cpu().numpy(), orc.slot_off)
    n_local = len(orc.perm)
    np.testing.assert_array_equal(step.perm.cpu().numpy()[:n_local], orc.perm)
    tol = TOL_BF16 if cfg.dtype == "bf16" else TOL_F32
    Yp = step.Yp.cpu().numpy()
    assert (Yp[n_local:] == 123.0).all()
    assert np.isfinite(Yp[:n_local]).all()
    e_yp = rel_fro(Yp[:n_local], orc.Yp)
    e_y = rel_fro(Y.float().cpu().numpy(), orc.Y)
    print(f"  rel Frobenius: Yp {e_yp:.3e}  Y {e_y:.3e}", flush=True)
    assert e_yp < tol and e_y < tol
    # row-wise as well, so a single wrong row cannot hide in the norm
    num = np.linalg.norm(Yp[:n_local] - orc.Yp, axis=1)
    den = np.linalg.norm(orc.Yp, axis=1)
    assert (num <= 2.5 * tol * den + 1e-30).all()
    # tokens without a local request are exactly zero
    no_local = (orc.O // cfg.C != orc.g_self).all(axis=1)
    assert not Y.float().cpu().numpy()[no_local].any()
    assert B.moe_workspace_status(step.workspace) == 0
    # a second step on the same buffers (counters were left cleared) gives the same bits
    Yp1 = step.Yp.clone()
    step.step(torch.from_numpy(orc.logits).cuda(), upload_x(cfg, orc.X))
    torch.cuda.synchronize()
    assert torch.equal(Yp1[:n_local], step.Yp[:n_local])
    assert B.moe_workspace_status(step.workspace) == 0


@pytest.mark.parametrize("cfg", [W.tiny(), W.dsv2lite(), W.qwen3(1024), W.dsv3(512), small("ragged", k=5, T=77),
                                 W.stress(8192, 1.25, 0.8), W.stress(2048, 1.125, 1.5), small("k1", k=1, T=1),
                                 small("many_slots", E=150, n_inst=2, C=80, k=4, T=200),
                                 # the chunked tail: more than 8192 requests (ragged last chunk, more than 64
                                 # slots), or a layout table too large for one workgroup's LDS
                                 small("chunks", E=150, n_inst=2, C=80, k=7, T=1300),
                                 small("big_table", E=1024, n_inst=16, C=70, k=8, T=20, zipf_s=0.0)],
                         ids=lambda c: f"{c.name}-T{c.T}")
def test_fused_front_equals_separate_calls(cfg):
    """moe_route_schedule_permute gives the bits of the three separate calls, call after call."""
    lay = W.build_placement(cfg)
    logits = torch.from_numpy(W.router_logits(cfg)).cuda()
    a = LayerStep(cfg, lay, cfg.n_inst - 1)
    b = LayerStep(cfg, lay, cfg.n_inst - 1)
    a.route(logits); a.schedule(); a.permute()
    for rep in range(3):
        for t in (b.topk_ids, b.rid, b.act_rep, b.load, b.slot_count, b.slot_off, b.perm, b.pos, b.blocks):
            t.fill_(-5)
        b.front(logits)
        torch.cuda.synchronize()
        n_local = int(a.slot_off[-1].item())
        for name in ("topk_ids", "topk_w", "rid", "act_rep", "load", "slot_count", "slot_off", "pos"):
            assert torch.equal(getattr(a, name), getattr(b, name)), (name, rep)
        assert torch.equal(a.perm[:n_local], b.perm[:n_local])
        n_blk = 4 * (1 + int(a.blocks[0].item()))
        assert torch.equal(a.blocks[:n_blk], b.blocks[:n_blk])
        assert int(b.sync[:33].abs().sum().item()) == 0


def test_all_instances_sum_to_dense_layer():
    """Tiny configuration: the instance partials of both instances add up to the dense
    per-token layer (replicas hold identical weights, so scheduling never changes the output)."""
    cfg = W.tiny()
    lay = W.build_placement(cfg)
    tot = np.zeros((cfg.T, cfg.d_h))
    orc0 = OracleRun(cfg, g_self=0, with_ffn=False)
    d_logits, d_X = torch.from_numpy(orc0.logits).cuda(), torch.from_numpy(orc0.X).cuda()
    for g in range(cfg.n_inst):
        step = LayerStep(cfg, lay, g)
        W13, W2 = W.instance_weights(cfg, lay, g)
        # slots that receive no request get NaN weights: they must never be read
        cnt, _, _ = dispatch.permute(orc0.O, g, cfg.C)
        W13[cnt == 0] = np.nan
        W2[cnt == 0] = np.nan
        upload_weights(step, cfg, W13, W2)
        tot += step.step(d_logits, d_X).float().cpu().numpy()
    dense = ffn.dense_layer(orc0.X, orc0.ids, orc0.w, lambda e: W.expert_weights(cfg, e))
    assert np.isfinite(tot).all()
    assert rel_fro(tot, dense) < TOL_F32


def test_unactivated_slots_are_not_read_bf16():
    cfg = small("nan_slots", T=6, E=16, n_inst=2, C=9)
    orc = OracleRun(cfg)
    W13, W2 = orc.W13.copy(), orc.W2.copy()
    W13[orc.slot_count == 0] = np.nan
    W2[orc.slot_count == 0] = np.nan
    assert (orc.slot_count == 0).any()
    step = LayerStep(cfg, orc.lay, orc.g_self)
    upload_weights(step, cfg, W13, W2)
    Y = step.step(torch.from_numpy(orc.logits).cuda(), upload_x(cfg, orc.X)).float().cpu().numpy()
    assert np.isfinite(Y).all() and rel_fro(Y, orc.Y) < TOL_BF16


@pytest.mark.parametrize("T", [70, 400], ids=["blocks32", "blocks64"])
@pytest.mark.parametrize("d_h,d_e", [(256, 192), (160, 96), (192, 160)], ids=["even-even", "odd-odd", "even-odd"])
def test_ffn_block_boundaries(d_h, d_e, T):
    """The grouped FFN alone on a hand-made dispatch whose slots hold 0, 1, 8, 9, 16, 17, 24, 25,
    32, 33, ... 65 rows (every number of 8-row halves, one and several blocks per slot, for blocks of
    32 and of 64 rows), for even and odd numbers of K-steps in either stage, against the oracle's
    grouped FFN.  A list cut for another block size is refused."""
    counts = [8, 9, 0, 16, 17, 24, 1, 25, 32, 33, 0, 65, 40, 41, 48, 49, 56, 57, 64]
    # slots with more than 64 requests can be computed as tiled GEMMs over blocks of 64 rows: one full
    # + 2 or 6 rows, exactly two, two + 1 row, several + a rest
    if T >= 400:
        counts += [66, 128, 129, 300]
    else:
        counts += [70, 130]
    C, k = len(counts), 12
    assert B.moe_block_rows(T) == (32 if T == 70 else 64)
    cfg = W.MoEConfig("blocks", E=C, k=k, d_h=d_h, d_e=d_e, T=T, n_inst=1, C=C, zipf_s=0.0, seed=11)
    rng = np.random.default_rng(3)
    slot_off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    n_local = int(slot_off[-1])
    perm = rng.permutation(T * k)[:n_local].astype(np.int32)
    X = W.activations(cfg)
    W13 = np.stack([W.expert_weights(cfg, e)[0] for e in range(C)])
    W2 = np.stack([W.expert_weights(cfg, e)[1] for e in range(C)])
    Yp_ref = ffn.grouped_ffn(X, W13, W2, slot_off, perm, k)
    blk = expected_blocks(slot_off, B.moe_block_rows(T))
    assert blk[0] <= B.moe_max_blocks(T, k, C)
    d_blk = torch.zeros((B.moe_block_list_len(T, k, C),), dtype=torch.int32)
    d_blk[:len(blk)] = torch.from_numpy(blk)
    d_blk = d_blk.cuda()
    W13p, W2p = torch.empty_like(to_device_bf16(W13)), torch.empty_like(to_device_bf16(W2))
    B.moe_pack_weights_bf16(to_device_bf16(W13), to_device_bf16(W2), C, d_h, d_e, W13p, W2p)
    ws = torch.empty((B.moe_workspace_bytes(T, k, C, d_h, d_e, B.MOE_DTYPE_BF16),), dtype=torch.uint8, device="cuda")
    B.moe_workspace_init(ws)
    Yp = torch.full((T * k, d_h), 123.0, dtype=torch.float32, device="cuda")
    for rep in range(3):
        # rep 1: the slots with more than 64 requests are computed as tiled-GEMM blocks even though this
        # batch has too few of them to fill the chip (the rule's threshold set to one workgroup)
        B.moe_workspace_set_option(ws, B.MOE_WS_OPT_WIDE_MIN_WORKGROUPS, 1 if rep == 1 else 0)
        Yp.fill_(123.0)
        B.moe_grouped_ffn(to_device_bf16(X), W13p, W2p, T, k, C, d_h, d_e, B.MOE_DTYPE_BF16,
                          torch.from_numpy(slot_off).cuda(), torch.from_numpy(perm).cuda(), d_blk, Yp, ws)
        torch.cuda.synchronize()
        got = Yp.cpu().numpy()
        assert (got[n_local:] == 123.0).all()
        num = np.linalg.norm(got[:n_local] - Yp_ref, axis=1)
        den = np.linalg.norm(Yp_ref, axis=1)
        assert (num <= 2.5 * TOL_BF16 * den + 1e-30).all(), (rep, int(np.argmax(num / den)))
        assert rel_fro(got[:n_local], Yp_ref) < TOL_BF16
        assert B.moe_workspace_status(ws) == 0
    # the same list with the other block size in its header: nothing is computed, bit 1 of the status
    d_blk[1] = 96 - B.moe_block_rows(T)
    Yp.fill_(123.0)
    B.moe_grouped_ffn(to_device_bf16(X), W13p, W2p, T, k, C, d_h, d_e, B.MOE_DTYPE_BF16,
                      torch.from_numpy(slot_off).cuda(), torch.from_numpy(perm).cuda(), d_blk, Yp, ws)
    torch.cuda.synchronize()
    assert (Yp == 123.0).all() and B.moe_workspace_status(ws) == 2
    B.moe_workspace_init(ws)
    assert B.moe_workspace_status(ws) == 0


@pytest.mark.parametrize("seed", range(6))
def test_ffn_random_dispatches_with_and_without_wide_blocks(seed):
    """The grouped FFN alone on randomly drawn hand-made dispatches (empty, light, 33-64-row and
    100-300-row slots mixed; channel counts that give more than eight groups of tiles per block and
    tile counts that are no multiple of eight; both block sizes), with the tiled-GEMM blocks taken by
    the default rule and forced on, against the oracle's grouped FFN."""
    rng = np.random.default_rng([77, seed])
    T = int(rng.choice([70, 200, 400, 600]))
    d_h = int(rng.choice([128, 320]))
    d_e = int(rng.choice([96, 608, 1088]))
    C, k = int(rng.integers(5, 12)), 8
    kinds = rng.integers(0, 5, size=C)
    counts = [int({0: 0, 1: rng.integers(1, 17), 2: rng.integers(17, 33), 3: rng.integers(33, 65),
                   4: rng.integers(65, 301)}[int(c)]) for c in kinds]
    counts[int(rng.integers(0, C))] = int(rng.integers(65, 301))        # at least one slot with several blocks
    while sum(counts) > T * k:
        counts[int(np.argmax(counts))] //= 2
    cfg = W.MoEConfig("random_blocks", E=C, k=k, d_h=d_h, d_e=d_e, T=T, n_inst=1, C=C, zipf_s=0.0, seed=100 + seed)
    slot_off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    n_local = int(slot_off[-1])
    perm = rng.permutation(T * k)[:n_local].astype(np.int32)
    X = W.activations(cfg)
    W13 = np.stack([W.expert_weights(cfg, e)[0] for e in range(C)])
    W2 = np.stack([W.expert_weights(cfg, e)[1] for e in range(C)])
    Yp_ref = ffn.grouped_ffn(X, W13, W2, slot_off, perm, k)
    blk = expected_blocks(slot_off, B.moe_block_rows(T))
    assert blk[0] <= B.moe_max_blocks(T, k, C)
    d_blk = torch.zeros((B.moe_block_list_len(T, k, C),), dtype=torch.int32)
    d_blk[:len(blk)] = torch.from_numpy(blk)
    d_blk = d_blk.cuda()
    W13p, W2p = torch.empty_like(to_device_bf16(W13)), torch.empty_like(to_device_bf16(W2))
    B.moe_pack_weights_bf16(to_device_bf16(W13), to_device_bf16(W2), C, d_h, d_e, W13p, W2p)
    ws = torch.empty((B.moe_workspace_bytes(T, k, C, d_h, d_e, B.MOE_DTYPE_BF16),), dtype=torch.uint8, device="cuda")
    B.moe_workspace_init(ws)
    Yp = torch.full((T * k, d_h), 123.0, dtype=torch.float32, device="cuda")
    for forced in (0, 1, 0):
        B.moe_workspace_set_option(ws, B.MOE_WS_OPT_WIDE_MIN_WORKGROUPS, forced)
        Yp.fill_(123.0)
        B.moe_grouped_ffn(to_device_bf16(X), W13p, W2p, T, k, C, d_h, d_e, B.MOE_DTYPE_BF16,
                          torch.from_numpy(slot_off).cuda(), torch.from_numpy(perm).cuda(), d_blk, Yp, ws)
        torch.cuda.synchronize()
        got = Yp.cpu().numpy()
        assert (got[n_local:] == 123.0).all(), (counts, forced)
        num = np.linalg.norm(got[:n_local] - Yp_ref, axis=1)
        den = np.linalg.norm(Yp_ref, axis=1)
        assert (num <= 2.5 * TOL_BF16 * den + 1e-30).all(), (counts, forced, int(np.argmax(num / den)))
        assert B.moe_workspace_status(ws) == 0


def test_ffn_rejects_small_workspace():
    cfg = small()
    step = LayerStep(cfg, W.build_placement(cfg), 0)
    with pytest.raises(B.MoeError) as ei:
        B.moe_grouped_ffn(step.Y, step.Y, step.Y, cfg.T, cfg.k, cfg.C, cfg.d_h, cfg.d_e, step.dtype,
                          step.slot_off, step.perm, step.blocks, step.Yp, step.workspace[:256])
    assert ei.value.code == B.MOE_EWORKSPACE


# ----------------------------------------------------------------------------- gate + selection
# The gate sums d_h fp32 products in an order of its own, so a logit differs from the oracle's
# (fp64, rounded once) by up to ~sqrt(d_h) * 2^-24 * |terms| ~ 5e-6 at d_h = 7168; the test allows
# GATE_ATOL.  A selection is compared bit for bit wherever the oracle's decision margin exceeds
# GATE_MARGIN (both neighbours may move by GATE_ATOL each); closer calls must still be a valid
# selection within that tolerance.
GATE_ATOL = 2e-5
GATE_MARGIN = 1e-4


def as_bf16(cfg, **kw):
    import dataclasses
    return dataclasses.replace(cfg, dtype="bf16", **kw)


def gate_oracle(cfg):
    from oracle import gating
    X = W.activations(cfg)
    Wr, bias = W.router_weights(cfg)
    z64 = gating.gate_logits(X, Wr, bias)
    z32 = z64.astype(np.float32)
    ids, w, info = oracle_route(cfg, z32)
    if info is None:
        sure = gating.selection_margin(z64, cfg.k) > GATE_MARGIN
    else:
        per = cfg.E // cfg.n_group
        kept = np.zeros((cfg.T, cfg.n_group), dtype=bool)
        np.put_along_axis(kept, info["kept_groups"], True, axis=1)
        masked = np.where(np.repeat(kept, per, axis=1), z64, -1e30)
        sure = (info["group_margin"] > GATE_MARGIN) & (gating.selection_margin(masked, cfg.k) > GATE_MARGIN)
    return X, Wr, bias, z64, ids, w, sure


def route_kwargs(cfg):
    if cfg.route == "softmax":
        return dict(mode=B.MOE_ROUTE_SOFTMAX)
    return dict(mode=B.MOE_ROUTE_SIGMOID_GROUP, n_group=cfg.n_group, topk_group=cfg.topk_group)


def check_selection(cfg, z64, ids, w, sure, g_ids, g_w):
    np.testing.assert_array_equal(g_ids[sure], ids[sure])
    np.testing.assert_allclose(g_w[sure], w[sure], rtol=2e-4)
    kth = -np.sort(-z64, axis=1)[:, cfg.k - 1]
    for i in np.nonzero(~sure)[0]:
        assert len(set(g_ids[i].tolist())) == cfg.k
        if cfg.route == "softmax":
            assert (z64[i, g_ids[i]] >= kth[i] - GATE_MARGIN).all()
        else:
            assert len(set((g_ids[i] // (cfg.E // cfg.n_group)).tolist())) <= cfg.topk_group
    np.testing.assert_allclose(g_w.sum(axis=1), 1.0, rtol=1e-5)


GATE_CFGS = [as_bf16(W.tiny()), W.dsv2lite(), W.qwen3(256), W.dsv3(512), W.stress(1024, 1.25, 0.8),
             small("odd", E=70, k=5, T=3), small("ragged", E=40, d_h=160, T=37), small("k1", k=1, T=1),
             small("e1024", E=1024, k=32, T=9, d_h=96, zipf_s=0.0)]


@pytest.mark.parametrize("cfg", GATE_CFGS, ids=lambda c: f"{c.name}-T{c.T}")
def test_gate_route_parity(cfg):
    X, Wr, bias, z64, ids, w, sure = gate_oracle(cfg)
    assert sure.mean() > 0.6
    d_X, d_Wr = to_device_bf16(X), to_device_bf16(Wr)
    d_bias = None if bias is None else torch.from_numpy(bias).cuda()
    sync = torch.zeros(B.moe_gate_sync_len(cfg.T), dtype=torch.int32, device="cuda")
    for rep in range(2):                                   # the second call finds the tickets cleared
        d_z = torch.full((cfg.T, cfg.E), float("nan"), dtype=torch.float32, device="cuda")
        d_ids = torch.full((cfg.T, cfg.k), -7, dtype=torch.int32, device="cuda")
        d_w = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
        B.moe_gate_route(d_X, d_Wr, d_bias, cfg.k, d_z, d_ids, d_w, sync, **route_kwargs(cfg))
        torch.cuda.synchronize()
        np.testing.assert_allclose(d_z.cpu().numpy(), z64, rtol=0, atol=GATE_ATOL)
        check_selection(cfg, z64, ids, w, sure, d_ids.cpu().numpy(), d_w.cpu().numpy())
        assert int(sync.abs().sum().item()) == 0


def all_sure_variant(cfg):
    """First seed from cfg.seed on for which every token's selection is decided by more than the
    margin (found with the oracle alone), so that every integer result downstream is unique."""
    for seed in range(cfg.seed, cfg.seed + 200):
        c = as_bf16(cfg, seed=seed)
        out = gate_oracle(c)
        if out[-1].all():
            return c, out
    raise AssertionError("no seed with clear margins")


FRONT_GATE_CFGS = [as_bf16(W.tiny()), W.dsv2lite(64), W.qwen3(32), W.dsv3(16), small("ragged", E=40, d_h=160, k=5, T=77, n_inst=4, C=12),
                   small("k1", k=1, T=1)]


@pytest.mark.parametrize("cfg", FRONT_GATE_CFGS, ids=lambda c: f"{c.name}-T{c.T}")
def test_gate_front_parity(cfg):
    """X, W_r -> everything a0-a4 produce, in one launch, against the oracle chain."""
    cfg, (X, Wr, bias, z64, ids, w, sure) = all_sure_variant(cfg)
    lay = W.build_placement(cfg)
    pl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    O, act_rep, load = scheduling.aebs(ids, pl)
    g_self = int(np.argmax(load))
    slot_count, slot_off, perm = dispatch.permute(O, g_self, cfg.C)
    pos = np.full(cfg.T * cfg.k, -1, dtype=np.int32)
    pos[perm] = np.arange(len(perm), dtype=np.int32)
    s = LayerStep(cfg, lay, g_self)
    d_X, d_Wr = to_device_bf16(X), to_device_bf16(Wr)
    d_bias = None if bias is None else torch.from_numpy(bias).cuda()
    for rep in range(2):
        for t in (s.topk_ids, s.rid, s.act_rep, s.load, s.slot_count, s.slot_off, s.perm, s.pos, s.blocks):
            t.fill_(-5)
        d_z = s.front_gate(d_X, d_Wr, d_bias)
        torch.cuda.synchronize()
        np.testing.assert_allclose(d_z.cpu().numpy(), z64, rtol=0, atol=GATE_ATOL)
        np.testing.assert_array_equal(s.topk_ids.cpu().numpy(), ids)
        np.testing.assert_allclose(s.topk_w.cpu().numpy(), w, rtol=2e-4)
        np.testing.assert_array_equal(s.rid.cpu().numpy().reshape(cfg.T, cfg.k), O)
        np.testing.assert_array_equal(s.act_rep.cpu().numpy(), act_rep)
        np.testing.assert_array_equal(s.load.cpu().numpy(), load)
        np.testing.assert_array_equal(s.slot_count.cpu().numpy(), slot_count)
        np.testing.assert_array_equal(s.slot_off.cpu().numpy(), slot_off)
        np.testing.assert_array_equal(s.perm.cpu().numpy()[:len(perm)], perm)
        np.testing.assert_array_equal(s.pos.cpu().numpy(), pos)
        exp = expected_blocks(slot_off, B.moe_block_rows(cfg.T))
        np.testing.assert_array_equal(s.blocks.cpu().numpy()[:len(exp)], exp)
        assert int(s.gate_sync.abs().sum().item()) == 0


@pytest.mark.parametrize("cfg", [W.dsv2lite(), W.qwen3(1024), W.dsv3(512), W.stress(8192, 1.25, 0.8)],
                         ids=lambda c: f"{c.name}-T{c.T}")
def test_gate_front_full_size_is_consistent(cfg):
    """At full size some selections are closer than the gate's rounding, so the chain is checked
    in two halves: logits and selection against the oracle (margin-aware), and Alg. 1 + dispatch
    bit for bit against the separately verified entry points run on the ids the launch chose."""
    X, Wr, bias, z64, ids, w, sure = gate_oracle(cfg)
    lay = W.build_placement(cfg)
    a = LayerStep(cfg, lay, cfg.n_inst - 1)
    b = LayerStep(cfg, lay, cfg.n_inst - 1)
    d_X, d_Wr = to_device_bf16(X), to_device_bf16(Wr)
    d_bias = None if bias is None else torch.from_numpy(bias).cuda()
    d_z = b.front_gate(d_X, d_Wr, d_bias)
    torch.cuda.synchronize()
    np.testing.assert_allclose(d_z.cpu().numpy(), z64, rtol=0, atol=GATE_ATOL)
    check_selection(cfg, z64, ids, w, sure, b.topk_ids.cpu().numpy(), b.topk_w.cpu().numpy())
    a.topk_ids.copy_(b.topk_ids)
    a.schedule(); a.permute()
    torch.cuda.synchronize()
    n_local = int(a.slot_off[-1].item())
    for name in ("rid", "act_rep", "load", "slot_count", "slot_off", "pos"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    assert torch.equal(a.perm[:n_local], b.perm[:n_local])
    n_blk = 4 * (1 + int(a.blocks[0].item()))
    assert torch.equal(a.blocks[:n_blk], b.blocks[:n_blk])


def test_schedule_over_the_alg3_layout():
    """The layout that Appendix B's rules build from a window of routed batches is a valid
    layout for the library, and Alg. 1 over it matches the oracle bit for bit."""
    from oracle import placement_opt, routing
    cfg = W.MoEConfig("alg3", E=64, k=6, d_h=64, d_e=64, T=48, n_inst=4, C=20, zipf_s=1.0, seed=3)
    tb = W.topic_bias(cfg, 4, 2.0, True)
    rng = np.random.default_rng(9)
    window = []
    for b in range(40):
        z = rng.standard_normal((cfg.T, cfg.E)).astype(np.float32) + tb[b % 4]
        window.append(routing.route_softmax(z, cfg.k)[0])
    window = np.stack(window)
    c, a = placement_opt.coactivation_counts(window, cfg.E)
    R = placement_opt.replica_counts(c, cfg.n_inst, cfg.C)
    lay = placement_opt.place_replicas(cfg.n_inst, cfg.C, R, c, a)
    np.testing.assert_array_equal(B.moe_place_replicas(cfg.n_inst, cfg.C, R, c, a), lay)
    opl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    pl = B.Placement(lay, cfg.E, cfg.n_inst, cfg.C)
    rid = torch.empty((cfg.T, cfg.k), dtype=torch.int32, device="cuda")
    rep = torch.empty((cfg.E,), dtype=torch.int32, device="cuda")
    load = torch.empty((cfg.n_inst,), dtype=torch.int32, device="cuda")
    for b in range(40, 48):
        z = rng.standard_normal((cfg.T, cfg.E)).astype(np.float32) + tb[b % 4]
        ids = routing.route_softmax(z, cfg.k)[0]
        O, act_rep, ld = scheduling.aebs(ids, opl)
        B.moe_schedule(pl, dev_i32(ids), cfg.T, cfg.k, rid, rep, load)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(rid.cpu().numpy(), O)
        np.testing.assert_array_equal(rep.cpu().numpy(), act_rep)
        np.testing.assert_array_equal(load.cpu().numpy(), ld)


@pytest.mark.parametrize("cfg,d_s", [(W.dsv2lite(), 2816), (small("ragged", k=5, T=77), 160), (W.tiny(), 512),
                                     (small("k1", k=1, T=1), 96), (W.qwen3(1024), 768)],
                         ids=lambda v: f"{v.name}-T{v.T}" if hasattr(v, "name") else str(v))
def test_layer_with_shared_expert(cfg, d_s):
    """Routed layer plus a shared expert over all tokens (several blocks of rows on one slot),
    against the oracle; the dispatch of the shared slot is checked bit for bit."""
    o = OracleRun(cfg)
    ws13, ws2 = W.shared_expert_weights(cfg, d_s)
    want = ffn.add_shared_expert(o.Y, o.X, ws13, ws2)
    s = LayerStep(cfg, o.lay, o.g_self)
    upload_weights(s, cfg, o.W13, o.W2)
    if cfg.dtype == "bf16":
        s.enable_shared(to_device_bf16(ws13), to_device_bf16(ws2))
    else:
        s.enable_shared(torch.from_numpy(ws13).cuda(), torch.from_numpy(ws2).cuda())
    torch.cuda.synchronize()
    assert s.s_slot_off.cpu().tolist() == [0, cfg.T]
    np.testing.assert_array_equal(s.s_perm.cpu().numpy()[:cfg.T], np.arange(cfg.T))
    exp = expected_blocks(np.array([0, cfg.T]), B.moe_block_rows(cfg.T))
    np.testing.assert_array_equal(s.s_blocks.cpu().numpy()[:len(exp)], exp)
    X = upload_x(cfg, o.X)
    logits = torch.from_numpy(o.logits).cuda()
    for rep in range(2):
        s.Y.zero_()
        s.step_fused_shared(logits, X)
        torch.cuda.synchronize()
        got = s.Y.float().cpu().numpy()
        tol = TOL_BF16 if cfg.dtype == "bf16" else TOL_F32
        assert rel_fro(got, want) < tol
        assert rel_fro(s.s_Yp.cpu().numpy(), ffn.expert_ffn(o.X, ws13, ws2)) < tol
        assert B.moe_workspace_status(s.workspace) == 0 and B.moe_workspace_status(s.s_workspace) == 0


def test_steps_replayed_from_a_hip_graph_match_eager():
    """The entry points neither allocate nor synchronise, so a layer step can be captured; every
    replay must reproduce the eager result bit for bit, with eager work in between."""
    cfg = W.dsv2lite()
    o = OracleRun(cfg)
    s = LayerStep(cfg, o.lay, o.g_self)
    upload_weights(s, cfg, o.W13, o.W2)
    X = upload_x(cfg, o.X)
    logits = torch.from_numpy(o.logits).cuda()
    other_logits = torch.from_numpy(W.router_logits(cfg, sub=3)).cuda()
    other_X = upload_x(cfg, W.activations(cfg, sub=3))
    s.step_fused(logits, X)
    torch.cuda.synchronize()
    assert rel_fro(s.Y.float().cpu().numpy(), o.Y) < TOL_BF16
    keep = {n: getattr(s, n).clone() for n in ("Y", "topk_ids", "rid", "load", "slot_off", "pos")}
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        s.step_fused(logits, X)
    torch.cuda.synchronize()
    for rep in range(4):
        s.step_fused(other_logits, other_X)                  # eager work on the same buffers in between
        torch.cuda.synchronize()
        assert not torch.equal(s.topk_ids, keep["topk_ids"])
        g.replay()
        torch.cuda.synchronize()
        for n, t in keep.items():
            assert torch.equal(getattr(s, n), t), (n, rep)
        assert B.moe_workspace_status(s.workspace) == 0


@pytest.mark.parametrize("cfg", [W.qwen3(1024), W.stress(2048, 1.25, 0.8), W.dsv3(512)], ids=lambda c: f"{c.name}-T{c.T}")
def test_layer_parity_with_wide_blocks_forced_on(cfg):
    """Full-size layers whose hottest slots hold more than 64 requests, with those slots computed as
    tiled-GEMM blocks (forced on: these batches have too few such blocks for the rule; blocks of 64
    rows, and of 128 rows in the launch for batches of at least 2048 tokens)."""
    orc = OracleRun(cfg, only_activated=True)
    assert (orc.slot_count > 64).any()
    step = LayerStep(cfg, orc.lay, orc.g_self)
    upload_weights(step, cfg, orc.W13, orc.W2)
    step.Yp.fill_(123.0)
    n_local = len(orc.perm)
    B.moe_workspace_set_option(step.workspace, B.MOE_WS_OPT_WIDE_MIN_WORKGROUPS, 1)
    for rep in range(2):
        Y = step.step_fused(torch.from_numpy(orc.logits).cuda(), upload_x(cfg, orc.X))
        torch.cuda.synchronize()
        Yp = step.Yp.cpu().numpy()
        assert (Yp[n_local:] == 123.0).all() and np.isfinite(Yp[:n_local]).all()
        num = np.linalg.norm(Yp[:n_local] - orc.Yp, axis=1)
        den = np.linalg.norm(orc.Yp, axis=1)
        assert (num <= 2.5 * TOL_BF16 * den + 1e-30).all()
        assert rel_fro(Yp[:n_local], orc.Yp) < TOL_BF16
        assert rel_fro(Y.float().cpu().numpy(), orc.Y) < TOL_BF16
        assert B.moe_workspace_status(step.workspace) == 0
    B.moe_workspace_set_option(step.workspace, B.MOE_WS_OPT_WIDE_MIN_WORKGROUPS, 0)


def test_token_heavy_batch_all_slots_wide():
    """Every slot of the instance holds 361 or 362 requests (config 2's shape, T = 1024): all slots are
    computed as tiled GEMMs over blocks of 64 rows (five full blocks and a partly filled one each).
    Dispatch through moe_permute, rows against the oracle's grouped FFN."""
    cfg = W.dsv2lite(1024)
    T, k, C = cfg.T, cfg.k, cfg.C
    lay = W.build_placement(cfg)
    g_self = 1
    rid = (g_self * C + np.arange(T * k, dtype=np.int32) % C).reshape(T, k)
    slot_count, slot_off, perm = dispatch.permute(rid, g_self, C)
    assert slot_count.min() > 64
    X = W.activations(cfg)
    W13, W2 = W.instance_weights(cfg, lay, g_self)
    Yp_ref = ffn.grouped_ffn(X, W13, W2, slot_off, perm, k)
    s = LayerStep(cfg, lay, g_self)
    upload_weights(s, cfg, W13, W2)
    s.rid.copy_(torch.from_numpy(rid))
    s.Yp.fill_(123.0)
    for rep in range(2):
        s.permute()
        s.ffn(upload_x(cfg, X))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(s.slot_off.cpu().numpy(), slot_off)
        blk = s.blocks.cpu().numpy()
        exp = expected_blocks(slot_off, 64)
        np.testing.assert_array_equal(blk[:len(exp)], exp)
        got = s.Yp.cpu().numpy()
        n_local = int(slot_off[-1])
        assert n_local == T * k
        num = np.linalg.norm(got - Yp_ref, axis=1)
        den = np.linalg.norm(Yp_ref, axis=1)
        assert (num <= 2.5 * TOL_BF16 * den + 1e-30).all()
        assert rel_fro(got, Yp_ref) < TOL_BF16
        assert B.moe_workspace_status(s.workspace) == 0


def test_ffn_long_block_list_wraps_around():
    """More blocks than get workgroups of their own (128): the workgroups of the first 128 blocks
    also take blocks 128 further on, in both stages, and a second call finds the counters cleared."""
    T, k, C, d_h, d_e = 400, 32, 150, 64, 96
    counts = [(65, 65, 64, 130, 17, 66)[s % 6] for s in range(C)]
    cfg = W.MoEConfig("wrap", E=C, k=k, d_h=d_h, d_e=d_e, T=T, n_inst=1, C=C, zipf_s=0.0, seed=13)
    rng = np.random.default_rng(4)
    slot_off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    n_local = int(slot_off[-1])
    assert n_local <= T * k
    perm = rng.permutation(T * k)[:n_local].astype(np.int32)
    X = W.activations(cfg)
    W13 = np.stack([W.expert_weights(cfg, e)[0] for e in range(C)])
    W2 = np.stack([W.expert_weights(cfg, e)[1] for e in range(C)])
    Yp_ref = ffn.grouped_ffn(X, W13, W2, slot_off, perm, k)
    blk = expected_blocks(slot_off, 64)
    assert 128 * 2 < blk[0] <= B.moe_max_blocks(T, k, C)
    d_blk = torch.zeros((B.moe_block_list_len(T, k, C),), dtype=torch.int32)
    d_blk[:len(blk)] = torch.from_numpy(blk)
    d_blk = d_blk.cuda()
    W13p, W2p = torch.empty_like(to_device_bf16(W13)), torch.empty_like(to_device_bf16(W2))
    B.moe_pack_weights_bf16(to_device_bf16(W13), to_device_bf16(W2), C, d_h, d_e, W13p, W2p)
    ws = torch.empty((B.moe_workspace_bytes(T, k, C, d_h, d_e, B.MOE_DTYPE_BF16),), dtype=torch.uint8, device="cuda")
    B.moe_workspace_init(ws)
    Yp = torch.full((T * k, d_h), 123.0, dtype=torch.float32, device="cuda")
    for rep in range(4):
        # reps 2 and 3: the slots with more than 64 requests as tiled-GEMM blocks
        B.moe_workspace_set_option(ws, B.MOE_WS_OPT_WIDE_MIN_WORKGROUPS, 1 if rep >= 2 else 100000)
        Yp.fill_(123.0)
        B.moe_grouped_ffn(to_device_bf16(X), W13p, W2p, T, k, C, d_h, d_e, B.MOE_DTYPE_BF16,
                          torch.from_numpy(slot_off).cuda(), torch.from_numpy(perm).cuda(), d_blk, Yp, ws)
        torch.cuda.synchronize()
        got = Yp.cpu().numpy()
        assert (got[n_local:] == 123.0).all()
        num = np.linalg.norm(got[:n_local] - Yp_ref, axis=1)
        den = np.linalg.norm(Yp_ref, axis=1)
        assert (num <= 2.5 * TOL_BF16 * den + 1e-30).all(), (rep, int(np.argmax(num / den)))
        assert B.moe_workspace_status(ws) == 0


def random_cfg(seed):
    """A small layer with randomly drawn shape parameters (seeded): odd token counts, expert counts
    that are not powers of two, both parities of the K-step counts, with and without spare slots."""
    r = np.random.default_rng(1000 + seed)
    n_inst = int(r.integers(1, 6))
    per = int(r.integers(1, 9))
    E = n_inst * per
    C = per + int(r.integers(0, 4))
    k = int(r.integers(1, min(E, 8) + 1))
    return W.MoEConfig(f"rand{seed}", E=E, k=k, d_h=32 * int(r.integers(1, 9)), d_e=32 * int(r.integers(1, 7)),
                       T=int(r.integers(1, 200)), n_inst=n_inst, C=C, zipf_s=float(r.choice([0.0, 0.8, 1.5])), seed=seed)


@pytest.mark.parametrize("seed", range(16))
def test_layer_parity_random_shapes(seed):
    cfg = random_cfg(seed)
    orc = OracleRun(cfg)
    for g_self in sorted({orc.g_self, 0, cfg.n_inst - 1}):
        o = orc if g_self == orc.g_self else OracleRun(cfg, g_self=g_self)
        step = LayerStep(cfg, o.lay, g_self)
        upload_weights(step, cfg, o.W13, o.W2)
        Y = step.step_fused(torch.from_numpy(o.logits).cuda(), upload_x(cfg, o.X))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(step.topk_ids.cpu().numpy(), o.ids)
        np.testing.assert_array_equal(step.rid.cpu().numpy(), o.O)
        np.testing.assert_array_equal(step.act_rep.cpu().numpy(), o.act_rep)
        np.testing.assert_array_equal(step.load.cpu().numpy(), o.load)
        np.testing.assert_array_equal(step.slot_off.cpu().numpy(), o.slot_off)
        n_local = len(o.perm)
        np.testing.assert_array_equal(step.perm.cpu().numpy()[:n_local], o.perm)
        np.testing.assert_array_equal(step.pos.cpu().numpy(), o.pos)
        if n_local:
            assert rel_fro(step.Yp.cpu().numpy()[:n_local], o.Yp) < TOL_BF16
            assert rel_fro(Y.float().cpu().numpy(), o.Y) < TOL_BF16
        else:
            assert not Y.float().cpu().numpy().any()
        assert B.moe_workspace_status(step.workspace) == 0


@pytest.mark.parametrize("a", [1, 2, 17])
def test_ffn_all_requests_on_a_slots(a):
    """The shape of the activated-expert sweep (Sec. 2.2: a fixed batch of 64 tokens whose T*k requests
    all land on exactly `a` experts of the instance, evenly): dispatch through moe_permute, rows
    against the oracle's grouped FFN.  With a < k a token names one slot several times."""
    cfg = W.dsv2lite(64)
    T, k, C = cfg.T, cfg.k, cfg.C
    lay = W.build_placement(cfg)
    rid = (np.arange(T * k, dtype=np.int32) % a).reshape(T, k)
    slot_count, slot_off, perm = dispatch.permute(rid, 0, C)
    assert (slot_count > 0).sum() == a and slot_count.sum() == T * k
    X = W.activations(cfg)
    W13 = np.full((C, 2 * cfg.d_e, cfg.d_h), np.nan, dtype=np.float32)
    W2 = np.full((C, cfg.d_h, cfg.d_e), np.nan, dtype=np.float32)
    for s_ in range(a):
        W13[s_], W2[s_] = W.expert_weights(cfg, int(lay[s_]))
    Yp_ref = ffn.grouped_ffn(X, W13, W2, slot_off, perm, k)
    st = LayerStep(cfg, lay, 0)
    upload_weights(st, cfg, W13, W2)
    st.rid.copy_(torch.from_numpy(rid))
    st.Yp.fill_(123.0)
    for rep in range(2):
        # second round: the slots with more than 64 requests as tiled-GEMM blocks
        B.moe_workspace_set_option(st.workspace, B.MOE_WS_OPT_WIDE_MIN_WORKGROUPS, rep)
        st.permute()
        st.ffn(upload_x(cfg, X))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(st.slot_off.cpu().numpy(), slot_off)
        np.testing.assert_array_equal(st.perm.cpu().numpy(), perm)
        blk = st.blocks.cpu().numpy()
        exp = expected_blocks(slot_off, B.moe_block_rows(T))
        assert exp[0] <= B.moe_max_blocks(T, k, C)
        np.testing.assert_array_equal(blk[:len(exp)], exp)
        got = st.Yp.cpu().numpy()
        num = np.linalg.norm(got - Yp_ref, axis=1)
        den = np.linalg.norm(Yp_ref, axis=1)
        assert (num <= 2.5 * TOL_BF16 * den + 1e-30).all()
        assert rel_fro(got, Yp_ref) < TOL_BF16
        assert B.moe_workspace_status(st.workspace) == 0


def test_ffn_wait_overrun_is_loud():
    """A second-stage workgroup whose block never becomes ready gives up after the workspace's spin
    limit: status bit 0, NaN rows for that block and nothing else touched; every kernel exits
    normally.  The condition is forced from the host: the block's first-stage counter is pre-loaded
    so that no workgroup completes the count, and the spin limit is a few thousand polls.  After
    moe_workspace_init the same call gives the bits of a clean run."""
    cfg = small("overrun", T=90, E=12, k=4, n_inst=2, C=8, d_h=128, d_e=96, zipf_s=1.2)
    orc = OracleRun(cfg)
    st = LayerStep(cfg, orc.lay, orc.g_self)
    upload_weights(st, cfg, orc.W13, orc.W2)
    logits, X = torch.from_numpy(orc.logits).cuda(), upload_x(cfg, orc.X)
    st.step_fused(logits, X)
    torch.cuda.synchronize()
    n_local = len(orc.perm)
    clean_Yp, clean_Y = st.Yp[:n_local].clone(), st.Y.clone()
    assert rel_fro(clean_Yp.cpu().numpy(), orc.Yp) < TOL_BF16 and B.moe_workspace_status(st.workspace) == 0
    blk = st.blocks.cpu().numpy().reshape(-1, 4)
    n_blocks, R = int(blk[0, 0]), int(blk[0, 1])
    assert n_blocks >= 3
    # the victim: the second entry of the list.  This batch has too few slots with more than 64 requests
    # for tiled-GEMM blocks, so every entry is a streaming block of its own
    assert int(blk[0, 2]) * -(-cfg.d_e // 64) < 64
    victim = 1
    _, r0, hi, lo = (int(v) for v in blk[1 + victim])
    rows = np.arange(r0, min(hi, r0 + R))
    ctrl = st.workspace.view(torch.int32)
    ctrl[(victim + 1) * 256] = 1000                          # the block's first-stage counter: never completes
    # long enough for the other blocks' first stage to finish (microseconds), short enough for a test:
    # a few milliseconds of polling instead of the default's second
    B.moe_workspace_set_option(st.workspace, B.MOE_WS_OPT_SPIN_LIMIT, 5000)
    st.Yp.fill_(123.0)
    st.ffn(X)
    st.combine()
    torch.cuda.synchronize()
    assert B.moe_workspace_status(st.workspace) == 1
    got = st.Yp[:n_local].cpu().numpy()
    assert np.isnan(got[rows]).all()
    others = np.setdiff1d(np.arange(n_local), rows)
    np.testing.assert_array_equal(got[others], clean_Yp.cpu().numpy()[others])
    assert (st.Yp[n_local:] == 123.0).all()
    # tokens with a request in the block carry the NaN into Y; the others are unchanged
    tok = np.unique(orc.perm[rows] // cfg.k)
    Y = st.Y.float().cpu().numpy()
    assert np.isnan(Y[tok]).all(axis=1).all()
    rest = np.setdiff1d(np.arange(cfg.T), tok)
    np.testing.assert_array_equal(Y[rest], clean_Y.float().cpu().numpy()[rest])
    # recovery
    B.moe_workspace_init(st.workspace)
    assert B.moe_workspace_status(st.workspace) == 0
    st.step_fused(logits, X)
    torch.cuda.synchronize()
    assert torch.equal(st.Yp[:n_local], clean_Yp) and torch.equal(st.Y, clean_Y)
    assert B.moe_workspace_status(st.workspace) == 0
    assert int(ctrl[2].item()) == 0                          # the option was reset with the region


def test_permute_tolerates_repeated_slots_and_foreign_ids():
    """rid is caller-supplied: every choice of every token on ONE slot (more than T requests on it),
    the rest anywhere; the list stays within moe_max_blocks and the FFN computes every row."""
    cfg = small("dups", T=50, E=6, k=5, n_inst=2, C=4, d_h=64, d_e=64)
    T, k, C = cfg.T, cfg.k, cfg.C
    lay = W.build_placement(cfg)
    rid = np.full((T, k), C + 2, dtype=np.int32)            # instance 1, slot 2
    rid[::7, 0] = 10 ** 6                                    # not a replica id of any instance
    rid[::5, 1] = -3
    slot_count, slot_off, perm = dispatch.permute(rid, 1, C)
    assert slot_count.max() > T
    st = LayerStep(cfg, lay, 1)
    W13, W2 = W.instance_weights(cfg, lay, 1)
    upload_weights(st, cfg, W13, W2)
    st.rid.copy_(torch.from_numpy(rid))
    st.blocks.fill_(-9)
    st.permute()
    X = W.activations(cfg)
    st.ffn(upload_x(cfg, X))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(st.slot_off.cpu().numpy(), slot_off)
    np.testing.assert_array_equal(st.perm.cpu().numpy()[:len(perm)], perm)
    exp = expected_blocks(slot_off, B.moe_block_rows(T))
    assert exp[0] <= B.moe_max_blocks(T, k, C)
    blk = st.blocks.cpu().numpy()
    np.testing.assert_array_equal(blk[:len(exp)], exp)
    assert (blk[len(exp):] == -9).all()
    ref = ffn.grouped_ffn(X, W13, W2, slot_off, perm, k)
    assert rel_fro(st.Yp.cpu().numpy()[:len(perm)], ref) < TOL_BF16
    assert B.moe_workspace_status(st.workspace) == 0


@pytest.mark.parametrize("cfg,N", [(W.stress(64, 1.25, 0.8), 40), (small("ragged", k=5, T=77), 9), (W.dsv2lite(128), 12),
                                   (W.stress(1024, 1.125, 1.5), 5)], ids=lambda v: f"{v.name}-T{v.T}" if hasattr(v, "name") else f"N{v}")
def test_schedule_batched_parity(cfg, N):
    """moe_schedule_batched / moe_schedule_baseline_batched: N sampled batches in one launch, every
    batch bit for bit what the oracle's Alg. 1 (and the two baseline policies) give for it, with and
    without the optional outputs."""
    lay = W.build_placement(cfg)
    opl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
    pl = B.Placement(lay, cfg.E, cfg.n_inst, cfg.C)
    T, k = cfg.T, cfg.k
    ids = np.stack([oracle_route(cfg, W.router_logits(cfg, sub=b))[0] for b in range(N)]).astype(np.int32)
    U = np.random.default_rng(cfg.seed + 23).integers(0, 1 << 32, size=ids.shape, dtype=np.uint64)
    want = [scheduling.aebs(ids[b], opl) for b in range(N)]
    d_ids = dev_i32(ids)
    d_rid = torch.full((N, T, k), -9, dtype=torch.int32, device="cuda")
    d_rep = torch.full((N, cfg.E), -9, dtype=torch.int32, device="cuda")
    d_load = torch.full((N, cfg.n_inst), -9, dtype=torch.int32, device="cuda")
    B.moe_schedule_batched(pl, d_ids, N, T, k, d_rid, d_rep, d_load)
    torch.cuda.synchronize()
    for b in range(N):
        O, act_rep, load = want[b]
        np.testing.assert_array_equal(d_rid[b].cpu().numpy(), O)
        np.testing.assert_array_equal(d_rep[b].cpu().numpy(), act_rep)
        np.testing.assert_array_equal(d_load[b].cpu().numpy(), load)
    # loads only
    d_load2 = torch.full((N, cfg.n_inst), -9, dtype=torch.int32, device="cuda")
    B.moe_schedule_batched(pl, d_ids, N, T, k, None, None, d_load2)
    torch.cuda.synchronize()
    assert torch.equal(d_load, d_load2)
    # baselines
    d_draws = torch.from_numpy(U.astype(np.uint32).view(np.int32)).cuda()
    for policy in (B.MOE_POLICY_HOME, B.MOE_POLICY_RANDOM):
        d_rid.fill_(-9); d_load.fill_(-9)
        B.moe_schedule_baseline_batched(pl, d_ids, N, T, k, policy, d_draws if policy == B.MOE_POLICY_RANDOM else None,
                                        d_rid, d_load)
        torch.cuda.synchronize()
        for b in range(N):
            O = (scheduling.home_only(ids[b], opl) if policy == B.MOE_POLICY_HOME
                 else scheduling.random_replica_from_draws(ids[b], opl, U[b]))
            np.testing.assert_array_equal(d_rid[b].cpu().numpy(), O)
            np.testing.assert_array_equal(d_load[b].cpu().numpy(), scheduling.loads_of(O, opl))
