#!/usr/bin/env python3
"""Benchmark of the MoE-instance layer step on one MI355X.

One step = route -> AEBS schedule -> permute -> grouped expert FFN -> combine for the
straggler instance of a seeded synthetic batch, queued on one stream with no host
synchronisation, as three launches (fused front, fused FFN, combine).  Consecutive steps use different weight copies and different batches
from a ring (>= 1 GiB of weights in total), so expert weights come from HBM and not from
the 256 MB memory-side cache.

Prints ONE JSON line for the largest configuration of the workload list (DeepSeek-V3-shaped,
T = 512).  `value` = algorithmic bytes of a step (activated experts' weights + activation
traffic) / step time, in GB/s; the `roofline` object prices the dominant kernel (the grouped FFN)
alone, with its duration taken from HIP events recorded in the timed region on the launching
stream; `cpu_baseline` times the CPU oracle on the same workload; `other_decode_configs` carries
the same measurement for the other decode configurations (DeepSeek-V2-Lite-shaped T = 128,
Qwen3-30B-A3B-shaped T = 32 and 256).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "ffn_kernel_hbm_traffic.json")

# The headline line is quoted on the largest single-GPU configuration of the workload list; the other
# decode configurations are measured in the same run and carried as extra rows of the same JSON line.
HEADLINE = ("dsv3", 512)
OTHER_ROWS = [("dsv2lite", 128), ("qwen3", 32), ("qwen3", 256)]


def make_cfg(name: str, T):
    from paper_2512_13525_amd import workloads as W
    if name == "dsv2lite":
        return W.dsv2lite(T or 128)
    if name == "qwen3":
        return W.qwen3(T or 256)
    if name == "dsv3":
        return W.dsv3(T or 512)
    if name == "stress":
        return W.stress(T or 64, 1.25, 0.8)
    raise SystemExit(f"unknown workload {name}")


def measured_traffic(workload: str, T: int):
    """HBM bytes per FFN launch from the committed summary of the rocprofv3 FETCH_SIZE / WRITE_SIZE runs
    (written by `bench.py --mode pmc_summary`), or None when no run of this workload is on record."""
    try:
        with open(TRAFFIC_JSON) as f:
            rec = json.load(f).get(f"{workload}-T{T}")
    except (OSError, ValueError):
        return None, None
    if not rec:
        return None, None
    return rec.get("hbm_bytes_per_launch"), {"file": os.path.relpath(TRAFFIC_JSON, ROOT), "kernel": rec.get("kernel"),
                                             "source_commit": rec.get("commit")}


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=None, choices=["dsv2lite", "qwen3", "dsv3", "stress"],
                    help="step mode: measure only this workload (default: the headline dsv3 T=512 plus the other "
                         "decode configurations as extra rows)")
    ap.add_argument("--tokens", type=int, default=None)
    ap.add_argument("--ring-bytes", type=float, default=1.25e9, help="minimum total bytes of rotating weight copies")
    ap.add_argument("--rows-per-slot", type=int, default=0,
                    help="act_sweep: requests on every activated slot (0 = spread all T*k requests over them)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="do not record per-kernel events in the timed region")
    ap.add_argument("--no-other-rows", action="store_true", help="step mode: only the headline workload")
    ap.add_argument("--batches", type=int, default=2000, help="amax: sampled batches per (n_e, B)")
    ap.add_argument("--pmc-dir", default=None, help="pmc_summary: folder with the rocprofv3 counter CSVs")
    ap.add_argument("--mode", default="step", choices=["step", "sched", "act_sweep", "skew", "batch_sweep", "amax", "gate", "placement", "scaling", "shared", "graph", "configs", "probe_sweep", "calib_copy", "pmc_summary"],
                    help="step: the headline line (default); sched: scheduler us and a_max vs optimum over the "
                         "stress sweep; act_sweep: layer us vs number of activated experts; skew: same "
                         "activated set with an even and a Zipf split of the requests; batch_sweep: layer "
                         "us vs batch size with every slot activated; amax: Monte-Carlo a_max of AEBS and the "
                         "baseline policies over sampled batches, against the exact optimum and Eq. 5; gate: the front "
                         "launch with and without the router's linear layer in it; placement: a_max of AEBS over the "
                         "layout of Alg. 3 (Appendix B) against the contiguous layout on traces with topics; scaling: "
                         "Alg. 2 fed with the measured MoE-side coefficients and a_max table; shared: the step with a "
                         "shared expert run on the instance; graph: the step queued eagerly against the same steps "
                         "replayed from a captured HIP graph; configs: one line per workload configuration and "
                         "token count of the workload list; probe_sweep: the plain read probe over launch shapes; "
                         "calib_copy: a device-to-device copy of known size (counter calibration); pmc_summary: "
                         "turn rocprofv3 FETCH_SIZE / WRITE_SIZE CSVs into profiles/ffn_kernel_hbm_traffic.json (no GPU)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("this build runs on ONE GPU: the other MoE instances exist only as replica placement "
                         "seen by the scheduler; run with --gpus 1")
    if args.mode == "pmc_summary":
        return pmc_summary(args)

    import numpy as np
    import torch
    from paper_2512_13525_amd import binding as B

    B.lib()                                   # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    torch.cuda.set_device(0)
    modes = {"sched": sched_sweep, "act_sweep": act_sweep, "skew": split_sweeps, "batch_sweep": split_sweeps,
             "amax": amax_study, "gate": gate_front, "placement": placement_study, "scaling": scaling_study,
             "shared": shared_step, "graph": graph_step, "configs": all_configs, "probe_sweep": probe_sweep,
             "calib_copy": calib_copy}
    if args.mode in modes:
        return modes[args.mode](args)

    if args.workload:
        name, T = args.workload, make_cfg(args.workload, args.tokens).T
        others = []
    else:
        name, T = HEADLINE
        others = [] if args.no_other_rows else OTHER_ROWS
    out = step_bench(args, name, T, args.steps, args.warmup, full=True)
    rows = []
    for oname, oT in others:
        # the extra rows always take 100 steps after 10: their steps are short (30-50 us), an event pair costs
        # 4 us of such a step, and with 100 steps only every 4th step carries one
        r = step_bench(args, oname, oT, 100, 10, full=False)
        rows.append({"workload": r["config"]["workload"], "step_us": r["step_us"], "value_GBps": r["value"],
                     "pct_hbm_peak_whole_step": r["pct_hbm_peak_whole_step"],
                     "activated_experts_a_g": r["activated_experts_a_g"], "n_local_mean": r["n_local_mean"],
                     "steps": r["steps"], "roofline": r["roofline"]})
    if rows:
        out["other_decode_configs"] = rows
    print(json.dumps(out), flush=True)


def step_bench(args, name: str, T: int, steps: int, warmup: int, full: bool) -> dict:
    """The layer step of one workload: K timed steps (front, FFN, combine queued on one stream over a ring of
    batches and weight copies), the FFN launch timed by HIP events inside that region, and with `full`
    the per-stage times, the single-step latency, the read probe and the CPU baseline."""
    import numpy as np
    import torch
    from paper_2512_13525_amd import binding as B
    from paper_2512_13525_amd import workloads as W
    from paper_2512_13525_amd.layer import LayerStep, to_device_bf16

    cfg = make_cfg(name, T)
    lay = W.build_placement(cfg)
    T, k, C, d_h, d_e = cfg.T, cfg.k, cfg.C, cfg.d_h, cfg.d_e

    # ---- ring of input batches and weight copies
    per_copy = C * 3 * d_h * d_e * 2
    n_ring = max(4, int(-(-args.ring_bytes // per_copy)))
    logits = [torch.from_numpy(W.router_logits(cfg, sub=i)).cuda() for i in range(n_ring)]
    Xs = [to_device_bf16(W.activations(cfg, sub=i)) for i in range(n_ring)]
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    W13s, W2s = [], []
    for i in range(n_ring):
        # packed layout is a fixed permutation of the canonical one: seeded N(0, 0.02) values
        # drawn straight into it are the same workload (one slot at a time: the fp32 draw of a whole
        # instance would take several GB at the largest shape)
        w13 = torch.empty((C, 2 * d_e, d_h), dtype=torch.bfloat16, device="cuda")
        w2 = torch.empty((C, d_h, d_e), dtype=torch.bfloat16, device="cuda")
        for s_ in range(C):
            w13[s_] = (torch.randn((2 * d_e, d_h), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
            w2[s_] = (torch.randn((d_h, d_e), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
        W13s.append(w13); W2s.append(w2)

    # ---- choose the straggler instance of batch 0 (set-up, not timed)
    step = LayerStep(cfg, lay, 0)
    step.route(logits[0]); step.schedule()
    torch.cuda.synchronize()
    g_self = int(torch.argmax(step.load).item())
    step = LayerStep(cfg, lay, g_self)

    def check_status(where):
        st = B.moe_workspace_status(step.workspace)
        if st != 0:
            raise SystemExit(f"bench.py: FFN workspace status {st} after {where}: results of that section are invalid")

    def run_step(i):
        # three launches: front (route + Alg. 1 + dispatch), grouped FFN, combine
        j = i % n_ring
        step.front(logits[j])
        step.ffn(Xs[j], W13=W13s[j], W2=W2s[j])
        step.combine()

    # per-ring-entry facts (a_g, n_local) for the byte count; read back outside the timed region
    a_g, n_local, a_max = [], [], []
    for j in range(n_ring):
        run_step(j)
        torch.cuda.synchronize()
        cnt = step.slot_count.cpu().numpy()
        a_g.append(int((cnt > 0).sum())); n_local.append(int(cnt.sum())); a_max.append(int(step.load.max().item()))

    def bytes_ffn(j):
        return a_g[j] * 3 * d_h * d_e * 2 + min(T, n_local[j]) * d_h * 2 + n_local[j] * d_h * 4

    def bytes_step(j):
        # + combine (read Yp, write Y) + routing/schedule index traffic
        return (bytes_ffn(j) + n_local[j] * d_h * 4 + T * d_h * 2 + T * cfg.E * 4 + 6 * T * k * 4)

    # the plain read of the same number of bytes (mean over the ring), measured before the timed region:
    # a reference point for the FFN launch, and the GPU has reached its streaming clocks when the
    # warm-up steps begin (a run of 20 steps after 5 warm-up steps alone read 2-3 % slow)
    mean_b = statistics.mean(bytes_ffn(j) for j in range(n_ring))
    probe = read_probe_best(W13s, int(mean_b)) if (full and not args.no_events) else None

    for i in range(warmup):
        run_step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps, with an event pair around the FFN launch.  An event record costs
    # the stream a few us, which is time of the step: every step carries a pair when the step is long
    # (more than 0.5 GB per launch) or the run is short (<= 50 steps), every 4th step otherwise.  The
    # events are created without the system-scope fence of default events (a cache write-back between
    # the kernels they separate).
    every = 1 if (steps <= 50 or mean_b > 5e8) else 4
    timed = [] if args.no_events else [i for i in range(steps) if i % every == 0]
    te = TimingEvents()
    ev = {i: (te.new(), te.new()) for i in timed}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        j = i % n_ring
        step.front(logits[j])
        if i in ev:
            te.record(ev[i][0])
        step.ffn(Xs[j], W13=W13s[j], W2=W2s[j])
        if i in ev:
            te.record(ev[i][1])
        step.combine()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    check_status("the timed region")
    ms_per_step = (t1 - t0) * 1e3 / steps
    mean_bytes_step = statistics.mean(bytes_step(i % n_ring) for i in range(steps))
    value = mean_bytes_step / (ms_per_step * 1e-3) / 1e9

    roofline = None
    if timed:
        ffn_us = [te.us(ev[i][0], ev[i][1]) for i in timed]
        ffn_avg_us = statistics.mean(ffn_us)
        ffn_p50_us = statistics.median(ffn_us)
        mean_bytes_ffn = statistics.mean(bytes_ffn(i % n_ring) for i in timed)
        achieved = mean_bytes_ffn / (ffn_avg_us * 1e-6) / 1e9
        # what an event pair reads with nothing between its two records, queued like the pairs above
        # (the part of avg_us that is not the kernel; rocprofv3's kernel durations do not contain it)
        cal = [(te.new(), te.new()) for _ in range(50)]
        for a, b in cal:
            step.front(logits[0]); te.record(a); te.record(b); step.combine()
        torch.cuda.synchronize()
        empty_pair_us = statistics.median(te.us(a, b) for a, b in cal)
        traffic, traffic_src = measured_traffic(name, T)
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBPS, 4),
                    "frac_p50": round(mean_bytes_ffn / (ffn_p50_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                    "traffic": traffic, "traffic_unit": "bytes per launch", "traffic_from": traffic_src,
                    "kernel": "moe_grouped_ffn", "avg_us": round(ffn_avg_us, 2), "launches_timed": len(timed),
                    "empty_event_pair_us": round(empty_pair_us, 2),
                    "p10_us": round(float(np.percentile(ffn_us, 10)), 2),
                    "p50_us": round(ffn_p50_us, 2),
                    "p90_us": round(float(np.percentile(ffn_us, 90)), 2),
                    "algorithmic_bytes": int(mean_bytes_ffn)}
        if probe is not None:
            roofline["read_probe_same_bytes"] = probe
    te.close()

    out = {
        "metric": "moe_layer_step_algorithmic_GBps", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} MoE layer: E={cfg.E} k={k} d_h={d_h} d_e={d_e} T={T}, "
                               f"{cfg.n_inst} instances x C={C} slots, Zipf s={cfg.zipf_s}, instance g_self={g_self} "
                               f"(straggler of batch 0)",
                   "ring_copies": n_ring, "ring_bytes": n_ring * per_copy},
        "step_us": round(ms_per_step * 1e3, 2),
        "pct_hbm_peak_whole_step": round(100 * value / HBM_PEAK_GBPS, 2),
        "activated_experts_a_g": {"mean": round(statistics.mean(a_g), 2), "min": min(a_g), "max": max(a_g)},
        "a_max_over_instances": {"mean": round(statistics.mean(a_max), 2), "max": max(a_max)},
        "n_local_mean": round(statistics.mean(n_local), 1),
        "launches_per_step": 3,
        "roofline": roofline,
    }
    if not full:
        del W13s, W2s, step
        torch.cuda.empty_cache()
        return out

    # ---- per-stage times (separate instrumented pass; events between all stages)
    stages = ["route", "schedule", "permute", "ffn", "combine"]
    acc = {s: [] for s in stages}
    n_inst_steps = min(steps, 100)
    te2 = TimingEvents()
    marks = [[te2.new() for _ in range(6)] for _ in range(n_inst_steps)]
    torch.cuda.synchronize()
    for i in range(n_inst_steps):
        j = i % n_ring
        m = marks[i]
        te2.record(m[0]); step.route(logits[j])
        te2.record(m[1]); step.schedule()
        te2.record(m[2]); step.permute()
        te2.record(m[3]); step.ffn(Xs[j], W13=W13s[j], W2=W2s[j])
        te2.record(m[4]); step.combine()
        te2.record(m[5])
    torch.cuda.synchronize()
    for m in marks:
        for si, s in enumerate(stages):
            acc[s].append(te2.us(m[si], m[si + 1]))
    stage_us = {s: round(statistics.median(v), 2) for s, v in acc.items()}
    # the fused front launch (what the timed region uses instead of route + schedule + permute)
    fm = [(te2.new(), te2.new()) for _ in range(n_inst_steps)]
    for i in range(n_inst_steps):
        te2.record(fm[i][0]); step.front(logits[i % n_ring]); te2.record(fm[i][1])
        step.ffn(Xs[i % n_ring], W13=W13s[i % n_ring], W2=W2s[i % n_ring]); step.combine()
    torch.cuda.synchronize()
    stage_us["front_fused"] = round(statistics.median(te2.us(a, b) for a, b in fm), 2)
    te2.close()

    # ---- one step at a time: submit, wait, host wall clock (launch and completion latency included)
    single = []
    for i in range(min(steps, 50)):
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        run_step(i)
        torch.cuda.synchronize()
        single.append((time.perf_counter() - c0) * 1e6)
    check_status("the instrumented passes")

    out.update({
        "stage_us_median": stage_us,
        "single_step_latency_us": {"p50": round(statistics.median(single), 1),
                                   "p10": round(float(np.percentile(single, 10)), 1),
                                   "p90": round(float(np.percentile(single, 90)), 1)},
        "sched_us": stage_us["schedule"],
        "layer_us_permute_ffn_combine": round(stage_us["permute"] + stage_us["ffn"] + stage_us["combine"], 2),
    })

    # ---- CPU baseline: the oracle, as it stands, on this machine's host cores
    if not args.no_cpu_baseline:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from oracle import dispatch, ffn, scheduling
        from helpers import oracle_route
        try:
            cores = len(os.sched_getaffinity(0))
        except AttributeError:
            cores = os.cpu_count() or 1
        # untimed: input generation (only the slots batch 0 activates on this instance: the oracle
        # reads no other)
        lg, Xh = W.router_logits(cfg, sub=0), W.activations(cfg, sub=0)
        opl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
        ids0, _, _ = oracle_route(cfg, lg)
        O0, _, _ = scheduling.aebs(ids0, opl)
        cnt0, _, _ = dispatch.permute(O0, g_self, C)
        W13h = np.zeros((C, 2 * d_e, d_h), dtype=np.float32)
        W2h = np.zeros((C, d_h, d_e), dtype=np.float32)
        for s_ in np.nonzero(cnt0 > 0)[0]:
            W13h[s_], W2h[s_] = W.expert_weights(cfg, int(lay[g_self * C + s_]))
        reps, spent, sched_us = 0, 0.0, []
        while spent < 10.0 and reps < 20:
            c0 = time.perf_counter()
            ids, w, _ = oracle_route(cfg, lg)
            s0 = time.perf_counter()
            O, _, _ = scheduling.aebs(ids, opl)
            s1 = time.perf_counter()
            _, off, perm = dispatch.permute(O, g_self, C)
            Yp = ffn.grouped_ffn(Xh, W13h, W2h, off, perm, k)
            dispatch.combine(Yp, perm, w, T, k)
            c1 = time.perf_counter()
            spent += c1 - c0; reps += 1; sched_us.append((s1 - s0) * 1e6)
        cpu_s = spent / reps
        out["cpu_baseline"] = {"value": round(bytes_step(0) / cpu_s / 1e9, 3), "unit": "GB/s", "cores": cores,
                               "kind": "oracle",
                               "sample": f"{reps} whole layer steps of the same workload (batch 0, instance {g_self}), "
                                         f"NumPy fp64 oracle; {cpu_s * 1e3:.1f} ms per step, of which Alg. 1 "
                                         f"{statistics.median(sched_us):.0f} us",
                               "ms_per_step": round(cpu_s * 1e3, 2)}
    del W13s, W2s, step
    torch.cuda.empty_cache()
    return out


class TimingEvents:
    """HIP events for timing only: created with hipEventDisableSystemFence, so that recording one does
    not put a system-scope fence (a cache write-back) between the kernels it separates, which the
    default events of torch.cuda.Event do."""

    def __init__(self):
        import ctypes
        import torch
        lib = None
        for name in ("libamdhip64.so.7", "libamdhip64.so",
                     os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")):
            try:
                lib = ctypes.CDLL(name)
                break
            except OSError:
                continue
        if lib is None:
            raise RuntimeError("libamdhip64 not found")
        self.ct, self.lib = ctypes, lib
        lib.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
        lib.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.made = []

    def new(self):
        ev = self.ct.c_void_p()
        rc = self.lib.hipEventCreateWithFlags(self.ct.byref(ev), 0x20000000)     # hipEventDisableSystemFence
        if rc != 0:
            raise RuntimeError(f"hipEventCreateWithFlags: {rc}")
        self.made.append(ev)
        return ev

    def record(self, ev):
        import torch
        rc = self.lib.hipEventRecord(ev, self.ct.c_void_p(torch.cuda.current_stream().cuda_stream or None))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord: {rc}")

    def us(self, a, b):
        ms = self.ct.c_float(0.0)
        rc = self.lib.hipEventElapsedTime(self.ct.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime: {rc}")
        return ms.value * 1e3

    def close(self):
        for ev in self.made:
            self.lib.hipEventDestroy(ev)
        self.made = []


def _time_us(fn, reps):
    """Mean microseconds per call of fn over `reps` back-to-back launches (HIP events)."""
    import torch
    for _ in range(5):
        fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / reps


def _time_us_each(fn, reps):
    """Median microseconds of ONE call of fn, every call between an event pair of its own (queued back
    to back): consecutive launches cannot hide each other's start and end, which a pair around the
    whole run allows."""
    import torch
    for _ in range(5):
        fn()
    te = TimingEvents()
    ev = [(te.new(), te.new()) for _ in range(reps)]
    torch.cuda.synchronize()
    for a, b in ev:
        te.record(a); fn(); te.record(b)
    torch.cuda.synchronize()
    us = statistics.median(te.us(a, b) for a, b in ev)
    te.close()
    return us


def _time_us_graph(fn, per_graph=50, reps=8):
    """Mean microseconds per call of fn on the GPU's own timeline: per_graph back-to-back calls are
    captured in a HIP graph and the graph is replayed, so that the Python and launch-call overhead
    of the host (about 4 us per call through the ctypes binding) does not bound small kernels."""
    import torch
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(per_graph):
            fn()
    torch.cuda.synchronize()
    return _time_us(g.replay, reps) / per_graph


PROBE_SHAPES = [(wg, u) for wg in (256, 512, 1024, 2048, 4096, 8192) for u in (2, 4, 8, 16)]


def read_probe_sweep(bufs, nbytes: int):
    """A plain streaming read (moe_read_probe, libmoe_bench) of `nbytes` from each copy of the weight
    ring in turn, one launch between two HIP events like the FFN launch it is compared with, for every
    launch shape of PROBE_SHAPES (workgroups of 256 threads x independent 16-byte loads in flight per
    thread).  Returns a list of (workgroups, loads, median us, GB/s)."""
    import torch
    from paper_2512_13525_amd import binding as B
    sink = torch.zeros((64,), dtype=torch.int32, device="cuda")
    n = min(nbytes, min(t.numel() * t.element_size() for t in bufs)) // 16 * 16
    te = TimingEvents()
    res = []
    for wg, u in PROBE_SHAPES:
        ev = []
        for rep in range(4):                       # queued back to back, like the steps of the timed region
            for t in bufs:
                a, b = te.new(), te.new()
                te.record(a); B.moe_read_probe(t, n, sink, wg, u); te.record(b)
                ev.append((a, b))
        torch.cuda.synchronize()
        us = statistics.median(te.us(a, b) for a, b in ev[len(bufs):])
        res.append((wg, u, us, n / (us * 1e-6) / 1e9))
    te.close()
    return res


def read_probe_best(bufs, nbytes: int) -> dict:
    """The best point of the read probe's launch-shape sweep for a launch of `nbytes`."""
    wg, u, us, gbps = max(read_probe_sweep(bufs, nbytes), key=lambda r: r[3])
    return {"us": round(us, 1), "GBps": round(gbps, 1), "workgroups": wg, "loads_in_flight": u,
            "shapes_tried": len(PROBE_SHAPES)}


def probe_sweep(args) -> None:
    """The read probe over its launch shapes, for launches of the three decode workloads' byte counts."""
    import torch
    bufs = [torch.randint(0, 255, (int(1.6e9),), dtype=torch.uint8, device="cuda") for _ in range(4)]
    for label, nbytes in (("qwen3 T=32", 77e6), ("qwen3 T=256", 115e6), ("dsv2lite T=128", 206e6), ("dsv3 T=512", 1290e6)):
        for wg, u, us, gbps in read_probe_sweep(bufs, int(nbytes)):
            print(json.dumps({"mode": "probe_sweep", "bytes_like": label, "MB": round(nbytes / 1e6, 1), "workgroups": wg,
                              "loads_in_flight": u, "us": round(us, 2), "GBps": round(gbps, 1),
                              "frac_of_8TBps": round(gbps / HBM_PEAK_GBPS, 3)}), flush=True)


def calib_copy(args) -> None:
    """Counter calibration: plain device-to-device copies of known size, so that what rocprofv3's
    FETCH_SIZE / WRITE_SIZE read for them can scale the same counters read for the FFN kernel."""
    import torch
    mib, reps = 512, 4
    n = mib << 20
    # distinct source buffers so that every copy reads from HBM, not from the memory-side cache
    srcs = [torch.full((n,), i + 1, dtype=torch.uint8, device="cuda") for i in range(reps)]
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for t in srcs:
        dst.copy_(t)
    torch.cuda.synchronize()
    print(json.dumps({"mode": "calib_copy", "copies": reps, "bytes_read_per_copy": n, "bytes_written_per_copy": n}), flush=True)


def pmc_summary(args) -> None:
    """No GPU: reads the rocprofv3 counter CSVs of four runs under --pmc-dir
    (`<wl>_fetch/`, `<wl>_write/`: `bench.py --workload <wl> --no-other-rows --steps 20 --warmup 2 --no-cpu-baseline` under
    `--pmc FETCH_SIZE` / `--pmc WRITE_SIZE`; `copy_fetch/`, `copy_write/`: `bench.py --mode calib_copy` under the same
    counters), scales the FFN kernel's counters by the copy's, and records the HBM bytes per launch in
    profiles/ffn_kernel_hbm_traffic.json, which the step mode quotes as `roofline.traffic`."""
    import collections
    import csv
    import glob
    import subprocess

    def read(sub, counter):
        vals = collections.defaultdict(list)
        for f in glob.glob(os.path.join(args.pmc_dir, sub, "**", "*counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                if r["Counter_Name"] == counter:
                    vals[r["Kernel_Name"]].append(float(r["Counter_Value"]))
        return vals

    def mean_of(vals, pattern):
        hits = [v for kname, vs in vals.items() if pattern in kname for v in vs]
        return (statistics.mean(hits), len(hits)) if hits else (None, 0)

    copy_bytes_kib = 512 * 1024
    cf, _ = mean_of(read("copy_fetch", "FETCH_SIZE"), "copyBuffer")
    cw, _ = mean_of(read("copy_write", "WRITE_SIZE"), "copyBuffer")
    if not cf or not cw:
        raise SystemExit("pmc_summary: the calibration copy's counters are missing")
    f_fac, w_fac = copy_bytes_kib / cf, copy_bytes_kib / cw
    try:
        commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], stdout=subprocess.PIPE, text=True).stdout.strip()
    except OSError:
        commit = None
    try:
        table = json.load(open(TRAFFIC_JSON))
    except (OSError, ValueError):
        table = {}
    table["_calibration"] = {"FETCH_SIZE_factor": round(f_fac, 4), "WRITE_SIZE_factor": round(w_fac, 4),
                             "copy_KiB": copy_bytes_kib, "FETCH_SIZE_read_KiB": round(cf, 1), "WRITE_SIZE_read_KiB": round(cw, 1)}
    for wl, T in [HEADLINE] + OTHER_ROWS:
        tag = f"{wl}_T{T}"
        fetch, nf = mean_of(read(f"{tag}_fetch", "FETCH_SIZE"), "ffn_stream_kernel")
        write, nw = mean_of(read(f"{tag}_write", "WRITE_SIZE"), "ffn_stream_kernel")
        if fetch is None or write is None:
            continue
        rd, wr = fetch * f_fac * 1024, write * w_fac * 1024
        table[f"{wl}-T{T}"] = {"hbm_bytes_per_launch": int(rd + wr), "read_bytes": int(rd), "written_bytes": int(wr),
                               "dispatches": min(nf, nw), "kernel": "ffn_stream_kernel", "commit": commit,
                               "command": f"rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE -- python3 bench.py --workload {wl} "
                                          f"--tokens {T} --no-other-rows --steps 20 --warmup 2 --no-cpu-baseline"}
        print(json.dumps({"mode": "pmc_summary", "workload": wl, "T": T, **table[f"{wl}-T{T}"]}), flush=True)
    with open(TRAFFIC_JSON, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")


def sched_sweep(args) -> None:
    """Scheduler-stress sweep: 256 experts, top-8, 16 instances; one JSON line per point with the
    scheduler time (Alg. 1, one launch), a_max of AEBS on the GPU, the exact optimum and the
    static home-replica policy from the CPU oracle."""
    import numpy as np
    import torch
    from oracle import optimum, scheduling
    from paper_2512_13525_amd import binding as B
    from paper_2512_13525_amd import workloads as W
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import oracle_route

    for r in (1.0, 1.125, 1.25):
        for s in (0.0, 0.8, 1.5):
            for T in (64, 128, 256, 512, 1024, 2048, 4096, 8192):
                cfg = W.stress(T, r, s)
                lay = W.build_placement(cfg)
                pl = B.Placement(lay, cfg.E, cfg.n_inst, cfg.C)
                logits = W.router_logits(cfg)
                d_logits = torch.from_numpy(logits).cuda()
                ids = torch.empty((T, cfg.k), dtype=torch.int32, device="cuda")
                w = torch.empty((T, cfg.k), dtype=torch.float32, device="cuda")
                rid = torch.empty((T, cfg.k), dtype=torch.int32, device="cuda")
                rep = torch.empty((cfg.E,), dtype=torch.int32, device="cuda")
                load = torch.empty((cfg.n_inst,), dtype=torch.int32, device="cuda")
                B.moe_route(d_logits, cfg.k, ids, w)
                us = _time_us_graph(lambda: B.moe_schedule(pl, ids, T, cfg.k, rid, rep, load))
                route_us = _time_us_graph(lambda: B.moe_route(d_logits, cfg.k, ids, w))
                a_max = int(load.max().item())
                o_ids, _, _ = oracle_route(cfg, logits)
                opl = scheduling.make_placement(lay, cfg.E, cfg.n_inst, cfg.C)
                act = sorted(set(o_ids.reshape(-1).tolist()))
                opt = optimum.optimum_matching(act, opl)
                home = int(scheduling.loads_of(scheduling.home_only(o_ids, opl), opl).max())
                print(json.dumps({"mode": "sched", "T": T, "replication": r, "zipf_s": s, "sched_us": round(us, 2),
                                  "route_us": round(route_us, 2), "activated": len(act), "a_max_aebs": a_max,
                                  "a_max_optimum": opt, "a_max_home_only": home}), flush=True)


def gate_front(args) -> None:
    """The front of the step with the router's linear layer inside the launch (Sec. 3.3: the gate
    runs on the MoE side): us per launch of logits -> a0-a4 (moe_route_schedule_permute), of
    X, W_r -> selection (moe_gate_route) and of X, W_r -> a0-a4 (moe_gate_route_schedule_permute),
    one JSON line per workload.  Inputs rotate over 8 batches."""
    import torch
    from paper_2512_13525_amd import binding as B
    from paper_2512_13525_amd import workloads as W
    from paper_2512_13525_amd.layer import LayerStep, to_device_bf16

    for name in ("dsv2lite", "qwen3", "dsv3"):
        cfg = make_cfg(name, args.tokens)
        lay = W.build_placement(cfg)
        s = LayerStep(cfg, lay, 0)
        Wr, bias = W.router_weights(cfg)
        d_Wr = to_device_bf16(Wr)
        d_bias = None if bias is None else torch.from_numpy(bias).cuda()
        Xs = [to_device_bf16(W.activations(cfg, sub=i)) for i in range(8)]
        zs = [torch.from_numpy(W.router_logits(cfg, sub=i)).cuda() for i in range(8)]
        group = cfg.route != "softmax"
        kw = dict(mode=B.MOE_ROUTE_SIGMOID_GROUP, n_group=cfg.n_group, topk_group=cfg.topk_group) if group else {}
        it = [0]

        def nxt(xs):
            it[0] += 1
            return xs[it[0] % len(xs)]

        front = _time_us(lambda: s.front(nxt(zs)), 400)
        gate_only = _time_us(lambda: B.moe_gate_route(nxt(Xs), d_Wr, d_bias, cfg.k, s.gate_logits, s.topk_ids,
                                                      s.topk_w, s.gate_sync, **kw), 400)
        gate_front_us = _time_us(lambda: s.front_gate(nxt(Xs), d_Wr, d_bias), 400)
        flops = 2.0 * cfg.T * cfg.E * cfg.d_h
        gate_bytes = (cfg.T + cfg.E) * cfg.d_h * 2 + cfg.T * cfg.E * 4
        print(json.dumps({"mode": "gate", "workload": cfg.name, "T": cfg.T, "E": cfg.E, "d_h": cfg.d_h,
                          "front_from_logits_us": round(front, 2), "gate_route_us": round(gate_only, 2),
                          "front_from_activations_us": round(gate_front_us, 2),
                          "gate_gflop": round(flops / 1e9, 3), "gate_operand_MB": round(gate_bytes / 1e6, 2)}), flush=True)


def act_sweep(args) -> None:
    """Layer time (permute + FFN + combine) against the number of activated experts at a fixed
    batch (the paper's microbenchmark of Sec. 2.2: batch 64, requests spread evenly over exactly
    `a` experts of the instance); fits t = beta*a + c_e (Eq. 1c)."""
    import numpy as np
    import torch
    from paper_2512_13525_amd import workloads as W
    from paper_2512_13525_amd.layer import LayerStep, to_device_bf16

    cfg = make_cfg(args.workload, args.tokens or 64)
    lay = W.build_placement(cfg)
    T, k, C, d_h, d_e = cfg.T, cfg.k, cfg.C, cfg.d_h, cfg.d_e
    step = LayerStep(cfg, lay, 0)
    per_copy = C * 3 * d_h * d_e * 2
    n_ring = max(4, int(-(-args.ring_bytes // per_copy)))
    gen = torch.Generator(device="cuda").manual_seed(1)
    W13s = [(torch.randn((C, 2 * d_e, d_h), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
    W2s = [(torch.randn((C, d_h, d_e), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
    X = to_device_bf16(W.activations(cfg))
    step.topk_w.fill_(1.0 / k)
    pts = []
    a_hi = min(C, T * k // args.rows_per_slot) if args.rows_per_slot else C
    for a in range(1, a_hi + 1):
        # every request goes to one of the first `a` local slots of instance 0, round-robin; with
        # --rows-per-slot only a*rows requests do and the others are not local
        rid = np.arange(T * k, dtype=np.int32) % a
        if args.rows_per_slot:
            assert args.rows_per_slot <= T and a * args.rows_per_slot <= T * k
            rid = np.where(np.arange(T * k) < a * args.rows_per_slot, rid, C * 1000).astype(np.int32)
        rid = rid.reshape(T, k)
        step.rid.copy_(torch.from_numpy(rid))
        i = [0]

        def layer():
            j = i[0] % n_ring
            i[0] += 1
            step.permute()
            step.ffn(X, W13=W13s[j], W2=W2s[j])
            step.combine()

        def ffn_only():
            j = i[0] % n_ring
            i[0] += 1
            step.ffn(X, W13=W13s[j], W2=W2s[j])

        us = _time_us(layer, 100)
        ffn_us = _time_us_each(ffn_only, 100)
        gbps = a * 3 * d_h * d_e * 2 / (ffn_us * 1e-6) / 1e9
        pts.append((a, us))
        print(json.dumps({"mode": "act_sweep", "workload": cfg.name, "T": T, "activated": a,
                          "rows_per_slot": args.rows_per_slot or round(T * k / a, 1), "layer_us": round(us, 2),
                          "ffn_us": round(ffn_us, 2), "ffn_weight_GBps": round(gbps, 1),
                          "pct_hbm_peak": round(100 * gbps / HBM_PEAK_GBPS, 1)}), flush=True)
    xs = np.array([p[0] for p in pts], dtype=np.float64)
    ys = np.array([p[1] for p in pts], dtype=np.float64)
    beta, c_e = np.polyfit(xs, ys, 1)
    print(json.dumps({"mode": "act_sweep_fit", "workload": cfg.name, "beta_us_per_expert": round(float(beta), 3),
                      "c_e_us": round(float(c_e), 3),
                      "beta_at_hbm_peak_us": round(3 * d_h * d_e * 2 / (HBM_PEAK_GBPS * 1e3), 3)}), flush=True)


def split_sweeps(args) -> None:
    """skew: the paper's check that the layer time follows the activated set, not how the tokens
    are split over it (Sec. 2.2): all C slots activated, T*k requests split evenly or Zipf(1.2).
    batch_sweep: layer time against the batch size with all C slots activated and an even split
    (Sec. 2.2: flat until the batch reaches thousands of tokens)."""
    import numpy as np
    import torch
    from paper_2512_13525_amd import workloads as W
    from paper_2512_13525_amd.layer import LayerStep, to_device_bf16

    if args.mode == "skew":
        Ts = [args.tokens or 64]
    else:
        Ts = [args.tokens] if args.tokens else [16, 32, 64, 128, 256, 512, 1024, 2048, 4096]
    for T in Ts:
        cfg = make_cfg(args.workload, T)
        lay = W.build_placement(cfg)
        k, C, d_h, d_e = cfg.k, cfg.C, cfg.d_h, cfg.d_e
        step = LayerStep(cfg, lay, 0)
        per_copy = C * 3 * d_h * d_e * 2
        n_ring = max(4, int(-(-args.ring_bytes // per_copy)))
        gen = torch.Generator(device="cuda").manual_seed(1)
        W13s = [(torch.randn((C, 2 * d_e, d_h), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
        W2s = [(torch.randn((C, d_h, d_e), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
        X = to_device_bf16(W.activations(cfg))
        step.topk_w.fill_(1.0 / k)
        splits = {"even": None}
        if args.mode == "skew":
            p = 1.0 / np.arange(1, C + 1) ** 1.2
            splits["zipf1.2"] = p / p.sum()
        for name, p in splits.items():
            n = T * k
            if p is None:
                slot = np.arange(n, dtype=np.int32) % C
            else:
                # every slot keeps at least one request; a slot gets at most one request per token
                cnt = np.maximum(1, np.floor(p * (n - C)).astype(np.int64) + 1)
                cnt = np.minimum(cnt, T)
                while cnt.sum() > n:
                    cnt[np.argmax(cnt)] -= 1
                slot = np.repeat(np.arange(C, dtype=np.int32), cnt)
                slot = np.concatenate([slot, np.full(n - len(slot), C * 1000, dtype=np.int32)])  # not local
            rid = slot.reshape(T, k) if p is None else slot[np.argsort(np.arange(n) % T, kind="stable")].reshape(T, k)
            step.rid.copy_(torch.from_numpy(np.ascontiguousarray(rid)))
            i = [0]

            def layer():
                j = i[0] % n_ring
                i[0] += 1
                step.permute()
                step.ffn(X, W13=W13s[j], W2=W2s[j])
                step.combine()

            us = _time_us(layer, 100)
            cnts = step.slot_count.cpu().numpy()
            print(json.dumps({"mode": args.mode, "workload": cfg.name, "T": T, "split": name,
                              "activated": int((cnts > 0).sum()), "n_local": int(cnts.sum()),
                              "max_rows_per_slot": int(cnts.max()), "layer_us": round(us, 2),
                              "weight_GBps": round(C * 3 * d_h * d_e * 2 / (us * 1e-6) / 1e9, 1)}), flush=True)
        del W13s, W2s, step
        torch.cuda.empty_cache()


def sample_loads(pl, bias, E, k, T, n_batches, gen, policies=("aebs",), keep_ids=0):
    """Monte-Carlo sample for one cell of the a_max table: n_batches batches of T tokens drawn on the GPU
    (logits N(0,1) + bias), routed in one launch and scheduled in ONE launch per policy
    (moe_schedule_batched: one workgroup per batch).  Returns ({policy: loads [n_batches, n_inst]},
    the first keep_ids batches' expert ids on the host, us of the AEBS launch per batch)."""
    import torch
    from paper_2512_13525_amd import binding as B
    n_inst = pl.n_inst
    ids = torch.empty((n_batches, T, k), dtype=torch.int32, device="cuda")
    wts = torch.empty((n_batches * T, k), dtype=torch.float32, device="cuda")
    chunk = max(1, (1 << 28) // (T * E))                    # batches per draw: at most 1 GiB of fp32 logits
    for b0 in range(0, n_batches, chunk):
        nb = min(chunk, n_batches - b0)
        logits = torch.randn((nb * T, E), generator=gen, device="cuda") + bias
        B.moe_route(logits, k, ids[b0:b0 + nb].view(nb * T, k), wts[:nb * T])
    out = {}
    us = None
    for pol in policies:
        loads = torch.zeros((n_batches, n_inst), dtype=torch.int32, device="cuda")
        if pol == "aebs":
            fn = lambda: B.moe_schedule_batched(pl, ids, n_batches, T, k, None, None, loads)
            fn()
            us = _time_us(fn, 5) / n_batches
        elif pol == "home":
            B.moe_schedule_baseline_batched(pl, ids, n_batches, T, k, B.MOE_POLICY_HOME, None, None, loads)
        else:
            draws = torch.randint(0, 1 << 31, (n_batches, T, k), generator=gen, device="cuda", dtype=torch.int32)
            B.moe_schedule_baseline_batched(pl, ids, n_batches, T, k, B.MOE_POLICY_RANDOM, draws, None, loads)
        out[pol] = loads
    torch.cuda.synchronize()
    return out, (ids[:keep_ids].cpu().numpy() if keep_ids else None), us


def amax_study(args) -> None:
    """Monte-Carlo table of a_max (the largest per-instance number of activated experts, which
    Eq. 1c turns into the MoE-side latency) over sampled decode batches, for AEBS and for the two
    baseline policies (first replica only; random replica per request), next to the exact optimum
    on a subsample and the balls-into-bins bound of Eq. 5 (Appendix A).  E = 256, k = 8, Zipf 0.8,
    replication 1.25; n_e instances and batch size B vary; --batches sampled batches per cell
    (default 2000), all scheduled by one launch per policy.  Logits are drawn on the GPU with the
    recipe of the other workloads (N(0,1) + ln(E p_e)).  The last line is the table a_max(n_e, B) in the
    form moe_scaling_solve reads."""
    import numpy as np
    import torch
    from oracle import bounds, optimum, scheduling
    from paper_2512_13525_amd import binding as B
    from paper_2512_13525_amd import workloads as W

    E, k, s, r, n_batches, n_opt = 256, 8, 0.8, 1.25, args.batches, 16
    gen = torch.Generator(device="cuda").manual_seed(7)
    ne_values, B_values = [8, 16, 32], [64, 128, 256, 512, 1024]
    table = np.zeros((len(ne_values), len(B_values)))
    for ri, n_inst in enumerate(ne_values):
        C = int(np.ceil(E * r / n_inst))
        cfg0 = W.MoEConfig(f"amax_ne{n_inst}", E=E, k=k, d_h=64, d_e=64, T=1, n_inst=n_inst, C=C, zipf_s=s, seed=0)
        lay = W.build_placement(cfg0)
        pl = B.Placement(lay, E, n_inst, C)
        opl = scheduling.make_placement(lay, E, n_inst, C)
        bias = torch.from_numpy(np.log(E * W.expert_popularity(cfg0)).astype(np.float32)).cuda()
        # p_e = probability that one token selects e, from a calibration sample of routed tokens
        Tc = 1 << 15
        ids = torch.empty((Tc, k), dtype=torch.int32, device="cuda")
        wts = torch.empty((Tc, k), dtype=torch.float32, device="cuda")
        B.moe_route(torch.randn((Tc, E), generator=gen, device="cuda") + bias, k, ids, wts)
        p_e = np.bincount(ids.cpu().numpy().reshape(-1), minlength=E) / Tc
        hosted = [[int(e) for e in lay[g * C:(g + 1) * C] if e >= 0] for g in range(n_inst)]
        for ci, T in enumerate(B_values):
            loads, ids_keep, us_batch = sample_loads(pl, bias, E, k, T, n_batches, gen, ("aebs", "home", "random"), n_opt)
            amax = {p: v.max(dim=1).values.cpu().numpy() for p, v in loads.items()}
            # one launch per batch, for comparison (the single-batch entry point, graph-replayed)
            one = torch.from_numpy(ids_keep[0]).cuda()
            rid = torch.empty((T, k), dtype=torch.int32, device="cuda")
            rep = torch.empty((E,), dtype=torch.int32, device="cuda")
            ld = torch.empty((n_inst,), dtype=torch.int32, device="cuda")
            us_single = _time_us_graph(lambda: B.moe_schedule(pl, one, T, k, rid, rep, ld), 20, 4)
            opt = [optimum.optimum_matching(sorted(set(i.reshape(-1).tolist())), opl) for i in ids_keep]
            a_bar = max(bounds.expected_activated(p_e, h, T) for h in hosted)
            table[ri, ci] = float(amax["aebs"].mean())
            print(json.dumps({"mode": "amax", "n_inst": n_inst, "C": C, "B": T, "batches": n_batches,
                              "a_max_aebs": {"mean": round(float(amax["aebs"].mean()), 3), "max": int(amax["aebs"].max())},
                              "a_max_home_only": {"mean": round(float(amax["home"].mean()), 3), "max": int(amax["home"].max())},
                              "a_max_random": {"mean": round(float(amax["random"].mean()), 3), "max": int(amax["random"].max())},
                              "a_max_optimum_mean_first16": round(float(np.mean(opt)), 2),
                              "a_max_aebs_mean_first16": round(float(amax["aebs"][:n_opt].mean()), 2),
                              "eq4_expected_max": round(a_bar, 2), "eq5_bound": bounds.a_max_bound(a_bar, C, n_inst),
                              "sched_us_per_batch_batched_launch": round(us_batch, 3),
                              "sched_us_single_launch": round(us_single, 2)}), flush=True)
    print(json.dumps({"mode": "amax_table", "policy": "aebs", "batches_per_cell": n_batches, "ne_values": ne_values,
                      "B_values": B_values, "a_max_table": np.round(table, 3).tolist()}), flush=True)


def all_configs(args) -> None:
    """One line per configuration and token count of the workload list: the step (front + FFN +
    combine, queued back to back over a ring of batches and weight copies) on the instance with the
    largest load of batch 0, the FFN launch alone (every launch between an event pair of its own), the activated experts and requests of that
    instance, and the FFN's algorithmic GB/s and fraction of the 8 TB/s peak."""
    import numpy as np
    import torch
    from paper_2512_13525_amd import workloads as W
    from paper_2512_13525_amd.layer import LayerStep, to_device_bf16

    cfgs = [W.tiny(), W.dsv2lite(128), W.qwen3(32), W.qwen3(256), W.qwen3(1024), W.dsv3(512)]
    cfgs += [W.stress(T, 1.25, 0.8) for T in (64, 512, 2048, 8192)]
    for cfg in cfgs:
        lay = W.build_placement(cfg)
        T, k, C, d_h, d_e = cfg.T, cfg.k, cfg.C, cfg.d_h, cfg.d_e
        bf16 = cfg.dtype == "bf16"
        esz = 2 if bf16 else 4
        n_ring = max(2, min(8, int(-(-args.ring_bytes // (C * 3 * d_h * d_e * esz)))))
        gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
        tdt = torch.bfloat16 if bf16 else torch.float32
        W13s = [(torch.randn((C, 2 * d_e, d_h), generator=gen, device="cuda") * 0.02).to(tdt) for _ in range(n_ring)]
        W2s = [(torch.randn((C, d_h, d_e), generator=gen, device="cuda") * 0.02).to(tdt) for _ in range(n_ring)]
        logits = [torch.from_numpy(W.router_logits(cfg, sub=i)).cuda() for i in range(n_ring)]
        Xs = [to_device_bf16(W.activations(cfg, sub=i)) if bf16 else torch.from_numpy(W.activations(cfg, sub=i)).cuda()
              for i in range(n_ring)]
        s = LayerStep(cfg, lay, 0)
        s.route(logits[0]); s.schedule()
        torch.cuda.synchronize()
        s = LayerStep(cfg, lay, int(torch.argmax(s.load).item()))
        a_g, n_local = [], []
        for j in range(n_ring):
            s.step_fused(logits[j], Xs[j], W13=W13s[j], W2=W2s[j])
            torch.cuda.synchronize()
            cnt = s.slot_count.cpu().numpy()
            a_g.append(int((cnt > 0).sum())); n_local.append(int(cnt.sum()))
        i = [0]

        def nxt():
            i[0] += 1
            return i[0] % n_ring

        def step():
            j = nxt()
            s.step_fused(logits[j], Xs[j], W13=W13s[j], W2=W2s[j])

        def ffn():
            j = nxt()
            s.ffn(Xs[j], W13=W13s[j], W2=W2s[j])

        def front():
            s.front(logits[nxt()])

        reps = 200 if T <= 1024 else 50
        step_us, front_us = _time_us(step, reps), _time_us_graph(front, 20, 4)
        ffn_us = _time_us_each(ffn, reps)     # the dispatch of the last step stays in place: the batch of copy j
        bytes_ffn = float(np.mean([a * 3 * d_h * d_e * esz + min(T, n) * d_h * esz + n * d_h * 4 for a, n in zip(a_g, n_local)]))
        gbps = bytes_ffn / (ffn_us * 1e-6) / 1e9
        print(json.dumps({"mode": "configs", "workload": cfg.name, "T": T, "dtype": cfg.dtype, "E": cfg.E, "k": k,
                          "d_h": d_h, "d_e": d_e, "n_inst": cfg.n_inst, "C": C,
                          "activated_a_g_mean": round(float(np.mean(a_g)), 2), "n_local_mean": round(float(np.mean(n_local)), 1),
                          "step_us": round(step_us, 2), "front_us": round(front_us, 2), "ffn_us": round(ffn_us, 2),
                          "ffn_algorithmic_MB": round(bytes_ffn / 1e6, 1), "ffn_GBps": round(gbps, 1),
                          "ffn_frac_of_8TBps": round(gbps / HBM_PEAK_GBPS, 3)}), flush=True)
        del W13s, W2s, s
        torch.cuda.empty_cache()


def graph_step(args) -> None:
    """Every compute entry point is asynchronous, allocates nothing and reads nothing back, so
    a run of layer steps can be captured in a HIP graph: us per step for the ring of batches
    queued eagerly (three launches per step from Python) and for the same ring replayed from one
    captured graph."""
    import torch
    from paper_2512_13525_amd import workloads as W
    from paper_2512_13525_amd.layer import LayerStep, to_device_bf16

    for name in ("dsv2lite", "qwen3", "dsv3"):
        cfg = make_cfg(name, args.tokens)
        lay = W.build_placement(cfg)
        C, d_h, d_e = cfg.C, cfg.d_h, cfg.d_e
        n_ring = max(4, int(-(-args.ring_bytes // (C * 3 * d_h * d_e * 2))))
        gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
        W13s = [(torch.randn((C, 2 * d_e, d_h), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
        W2s = [(torch.randn((C, d_h, d_e), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
        logits = [torch.from_numpy(W.router_logits(cfg, sub=i)).cuda() for i in range(n_ring)]
        Xs = [to_device_bf16(W.activations(cfg, sub=i)) for i in range(n_ring)]
        s = LayerStep(cfg, lay, 0)
        s.route(logits[0]); s.schedule()
        torch.cuda.synchronize()
        s = LayerStep(cfg, lay, int(torch.argmax(s.load).item()))

        def ring():
            for j in range(n_ring):
                s.step_fused(logits[j], Xs[j], W13=W13s[j], W2=W2s[j])

        ring()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            ring()
        torch.cuda.synchronize()
        reps = max(1, 400 // n_ring)
        eager = _time_us(ring, reps) / n_ring
        graph = _time_us(g.replay, reps) / n_ring
        print(json.dumps({"mode": "graph", "workload": cfg.name, "T": cfg.T, "steps_per_graph": n_ring,
                          "eager_step_us": round(eager, 2), "graph_step_us": round(graph, 2)}), flush=True)
        del g, W13s, W2s
        torch.cuda.empty_cache()


def shared_step(args) -> None:
    """The layer step with the shared-expert option (the paper keeps the shared expert on the
    attention side, Sec. 4; this runs it on the instance as one more slot that all T tokens visit):
    us per step without and with it, and of the shared FFN launch alone."""
    import torch
    from paper_2512_13525_amd import binding as B
    from paper_2512_13525_amd import workloads as W
    from paper_2512_13525_amd.layer import LayerStep, to_device_bf16

    for name, d_s in (("dsv2lite", 2816), ("dsv3", 2048)):
        cfg = make_cfg(name, args.tokens)
        lay = W.build_placement(cfg)
        T, C, d_h, d_e = cfg.T, cfg.C, cfg.d_h, cfg.d_e
        n_ring = max(4, int(-(-args.ring_bytes // (C * 3 * d_h * d_e * 2))))
        gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
        W13s = [(torch.randn((C, 2 * d_e, d_h), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
        W2s = [(torch.randn((C, d_h, d_e), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
        logits = [torch.from_numpy(W.router_logits(cfg, sub=i)).cuda() for i in range(n_ring)]
        Xs = [to_device_bf16(W.activations(cfg, sub=i)) for i in range(n_ring)]
        s = LayerStep(cfg, lay, 0)
        s.route(logits[0]); s.schedule()
        torch.cuda.synchronize()
        s = LayerStep(cfg, lay, int(torch.argmax(s.load).item()))
        ws13, ws2 = W.shared_expert_weights(cfg, d_s)
        s.enable_shared(to_device_bf16(ws13), to_device_bf16(ws2))
        i = [0]

        def nxt():
            i[0] += 1
            return i[0] % n_ring

        def plain():
            j = nxt()
            s.step_fused(logits[j], Xs[j], W13=W13s[j], W2=W2s[j])

        def shared():
            j = nxt()
            s.step_fused_shared(logits[j], Xs[j], W13=W13s[j], W2=W2s[j])

        def shared_ffn():
            j = nxt()
            B.moe_grouped_ffn(Xs[j], s.s_W13, s.s_W2, T, 1, 1, d_h, d_s, s.dtype, s.s_slot_off, s.s_perm, s.s_blocks,
                              s.s_Yp, s.s_workspace)

        print(json.dumps({"mode": "shared", "workload": cfg.name, "T": T, "shared_width": d_s,
                          "shared_weight_MB": round(3 * d_h * d_s * 2 / 1e6, 1),
                          "step_us": round(_time_us(plain, 200), 2), "step_with_shared_us": round(_time_us(shared, 200), 2),
                          "shared_ffn_us": round(_time_us(shared_ffn, 200), 2)}), flush=True)
        del W13s, W2s
        torch.cuda.empty_cache()


def scaling_study(args) -> None:
    """Alg. 2 (Sec. 3.5) on this machine's measurements: the MoE-side coefficients of Eq. 1c
    (beta, c_e) are fitted from layer times of the default workload's shape at 6 activation counts
    (16 requests on every activated slot),
    a_max(n_e, B) is the Monte-Carlo mean of Alg. 1 on the GPU over --batches sampled batches per cell
    (default 2000, one batched launch per cell);
    the attention-side and communication coefficients have no counterpart in this build and are
    stated stand-ins.  Times in microseconds, demand in requests per microsecond."""
    import numpy as np
    import torch
    from paper_2512_13525_amd import binding as B
    from paper_2512_13525_amd import workloads as W
    from paper_2512_13525_amd.layer import LayerStep, to_device_bf16

    base = make_cfg("dsv2lite", 64)
    E, k, C, d_h, d_e, T = base.E, base.k, base.C, base.d_h, base.d_e, base.T
    # ---- beta, c_e: permute + FFN + combine against the number of activated experts
    step = LayerStep(base, W.build_placement(base), 0)
    gen = torch.Generator(device="cuda").manual_seed(1)
    n_ring = max(4, int(-(-args.ring_bytes // (C * 3 * d_h * d_e * 2))))
    W13s = [(torch.randn((C, 2 * d_e, d_h), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
    W2s = [(torch.randn((C, d_h, d_e), generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(n_ring)]
    X = to_device_bf16(W.activations(base))
    step.topk_w.fill_(1.0 / k)
    pts = []
    for a in (2, 5, 8, 11, 14, 17):
        # 16 requests on every activated slot, the other requests of the batch on other instances
        rid = np.where(np.arange(T * k) < a * 16, np.arange(T * k) % a, C * 1000).astype(np.int32)
        step.rid.copy_(torch.from_numpy(rid.reshape(T, k)))
        i = [0]

        def layer():
            j = i[0] % n_ring
            i[0] += 1
            step.permute(); step.ffn(X, W13=W13s[j], W2=W2s[j]); step.combine()

        pts.append((a, _time_us(layer, 100)))
    beta, c_e = (float(v) for v in np.polyfit([p[0] for p in pts], [p[1] for p in pts], 1))
    del W13s, W2s
    # ---- a_max table over (n_e, B): Monte-Carlo mean of Alg. 1, one batched launch per cell
    ne_values, B_values, n_batches = [4, 8, 16], [16, 64, 256, 1024], args.batches
    table = np.zeros((len(ne_values), len(B_values)))
    for r, n_inst in enumerate(ne_values):
        cfg = W.MoEConfig(f"scale_ne{n_inst}", E=E, k=k, d_h=64, d_e=64, T=1, n_inst=n_inst, C=C, zipf_s=base.zipf_s, seed=0)
        pl = B.Placement(W.build_placement(cfg), E, n_inst, C)
        bias = torch.from_numpy(np.log(E * W.expert_popularity(cfg)).astype(np.float32)).cuda()
        for c, Bt in enumerate(B_values):
            loads, _, _ = sample_loads(pl, bias, E, k, Bt, n_batches, gen)
            table[r, c] = float(loads["aebs"].max(dim=1).values.float().mean().item())
    print(json.dumps({"mode": "scaling_inputs", "beta_us_per_expert": round(beta, 3), "c_e_us": round(c_e, 3),
                      "fit_points": [[a, round(t, 2)] for a, t in pts], "ne_values": ne_values, "B_values": B_values,
                      "a_max_table": np.round(table, 2).tolist()}), flush=True)

    class M:                                   # stand-ins for what this build does not have (attention, network)
        L = 26
        c_a, alpha, c_kv = 30.0, 0.5, 4e-4
        comm0, comm1 = 20.0, 0.02
        S_ctx = 2048.0
        mem_budget, mem_fixed, mem_per_token = 288e9, 40e9, 70e3
    M.beta, M.c_e = beta, c_e
    for slo_ms in (4.0, 6.0):
        for lam in (0.002, 0.01, 0.03, 0.06, 0.1, 0.2):
            r = B.moe_scaling_solve(M, table, ne_values, B_values, lam, slo_ms * 1e3, 16, -(-E // C), 1024.0)
            out = {"mode": "scaling", "slo_ms": slo_ms, "lambda_req_per_us": lam}
            if r is None:
                out["feasible"] = False
            else:
                out.update({"feasible": True, "n_a": r[0], "n_e": r[1], "B_star": round(r[2], 1), "tpot_ms": round(r[3] / 1e3, 3)})
            print(json.dumps(out), flush=True)


def placement_study(args) -> None:
    """Effect of the activation-aware layout (Appendix B: replica counts from window statistics,
    Alg. 3 placement by co-activation) on what Alg. 1 achieves.  A synthetic trace with topics
    (each batch prefers one cluster of experts) is routed on the GPU; the first half of the
    batches is the statistics window (moe_coactivation_counts -> moe_replica_counts ->
    moe_place_replicas, host), the second half is scheduled by moe_schedule over (i) the contiguous
    layout of the other workloads and (ii) the Alg. 3 layout.  E = 256, k = 8, 16 instances x 20
    slots, Zipf 0.8; one JSON line per (cluster shape, batch size)."""
    import time
    import numpy as np
    import torch
    from oracle import optimum, placement_opt, scheduling
    from paper_2512_13525_amd import binding as B
    from paper_2512_13525_amd import workloads as W

    E, k, n_inst, C, n_topics, boost, n_batches, n_opt = 256, 8, 16, 20, 8, 2.0, 400, 16
    cfg = W.MoEConfig("placement", E=E, k=k, d_h=64, d_e=64, T=1, n_inst=n_inst, C=C, zipf_s=0.8, seed=0)
    gen = torch.Generator(device="cuda").manual_seed(11)
    for contiguous in (True, False):
        tb = torch.from_numpy(W.topic_bias(cfg, n_topics, boost, contiguous)).cuda()
        for T in (16, 64, 256):
            ids = torch.empty((n_batches, T, k), dtype=torch.int32, device="cuda")
            wts = torch.empty((T, k), dtype=torch.float32, device="cuda")
            topics = torch.randint(0, n_topics, (n_batches,), generator=gen, device="cuda")
            for b in range(n_batches):
                logits = torch.randn((T, E), generator=gen, device="cuda") + tb[topics[b]]
                B.moe_route(logits, k, ids[b], wts)
            torch.cuda.synchronize()
            half = n_batches // 2
            window = ids[:half].cpu().numpy()
            t0 = time.perf_counter()
            c, a = B.moe_coactivation_counts(window, E)
            R = B.moe_replica_counts(c, n_inst, C)
            t1 = time.perf_counter()
            lay3 = B.moe_place_replicas(n_inst, C, R, c, a)
            t2 = time.perf_counter()
            layouts = {"contiguous": W.build_placement(cfg), "alg3": lay3}
            out = {"mode": "placement", "clusters": "contiguous ids" if contiguous else "random subsets",
                   "B": T, "window_batches": half, "eval_batches": n_batches - half,
                   "stats_ms": round((t1 - t0) * 1e3, 2), "alg3_ms": round((t2 - t1) * 1e3, 2)}
            rid = torch.empty((T, k), dtype=torch.int32, device="cuda")
            rep = torch.empty((E,), dtype=torch.int32, device="cuda")
            for name, lay in layouts.items():
                pl = B.Placement(lay, E, n_inst, C)
                loads = torch.zeros((n_batches - half, n_inst), dtype=torch.int32, device="cuda")
                for b in range(half, n_batches):
                    B.moe_schedule(pl, ids[b], T, k, rid, rep, loads[b - half])
                torch.cuda.synchronize()
                amax = loads.max(dim=1).values.cpu().numpy()
                opl = scheduling.make_placement(lay, E, n_inst, C)
                opt = [optimum.optimum_matching(sorted(set(ids[half + i].cpu().numpy().reshape(-1).tolist())), opl)
                       for i in range(n_opt)]
                P = np.asarray(lay).reshape(n_inst, C)
                I = [placement_opt.coactivation_load([int(e) for e in P[g] if e >= 0], a) for g in range(n_inst)]
                out[name] = {"a_max_aebs_mean": round(float(amax.mean()), 2), "a_max_aebs_max": int(amax.max()),
                             "a_max_aebs_mean_first16": round(float(amax[:n_opt].mean()), 2),
                             "a_max_optimum_mean_first16": round(float(np.mean(opt)), 2),
                             "max_coactivation_load": round(max(I), 1)}
            print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
