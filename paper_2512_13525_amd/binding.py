"""Thin ctypes binding over libmoe_janus.so: same names as the C ABI (include/moe_janus.h),
argument marshalling only.  Tensors are torch CUDA tensors used purely as device memory;
every step of the path runs in the library's HIP kernels.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmoe_janus.so")
BENCH_LIB_PATH = os.path.join(_PKG, "libmoe_bench.so")

MOE_OK = 0
MOE_EINVAL, MOE_ESHAPE, MOE_EPLACEMENT, MOE_EHIP, MOE_ENOMEM, MOE_EWORKSPACE = -1, -2, -3, -4, -5, -6
MOE_DTYPE_BF16, MOE_DTYPE_F32 = 0, 1
MOE_ROUTE_SOFTMAX, MOE_ROUTE_SIGMOID_GROUP = 0, 1
MOE_FFN_BLOCK_ROWS = 64
MOE_POLICY_HOME, MOE_POLICY_RANDOM = 0, 1

EXPORTS = [
    "moe_strerror", "moe_last_error",
    "moe_placement_create", "moe_placement_destroy", "moe_placement_replicas", "moe_placement_dims",
    "moe_route", "moe_schedule", "moe_schedule_baseline", "moe_schedule_batched", "moe_schedule_baseline_batched", "moe_permute", "moe_block_rows", "moe_max_blocks", "moe_block_list_len",
    "moe_route_schedule_permute", "moe_front_sync_len", "moe_gate_sync_len", "moe_gate_route", "moe_gate_route_schedule_permute",
    "moe_coactivation_counts", "moe_replica_counts", "moe_place_replicas", "moe_scaling_solve",
    "moe_pack_weights_bf16",
    "moe_workspace_bytes", "moe_workspace_init", "moe_workspace_status", "moe_grouped_ffn", "moe_combine",
    "moe_shared_dispatch", "moe_combine_shared", "moe_workspace_set_option", "moe_grouped_ffn_static",
]
MOE_FFN_STATIC_SCRATCH_BYTES = 32 << 20
BENCH_EXPORTS = ["moe_read_probe"]
MOE_WS_OPT_SPIN_LIMIT, MOE_WS_OPT_WIDE_MIN_WORKGROUPS = 0, 1


class moe_scaling_model(ctypes.Structure):
    _fields_ = [("L", ctypes.c_int)] + [(n, ctypes.c_double) for n in (
        "c_a", "alpha", "c_kv", "beta", "c_e", "comm0", "comm1", "S_ctx", "mem_budget", "mem_fixed", "mem_per_token")]


class MoeError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(what)


class moe_route_cfg(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int), ("renormalize", ctypes.c_int), ("n_group", ctypes.c_int),
                ("topk_group", ctypes.c_int), ("scale", ctypes.c_float)]


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Load the library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MoeError(MOE_EINVAL, f"{LIB_PATH} is missing: build it with "
                                   f"`python -m paper_2512_13525_amd.build` (no CPU fallback exists)")
    L = ctypes.CDLL(LIB_PATH)
    vp, ci, cs = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.moe_strerror.restype = ctypes.c_char_p
    L.moe_strerror.argtypes = [ci]
    L.moe_last_error.restype = ctypes.c_char_p
    L.moe_last_error.argtypes = []
    L.moe_placement_create.restype = ci
    L.moe_placement_create.argtypes = [ctypes.POINTER(vp), ci, ci, ci, vp]
    L.moe_placement_destroy.restype = None
    L.moe_placement_destroy.argtypes = [vp]
    L.moe_placement_replicas.restype = ci
    L.moe_placement_replicas.argtypes = [vp, ci]
    L.moe_placement_dims.restype = ci
    L.moe_placement_dims.argtypes = [vp, ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ci)]
    L.moe_route.restype = ci
    L.moe_route.argtypes = [vp, ci, ci, ci, ctypes.POINTER(moe_route_cfg), vp, vp, vp]
    L.moe_schedule.restype = ci
    L.moe_schedule.argtypes = [vp, vp, ci, ci, vp, vp, vp, vp]
    L.moe_schedule_baseline.restype = ci
    L.moe_schedule_baseline.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp]
    L.moe_schedule_batched.restype = ci
    L.moe_schedule_batched.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp]
    L.moe_schedule_baseline_batched.restype = ci
    L.moe_schedule_baseline_batched.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, vp, vp]
    L.moe_permute.restype = ci
    L.moe_permute.argtypes = [vp, ci, vp, ci, ci, vp, vp, vp, vp, vp, vp]
    L.moe_block_rows.restype = ci
    L.moe_block_rows.argtypes = [ci]
    L.moe_max_blocks.restype = cs
    L.moe_max_blocks.argtypes = [ci, ci, ci]
    L.moe_block_list_len.restype = cs
    L.moe_block_list_len.argtypes = [ci, ci, ci]
    L.moe_route_schedule_permute.restype = ci
    L.moe_route_schedule_permute.argtypes = [vp, ci, vp, ci, ci, ctypes.POINTER(moe_route_cfg)] + [vp] * 12
    L.moe_coactivation_counts.restype = ci
    L.moe_coactivation_counts.argtypes = [vp, ci, ci, ci, vp, vp]
    L.moe_replica_counts.restype = ci
    L.moe_replica_counts.argtypes = [ci, ci, ci, vp, vp]
    L.moe_place_replicas.restype = ci
    L.moe_place_replicas.argtypes = [ci, ci, ci, vp, vp, vp, vp]
    cd = ctypes.c_double
    L.moe_scaling_solve.restype = ci
    L.moe_scaling_solve.argtypes = [vp, vp, vp, ci, vp, ci, cd, cd, ci, ci, cd, vp, vp, vp, vp]
    L.moe_front_sync_len.restype = cs
    L.moe_front_sync_len.argtypes = [vp, ci, ci]
    L.moe_gate_sync_len.restype = cs
    L.moe_gate_sync_len.argtypes = [ci]
    L.moe_gate_route.restype = ci
    L.moe_gate_route.argtypes = [vp, vp, vp, ci, ci, ci, ci, ctypes.POINTER(moe_route_cfg)] + [vp] * 5
    L.moe_gate_route_schedule_permute.restype = ci
    L.moe_gate_route_schedule_permute.argtypes = [vp, ci, vp, vp, vp, ci, ci, ci, ctypes.POINTER(moe_route_cfg)] + [vp] * 13
    L.moe_pack_weights_bf16.restype = ci
    L.moe_pack_weights_bf16.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp]
    L.moe_workspace_bytes.restype = cs
    L.moe_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
    L.moe_workspace_init.restype = ci
    L.moe_workspace_init.argtypes = [vp, cs, vp]
    L.moe_workspace_status.restype = ci
    L.moe_workspace_status.argtypes = [vp, ctypes.POINTER(ci)]
    L.moe_grouped_ffn.restype = ci
    L.moe_grouped_ffn.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, cs, vp]
    L.moe_grouped_ffn_static.restype = ci
    L.moe_grouped_ffn_static.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp]
    L.moe_combine.restype = ci
    L.moe_combine.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp]
    L.moe_workspace_set_option.restype = ci
    L.moe_workspace_set_option.argtypes = [vp, cs, ci, ci, vp]
    L.moe_shared_dispatch.restype = ci
    L.moe_shared_dispatch.argtypes = [ci, vp, vp, vp, vp]
    L.moe_combine_shared.restype = ci
    L.moe_combine_shared.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp]
    _lib = L
    return L


def _check(code: int, what: str) -> None:
    if code != MOE_OK:
        L = lib()
        msg = L.moe_strerror(code).decode()
        if code == MOE_EHIP:
            msg += ": " + L.moe_last_error().decode()
        raise MoeError(code, f"{what}: {msg}")


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    """hipStream_t of a torch stream (None = torch's current stream)."""
    import torch
    if stream is None:
        raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)
        if raw is not None:                   # the fast path: no Stream object is built
            return raw(torch.cuda.current_device()) or None
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


class Placement:
    """Owner of a moe_placement_t."""

    def __init__(self, slot_to_expert, E: int, n_inst: int, C: int):
        arr = np.ascontiguousarray(np.asarray(slot_to_expert), dtype=np.int32)
        if arr.shape != (n_inst * C,):
            raise MoeError(MOE_EINVAL, "slot_to_expert must have n_inst*C entries")
        self._h = ctypes.c_void_p()
        self.E, self.n_inst, self.C = E, n_inst, C
        _check(lib().moe_placement_create(ctypes.byref(self._h), E, n_inst, C, arr.ctypes.data),
               "moe_placement_create")

    @property
    def handle(self):
        return self._h

    def replicas(self, e: int) -> int:
        return lib().moe_placement_replicas(self._h, e)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            lib().moe_placement_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moe_route(logits, k: int, topk_ids, topk_w, mode: int = MOE_ROUTE_SOFTMAX, renormalize: bool = True,
              n_group: int = 1, topk_group: int = 1, scale: float = 1.0, stream=None) -> None:
    T, E = logits.shape
    cfg = moe_route_cfg(mode, int(renormalize), n_group, topk_group, scale)
    _check(lib().moe_route(_ptr(logits), T, E, k, ctypes.byref(cfg), _ptr(topk_ids), _ptr(topk_w),
                           _stream(stream)), "moe_route")


def moe_schedule(pl: Placement, topk_ids, T: int, k: int, rid, act_rep, load, stream=None) -> None:
    _check(lib().moe_schedule(pl.handle, _ptr(topk_ids), T, k, _ptr(rid), _ptr(act_rep), _ptr(load),
                              _stream(stream)), "moe_schedule")


def moe_schedule_baseline(pl: Placement, topk_ids, T: int, k: int, policy: int, draws, rid, load, stream=None) -> None:
    _check(lib().moe_schedule_baseline(pl.handle, _ptr(topk_ids), T, k, policy, _ptr(draws), _ptr(rid), _ptr(load),
                                       _stream(stream)), "moe_schedule_baseline")


def moe_schedule_batched(pl: Placement, topk_ids, n_batches: int, T: int, k: int, rid, act_rep, load, stream=None) -> None:
    _check(lib().moe_schedule_batched(pl.handle, _ptr(topk_ids), n_batches, T, k, _ptr(rid), _ptr(act_rep), _ptr(load),
                                      _stream(stream)), "moe_schedule_batched")


def moe_schedule_baseline_batched(pl: Placement, topk_ids, n_batches: int, T: int, k: int, policy: int, draws, rid, load,
                                  stream=None) -> None:
    _check(lib().moe_schedule_baseline_batched(pl.handle, _ptr(topk_ids), n_batches, T, k, policy, _ptr(draws), _ptr(rid),
                                               _ptr(load), _stream(stream)), "moe_schedule_baseline_batched")


def moe_permute(pl: Placement, g_self: int, rid, T: int, k: int, slot_count, slot_off, perm, pos, blocks,
                stream=None) -> None:
    _check(lib().moe_permute(pl.handle, g_self, _ptr(rid), T, k, _ptr(slot_count), _ptr(slot_off),
                             _ptr(perm), _ptr(pos), _ptr(blocks), _stream(stream)), "moe_permute")


def moe_block_rows(T: int) -> int:
    return int(lib().moe_block_rows(T))


def moe_max_blocks(T: int, k: int, C: int) -> int:
    return int(lib().moe_max_blocks(T, k, C))


def moe_block_list_len(T: int, k: int, C: int) -> int:
    return int(lib().moe_block_list_len(T, k, C))


def moe_route_schedule_permute(pl: Placement, g_self: int, logits, k: int, topk_ids, topk_w, rid, act_rep, load,
                               slot_count, slot_off, perm, pos, blocks, sync, mode: int = MOE_ROUTE_SOFTMAX,
                               renormalize: bool = True, n_group: int = 1, topk_group: int = 1, scale: float = 1.0,
                               stream=None) -> None:
    T = logits.shape[0]
    cfg = moe_route_cfg(mode, int(renormalize), n_group, topk_group, scale)
    _check(lib().moe_route_schedule_permute(pl.handle, g_self, _ptr(logits), T, k, ctypes.byref(cfg),
                                            _ptr(topk_ids), _ptr(topk_w), _ptr(rid), _ptr(act_rep), _ptr(load),
                                            _ptr(slot_count), _ptr(slot_off), _ptr(perm), _ptr(pos), _ptr(blocks),
                                            _ptr(sync),                                             _stream(stream)), "moe_route_schedule_permute")


def moe_coactivation_counts(ids, E: int):
    """ids: host int array [n_batches, ...] -> (c [E], a [E,E]) float64 host arrays."""
    import numpy as np
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    nb = ids.shape[0]
    pairs = int(ids.size // nb) if nb else 0
    c = np.empty(E, dtype=np.float64)
    a = np.empty((E, E), dtype=np.float64)
    _check(lib().moe_coactivation_counts(ids.ctypes.data, nb, pairs, E, c.ctypes.data, a.ctypes.data),
           "moe_coactivation_counts")
    return c, a


def moe_replica_counts(c, n_inst: int, C: int):
    import numpy as np
    c = np.ascontiguousarray(c, dtype=np.float64)
    R = np.empty(len(c), dtype=np.int32)
    _check(lib().moe_replica_counts(len(c), n_inst, C, c.ctypes.data, R.ctypes.data), "moe_replica_counts")
    return R


def moe_place_replicas(n_inst: int, C: int, R, c, a):
    import numpy as np
    R = np.ascontiguousarray(R, dtype=np.int32)
    c = np.ascontiguousarray(c, dtype=np.float64)
    a = np.ascontiguousarray(a, dtype=np.float64)
    E = len(R)
    assert a.shape == (E, E) and c.shape == (E,)
    lay = np.empty(n_inst * C, dtype=np.int32)
    _check(lib().moe_place_replicas(E, n_inst, C, R.ctypes.data, c.ctypes.data, a.ctypes.data, lay.ctypes.data),
           "moe_place_replicas")
    return lay


def moe_scaling_solve(model, table, ne_values, B_values, lam: float, slo: float, n_max: int, ne_min: int,
                      B_max: float):
    """model: any object with the fields of moe_scaling_model.  Returns (n_a, n_e, B*, TPOT) or None."""
    import numpy as np
    m = moe_scaling_model(*[getattr(model, n) for n, _ in moe_scaling_model._fields_])
    table = np.ascontiguousarray(table, dtype=np.float64)
    ne = np.ascontiguousarray(ne_values, dtype=np.int32)
    Bs = np.ascontiguousarray(B_values, dtype=np.float64)
    assert table.shape == (len(ne), len(Bs))
    n_a, n_e = ctypes.c_int(0), ctypes.c_int(0)
    b_star, t = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().moe_scaling_solve(ctypes.byref(m), table.ctypes.data, ne.ctypes.data, len(ne), Bs.ctypes.data, len(Bs),
                                   lam, slo, n_max, ne_min, B_max, ctypes.byref(n_a), ctypes.byref(n_e),
                                   ctypes.byref(b_star), ctypes.byref(t)), "moe_scaling_solve")
    if n_a.value == 0:
        return None
    return n_a.value, n_e.value, b_star.value, t.value


def moe_front_sync_len(pl: Placement, T: int, k: int) -> int:
    return int(lib().moe_front_sync_len(pl.handle, T, k))


def moe_gate_sync_len(T: int) -> int:
    return int(lib().moe_gate_sync_len(T))


def moe_gate_route(X, Wr, bias, k: int, logits, topk_ids, topk_w, sync, mode: int = MOE_ROUTE_SOFTMAX,
                   renormalize: bool = True, n_group: int = 1, topk_group: int = 1, scale: float = 1.0,
                   stream=None) -> None:
    T, d_h = X.shape
    E = Wr.shape[0]
    cfg = moe_route_cfg(mode, int(renormalize), n_group, topk_group, scale)
    _check(lib().moe_gate_route(_ptr(X), _ptr(Wr), _ptr(bias), T, E, d_h, k, ctypes.byref(cfg), _ptr(logits),
                                _ptr(topk_ids), _ptr(topk_w), _ptr(sync), _stream(stream)), "moe_gate_route")


def moe_gate_route_schedule_permute(pl: Placement, g_self: int, X, Wr, bias, k: int, logits, topk_ids, topk_w, rid,
                                    act_rep, load, slot_count, slot_off, perm, pos, blocks, sync,
                                    mode: int = MOE_ROUTE_SOFTMAX, renormalize: bool = True, n_group: int = 1,
                                    topk_group: int = 1, scale: float = 1.0, stream=None) -> None:
    T, d_h = X.shape
    cfg = moe_route_cfg(mode, int(renormalize), n_group, topk_group, scale)
    _check(lib().moe_gate_route_schedule_permute(pl.handle, g_self, _ptr(X), _ptr(Wr), _ptr(bias), T, d_h, k,
                                                 ctypes.byref(cfg), _ptr(logits), _ptr(topk_ids), _ptr(topk_w),
                                                 _ptr(rid), _ptr(act_rep), _ptr(load), _ptr(slot_count),
                                                 _ptr(slot_off), _ptr(perm), _ptr(pos), _ptr(blocks), _ptr(sync),
                                                 _stream(stream)), "moe_gate_route_schedule_permute")


def moe_pack_weights_bf16(W13, W2, C: int, d_h: int, d_e: int, W13_packed, W2_packed, stream=None) -> None:
    _check(lib().moe_pack_weights_bf16(_ptr(W13), _ptr(W2), C, d_h, d_e, _ptr(W13_packed), _ptr(W2_packed),
                                       _stream(stream)), "moe_pack_weights_bf16")


def moe_workspace_bytes(T: int, k: int, C: int, d_h: int, d_e: int, dtype: int) -> int:
    return int(lib().moe_workspace_bytes(T, k, C, d_h, d_e, dtype))


def moe_workspace_init(workspace, stream=None) -> None:
    _check(lib().moe_workspace_init(_ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream(stream)), "moe_workspace_init")


def moe_workspace_status(workspace) -> int:
    st = ctypes.c_int(-1)
    _check(lib().moe_workspace_status(_ptr(workspace), ctypes.byref(st)), "moe_workspace_status")
    return st.value


def moe_grouped_ffn(X, W13, W2, T: int, k: int, C: int, d_h: int, d_e: int, dtype: int, slot_off, perm,
                    blocks, Yp, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().moe_grouped_ffn(_ptr(X), _ptr(W13), _ptr(W2), T, k, C, d_h, d_e, dtype, _ptr(slot_off),
                                 _ptr(perm), _ptr(blocks), _ptr(Yp), _ptr(workspace), ws_bytes, _stream(stream)),
           "moe_grouped_ffn")


_bench_lib: Optional[ctypes.CDLL] = None


def bench_lib() -> ctypes.CDLL:
    """libmoe_bench.so: the measurement helpers of bench.py (include/moe_bench.h)."""
    global _bench_lib
    if _bench_lib is None:
        if not os.path.exists(BENCH_LIB_PATH):
            raise MoeError(MOE_EINVAL, f"{BENCH_LIB_PATH} is missing: build it with `python -m paper_2512_13525_amd.build`")
        L = ctypes.CDLL(BENCH_LIB_PATH)
        L.moe_read_probe.restype = ctypes.c_int
        L.moe_read_probe.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_void_p]
        _bench_lib = L
    return _bench_lib


def moe_read_probe(src, nbytes: int, sink, workgroups: int = 512, loads_in_flight: int = 8, stream=None) -> None:
    rc = bench_lib().moe_read_probe(_ptr(src), nbytes, _ptr(sink), workgroups, loads_in_flight, _stream(stream))
    if rc != 0:
        raise MoeError(rc, f"moe_read_probe: {rc}")


def moe_grouped_ffn_static(X, W13, W2, T: int, k: int, C: int, d_h: int, d_e: int, dtype: int, slot_off, perm,
                           blocks, Yp, stream=None) -> None:
    _check(lib().moe_grouped_ffn_static(_ptr(X), _ptr(W13), _ptr(W2), T, k, C, d_h, d_e, dtype, _ptr(slot_off),
                                        _ptr(perm), _ptr(blocks), _ptr(Yp), _stream(stream)),
           "moe_grouped_ffn_static")


def moe_combine(Yp, pos, topk_w, T: int, k: int, d_h: int, dtype: int, Y, stream=None) -> None:
    _check(lib().moe_combine(_ptr(Yp), _ptr(pos), _ptr(topk_w), T, k, d_h, dtype, _ptr(Y), _stream(stream)),
           "moe_combine")


def moe_shared_dispatch(T: int, slot_off, perm, blocks, stream=None) -> None:
    _check(lib().moe_shared_dispatch(T, _ptr(slot_off), _ptr(perm), _ptr(blocks), _stream(stream)), "moe_shared_dispatch")


def moe_combine_shared(Yp, pos, topk_w, Ys, T: int, k: int, d_h: int, dtype: int, Y, stream=None) -> None:
    _check(lib().moe_combine_shared(_ptr(Yp), _ptr(pos), _ptr(topk_w), _ptr(Ys), T, k, d_h, dtype, _ptr(Y),
                                    _stream(stream)), "moe_combine_shared")


def moe_workspace_set_option(workspace, option: int, value: int, stream=None) -> None:
    _check(lib().moe_workspace_set_option(_ptr(workspace), workspace.numel() * workspace.element_size(), option, value,
                                          _stream(stream)), "moe_workspace_set_option")
