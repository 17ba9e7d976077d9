"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments on the host before anything is launched.  CPU only: no compute call is made."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2512_13525_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="moe_janus.h"):
    src = open(os.path.join(ROOT, "include", header)).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", src)))


def test_header_symbols_are_exported():
    names = declared_functions()
    assert set(["moe_schedule", "moe_permute", "moe_grouped_ffn", "moe_combine", "moe_route"]) <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(names) == sorted(B.EXPORTS)
    # the measurement helpers of bench.py live in a library of their own
    bench = declared_functions("moe_bench.h")
    assert bench == sorted(B.BENCH_EXPORTS)
    for n in bench:
        assert hasattr(B.bench_lib(), n), n
        assert not hasattr(L, n), n


def test_strerror():
    L = B.lib()
    assert L.moe_strerror(0) == b"success"
    for code in (-1, -2, -3, -4, -5, -6):
        assert len(L.moe_strerror(code)) > 0
    assert b"unknown" in L.moe_strerror(-99)


def test_placement_validation_happens_on_host():
    L = B.lib()
    h = ctypes.c_void_p()

    def create(lay, E, n, C):
        arr = np.asarray(lay, dtype=np.int32)
        return L.moe_placement_create(ctypes.byref(h), E, n, C, arr.ctypes.data)

    assert create([0, 1, 0, 2, 1, -1], 4, 3, 2) == B.MOE_EPLACEMENT      # expert 3 has no replica
    assert create([0, 0, 1, 2, 1, 3], 4, 3, 2) == B.MOE_EPLACEMENT       # two replicas on one instance
    assert create([0, 1, 0, 2, 1, 4], 4, 3, 2) == B.MOE_EPLACEMENT       # id out of range
    assert create([0, 1, 0, 2, 1, -2], 4, 3, 2) == B.MOE_EPLACEMENT
    assert create([0], 0, 1, 1) == B.MOE_EINVAL
    assert create([0] * 2000, 2000, 1, 2000) == B.MOE_ESHAPE
    assert L.moe_placement_create(None, 1, 1, 1, None) == B.MOE_EINVAL
    assert not h
    L.moe_placement_destroy(None)                                          # no-op


def test_argument_validation_without_launch():
    L = B.lib()
    cfg = B.moe_route_cfg(B.MOE_ROUTE_SOFTMAX, 1, 1, 1, 1.0)
    assert L.moe_route(None, 4, 8, 2, None, None, None, None) == B.MOE_EINVAL
    assert L.moe_route(None, 4, 8, 9, ctypes.byref(cfg), None, None, None) == B.MOE_EINVAL     # k > E
    assert L.moe_route(None, 4, 4096, 2, ctypes.byref(cfg), None, None, None) == B.MOE_ESHAPE
    assert L.moe_route(None, 4, 8, 2, ctypes.byref(cfg), None, None, None) == B.MOE_EINVAL     # null buffers
    assert L.moe_route(None, 0, 8, 2, ctypes.byref(cfg), None, None, None) == B.MOE_OK         # T == 0
    g = B.moe_route_cfg(B.MOE_ROUTE_SIGMOID_GROUP, 1, 3, 2, 1.0)
    assert L.moe_route(None, 4, 8, 2, ctypes.byref(g), None, None, None) == B.MOE_ESHAPE       # 8 % 3
    assert L.moe_schedule(None, None, 4, 2, None, None, None, None) == B.MOE_EINVAL
    assert L.moe_schedule_baseline(None, None, 4, 2, 0, None, None, None, None) == B.MOE_EINVAL
    # gate: selection arguments, then the hidden size, then pointers; T == 0 launches nothing
    assert L.moe_front_sync_len(None, 4, 2) == 0
    assert L.moe_gate_sync_len(0) == 1 and L.moe_gate_sync_len(16) == 2 and L.moe_gate_sync_len(17) == 3
    gate = lambda T, E, d_h, k: L.moe_gate_route(None, None, None, T, E, d_h, k, ctypes.byref(cfg), None, None, None,
                                                 None, None)
    assert gate(4, 8, 64, 9) == B.MOE_EINVAL
    assert gate(4, 8, 48, 2) == B.MOE_ESHAPE
    assert gate(4, 8, 64, 2) == B.MOE_EINVAL
    assert L.moe_gate_route_schedule_permute(*([None, 0] + [None] * 3 + [4, 64, 2, ctypes.byref(cfg)] + [None] * 13)) == B.MOE_EINVAL
    assert L.moe_permute(None, 0, None, 4, 2, None, None, None, None, None, None) == B.MOE_EINVAL
    # FFN: shapes first, then pointers
    assert L.moe_grouped_ffn(None, None, None, 4, 2, 5, 100, 64, B.MOE_DTYPE_BF16, None, None, None, None, None, 0,
                             None) == B.MOE_ESHAPE
    assert L.moe_grouped_ffn(None, None, None, 4, 2, 5, 128, 64, B.MOE_DTYPE_BF16, None, None, None, None, None, 0,
                             None) == B.MOE_EINVAL
    assert L.moe_grouped_ffn(None, None, None, 4, 2, 5, 128, 64, 7, None, None, None, None, None, 0, None) == B.MOE_EINVAL
    assert L.moe_grouped_ffn(None, None, None, 0, 2, 5, 128, 64, B.MOE_DTYPE_BF16, None, None, None, None, None, 0,
                             None) == B.MOE_OK
    assert L.moe_combine(None, None, None, 4, 2, 130, B.MOE_DTYPE_F32, None, None) == B.MOE_ESHAPE
    assert L.moe_combine(None, None, None, 4, 2, 128, B.MOE_DTYPE_F32, None, None) == B.MOE_EINVAL
    assert L.moe_pack_weights_bf16(None, None, 2, 100, 64, None, None, None) == B.MOE_ESHAPE
    assert L.moe_workspace_init(None, 0, None) == B.MOE_EINVAL
    # one partly filled block per slot plus the full ones: C + T*k/R blocks of R rows
    assert L.moe_block_rows(128) == 32 and L.moe_block_rows(512) == B.MOE_FFN_BLOCK_ROWS == 64
    assert L.moe_max_blocks(128, 6, 17) == 17 + 128 * 6 // 32
    assert L.moe_max_blocks(16, 8, 36) == 36 + 16 * 8 // 32
    assert L.moe_max_blocks(512, 8, 36) == 36 + 512 * 8 // 64
    assert L.moe_block_list_len(128, 6, 17) == 4 * (1 + 41)
    assert L.moe_workspace_status(None, None) == B.MOE_EINVAL
    assert L.moe_workspace_set_option(None, 0, 0, 0, None) == B.MOE_EINVAL
    ws = L.moe_workspace_bytes(128, 6, 17, 2048, 1408, B.MOE_DTYPE_BF16)
    assert ws >= 128 * 6 * 1408 * 2 and ws % 256 == 0
    assert L.moe_workspace_bytes(64, 2, 5, 256, 512, B.MOE_DTYPE_F32) >= 64 * 2 * 512 * 4
