"""moe_grouped_ffn_static, the entry point for callers that cannot allocate: called through the C
ABI, two calls in a row on one GPU (the second with a smaller input, so it meets what the first left
in the shared array), each compared bit for bit with moe_grouped_ffn on a caller-owned workspace,
and with the oracle to the bar of the other FFN tests."""
import numpy as np
import pytest
import torch

from paper_2512_13525_amd import binding as B
from paper_2512_13525_amd import workloads as W
from paper_2512_13525_amd.layer import LayerStep, to_device_bf16

from helpers import OracleRun, rel_fro

pytestmark = pytest.mark.gpu


def run_both(cfg):
    """Dispatch through the library, then the FFN through both entry points on the same inputs."""
    orc = OracleRun(cfg, only_activated=cfg.dtype == "bf16")
    st = LayerStep(cfg, orc.lay, orc.g_self)
    if cfg.dtype == "bf16":
        st.set_weights(to_device_bf16(orc.W13), to_device_bf16(orc.W2))
        X = to_device_bf16(orc.X)
    else:
        st.set_weights(torch.from_numpy(orc.W13).cuda(), torch.from_numpy(orc.W2).cuda())
        X = torch.from_numpy(orc.X).cuda()
    st.front(torch.from_numpy(orc.logits).cuda())
    n_local = len(orc.perm)
    st.Yp.fill_(123.0)
    st.ffn(X)
    torch.cuda.synchronize()
    want = st.Yp.clone()
    assert B.moe_workspace_status(st.workspace) == 0
    got = torch.full_like(st.Yp, 123.0)
    c = cfg
    B.moe_grouped_ffn_static(X, st.W13, st.W2, c.T, c.k, c.C, c.d_h, c.d_e, st.dtype, st.slot_off, st.perm, st.blocks, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    tol = 2e-2 if cfg.dtype == "bf16" else 1e-5
    assert rel_fro(got[:n_local].cpu().numpy(), orc.Yp) < tol
    assert (got[n_local:] == 123.0).all()
    return st, X, got


def test_static_scratch_entry_point_two_calls_in_a_row():
    big = W.qwen3(256)                                       # a full-size decode configuration
    small = W.MoEConfig("after_big", E=16, k=4, d_h=256, d_e=128, T=48, n_inst=2, C=9, zipf_s=1.0, seed=1)
    st, X, got = run_both(big)
    run_both(small)                                          # smaller input on the array the first call used
    run_both(W.tiny())                                       # the fp32 kernels share the array too
    # and the first shape again: bit-identical to its first result
    c = big
    again = torch.full_like(got, 123.0)
    B.moe_grouped_ffn_static(X, st.W13, st.W2, c.T, c.k, c.C, c.d_h, c.d_e, st.dtype, st.slot_off, st.perm, st.blocks, again)
    torch.cuda.synchronize()
    assert torch.equal(again, got)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    c = W.stress(8192, 1.25, 0.8)
    assert B.moe_workspace_bytes(c.T, c.k, c.C, c.d_h, c.d_e, B.MOE_DTYPE_BF16) > B.MOE_FFN_STATIC_SCRATCH_BYTES
    with pytest.raises(B.MoeError) as ei:
        B.moe_grouped_ffn_static(None, None, None, c.T, c.k, c.C, c.d_h, c.d_e, B.MOE_DTYPE_BF16, None, None, None, None)
    assert ei.value.code == B.MOE_EWORKSPACE
