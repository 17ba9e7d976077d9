"""Pins for the oracle's scaling procedure (Sec. 3.5: Eq. 1a-1c, Eq. 2, Eq. 3, Alg. 2) and the
same checks on the library's host implementation.  CPU only."""
import ctypes

import numpy as np
import pytest

from oracle import scaling as S
from paper_2512_13525_amd import binding as B


def model(**kw):
    base = dict(L=4, c_a=50e-6, alpha=2e-6, c_kv=1e-9, beta=2e-6, c_e=30e-6, comm0=10e-6, comm1=0.05e-6,
                S_ctx=1000.0, mem_budget=100.0, mem_fixed=10.0, mem_per_token=1e-3)
    base.update(kw)
    return S.Model(**base)


NE = [2, 4, 8]
BS = [1.0, 16.0, 64.0, 256.0]
TABLE = np.array([[2.0, 14.0, 30.0, 32.0], [1.5, 9.0, 15.0, 16.0], [1.0, 5.0, 7.5, 8.0]])


def test_tpot_is_eq1_term_by_term():
    m = model()
    # b = 40: attention = max(50e-6, 2e-6*40 + 1e-9*40*1000 = 120e-6) = 120e-6
    # moe = 2e-6*10 + 30e-6 = 50e-6; comm = 10e-6 + 0.05e-6*80 = 14e-6; 4 layers
    assert S.tpot(m, 10.0, 80.0, 2) == pytest.approx(4 * (120e-6 + 50e-6 + 14e-6), rel=1e-12)
    # small batch: the memory-bound plateau c_a wins
    assert S.tpot(m, 1.0, 2.0, 2) == pytest.approx(4 * (50e-6 + 32e-6 + 10.1e-6), rel=1e-12)


def test_lookup_interpolates_and_clamps():
    assert S.a_max_lookup(TABLE, NE, BS, 4, 16.0) == 9.0
    assert S.a_max_lookup(TABLE, NE, BS, 4, 40.0) == pytest.approx(9.0 + 0.5 * 6.0)
    assert S.a_max_lookup(TABLE, NE, BS, 4, 0.5) == 1.5 and S.a_max_lookup(TABLE, NE, BS, 4, 1e6) == 16.0
    assert S.a_max_lookup(TABLE, NE, BS, 3, 16.0) is None


def test_steady_batch_closed_form_when_tpot_is_linear():
    # flat a_max table and no plateau: TPOT = p + q*B, so B* = lambda*p / (1 - lambda*q)
    m = model(c_a=0.0, c_kv=0.0)
    flat = np.full((3, 4), 10.0)
    lam, n_a = 2.0e4, 2
    p = m.L * (m.beta * 10.0 + m.c_e + m.comm0)
    q = m.L * (m.alpha / n_a + m.comm1)
    Bs = S.steady_batch(m, flat, NE, BS, lam, n_a, 4, 1e4)
    assert Bs == pytest.approx(lam * p / (1 - lam * q), rel=1e-9)
    assert Bs == pytest.approx(lam * S.tpot(m, 10.0, Bs, n_a), rel=1e-9)           # Little's law holds at B*
    # boundary cases named by the section
    assert S.steady_batch(m, flat, NE, BS, 1.0, n_a, 4, 1e4) == 1.0                # light load
    assert S.steady_batch(m, flat, NE, BS, 1e9, n_a, 4, 1e4) is None               # cannot sustain


def brute_force(m, table, lam, slo, n_max, ne_min, B_max):
    """Independent search: fixed point by a dense scan for the sign change of the residual."""
    best = None
    grid = np.linspace(1.0, B_max, 200001)
    for n_a in range(1, n_max + 1):
        for n_e in range(ne_min, n_max + 1):
            if n_e not in NE:
                continue
            a = np.interp(grid, BS, table[NE.index(n_e)])
            b = grid / n_a
            T = m.L * (np.maximum(m.c_a, m.alpha * b + m.c_kv * b * m.S_ctx) + m.beta * a + m.c_e + m.comm0 + m.comm1 * grid)
            f = grid - lam * T
            if f[0] >= 0:
                i = 0
            elif f[-1] < 0:
                continue
            else:
                i = int(np.argmax(f >= 0))
            if T[i] > slo or m.mem_fixed + m.mem_per_token * b[i] * m.S_ctx > m.mem_budget:
                continue
            if best is None or n_a + n_e < best[0] + best[1]:
                best = (n_a, n_e, grid[i], T[i])
    return best


@pytest.mark.parametrize("lam", [2e3, 2e4, 1e5, 3e5, 1e6])
@pytest.mark.parametrize("slo", [0.6e-3, 1.0e-3, 3.0e-3])
def test_alg2_against_brute_force_and_library(lam, slo):
    m = model()
    got = S.solve(m, TABLE, NE, BS, lam, slo, 8, 2, 256.0)
    ref = brute_force(m, TABLE, lam, slo, 8, 2, 256.0)
    lib = B.moe_scaling_solve(m, TABLE, NE, BS, lam, slo, 8, 2, 256.0)
    if ref is None:
        assert got is None and lib is None
        return
    assert got is not None and got[:2] == ref[:2]
    assert got[2] == pytest.approx(ref[2], abs=2e-3) and got[3] == pytest.approx(ref[3], rel=1e-4)
    assert got[3] <= slo
    assert lib is not None and lib[:2] == got[:2]
    assert lib[2] == pytest.approx(got[2], rel=1e-12) and lib[3] == pytest.approx(got[3], rel=1e-12)


def test_alg2_outcomes_cover_both_answers():
    m = model()
    outcomes = {S.solve(m, TABLE, NE, BS, lam, slo, 8, 2, 256.0) is None
                for lam in (2e3, 1e6) for slo in (0.6e-3, 3.0e-3)}
    assert outcomes == {True, False}
    # more demand never needs fewer GPUs
    sizes = []
    for lam in (2e3, 2e4, 1e5, 2e5):
        r = S.solve(m, TABLE, NE, BS, lam, 3.0e-3, 8, 2, 256.0)
        sizes.append(r[0] + r[1] if r else 99)
    assert sizes == sorted(sizes)


def test_memory_constraint_discards_configurations():
    m = model(mem_per_token=1e-3, mem_budget=10.0 + 1e-3 * 20 * 1000.0)             # room for b = 20 per attention GPU
    r = S.solve(m, TABLE, NE, BS, 1e5, 3.0e-3, 8, 2, 256.0)
    free = S.solve(model(mem_budget=1e9), TABLE, NE, BS, 1e5, 3.0e-3, 8, 2, 256.0)
    assert r is not None and free is not None
    assert r[2] / r[0] <= 20.0 + 1e-9
    assert r[0] + r[1] >= free[0] + free[1]
    lib = B.moe_scaling_solve(m, TABLE, NE, BS, 1e5, 3.0e-3, 8, 2, 256.0)
    assert lib[:2] == r[:2]


def test_library_rejects_bad_arguments():
    L = B.lib()
    assert L.moe_scaling_solve(None, None, None, 0, None, 0, 1.0, 1.0, 1, 1, 1.0, None, None, None, None) == B.MOE_EINVAL
