"""Pins for the oracle's gate (router linear layer).  CPU only.  Each pin is something other
than the oracle's own matmul call: a hand-worked example, explicit loops, special router
matrices whose logits are known without arithmetic, and linearity."""
import numpy as np
import pytest

from oracle import gating, routing
from paper_2512_13525_amd import workloads as W


def test_gate_hand_example():
    # worked by hand: rows of W_r are experts
    X = np.array([[1.0, 2.0], [3.0, 4.0]])
    Wr = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    z = gating.gate_logits(X, Wr)
    assert z.tolist() == [[1.0, 2.0, 3.0], [3.0, 4.0, 7.0]]
    zb = gating.gate_logits(X, Wr, bias=np.array([10.0, 0.0, -1.0]))
    assert zb.tolist() == [[11.0, 2.0, 2.0], [13.0, 4.0, 6.0]]
    assert gating.gate_logits_f32(X, Wr).dtype == np.float32


def test_gate_matches_explicit_loops():
    rng = np.random.default_rng(5)
    T, E, d = 5, 7, 11
    X = rng.standard_normal((T, d))
    Wr = rng.standard_normal((E, d))
    b = rng.standard_normal(E)
    z = gating.gate_logits(X, Wr, b)
    assert z.shape == (T, E)
    for i in range(T):
        for e in range(E):
            acc = 0.0
            for c in range(d):
                acc += X[i, c] * Wr[e, c]
            assert abs(z[i, e] - (acc + b[e])) < 1e-12


def test_gate_selector_matrix_copies_columns():
    # W_r row e = unit vector of column perm[e]: the logits are columns of X, nothing is summed
    rng = np.random.default_rng(6)
    T, d, E = 9, 12, 5
    X = rng.standard_normal((T, d))
    cols = rng.permutation(d)[:E]
    Wr = np.zeros((E, d))
    Wr[np.arange(E), cols] = 1.0
    np.testing.assert_array_equal(gating.gate_logits(X, Wr), X[:, cols])
    # and the selection that follows picks the largest of those columns
    ids, _ = routing.route_softmax(gating.gate_logits_f32(X, Wr), 2)
    for i in range(T):
        order = sorted(range(E), key=lambda e: (-np.float32(X[i, cols[e]]), e))
        assert ids[i].tolist() == order[:2]


def test_gate_is_linear_in_both_operands():
    rng = np.random.default_rng(7)
    X1, X2 = rng.standard_normal((2, 6, 16))
    W1, W2 = rng.standard_normal((2, 4, 16))
    np.testing.assert_allclose(gating.gate_logits(X1 + 2 * X2, W1),
                               gating.gate_logits(X1, W1) + 2 * gating.gate_logits(X2, W1), atol=1e-12)
    np.testing.assert_allclose(gating.gate_logits(X1, W1 - 3 * W2),
                               gating.gate_logits(X1, W1) - 3 * gating.gate_logits(X1, W2), atol=1e-12)
    # a transposed operand would not even have this symmetry: z(X, W)[i, e] == z(W, X)[e, i]
    np.testing.assert_allclose(gating.gate_logits(X1, W1), gating.gate_logits(W1, X1).T, atol=1e-12)


def test_selection_margin_hand_values():
    z = np.array([[5.0, 1.0, 4.0, 3.5, 0.0],      # sorted 5, 4, 3.5, 1, 0
                  [2.0, 2.0, 1.0, 0.0, -1.0]])
    assert gating.selection_margin(z, 2).tolist() == [0.5, 0.0]     # gaps (1, .5) / (0, 1)
    assert gating.selection_margin(z, 1).tolist() == [1.0, 0.0]
    assert gating.selection_margin(z, 5).tolist() == [0.5, 0.0]     # k == E: order inside only
    assert gating.selection_margin(z[:, :1], 1).tolist() == [np.inf, np.inf]


@pytest.mark.parametrize("cfg", [W.tiny(), W.dsv2lite(), W.qwen3(32)], ids=lambda c: c.name)
def test_generated_gate_has_unit_scale_logits_and_the_zipf_bias(cfg):
    X = W.activations(cfg)
    Wr, bias = W.router_weights(cfg)
    assert Wr.shape == (cfg.E, cfg.d_h) and X.shape == (cfg.T, cfg.d_h)
    if cfg.dtype == "bf16":
        np.testing.assert_array_equal(Wr, W.round_to_bf16(Wr))
    z0 = gating.gate_logits(X, Wr)
    assert 0.8 < z0.std() < 1.2
    if cfg.zipf_s != 0.0:
        np.testing.assert_allclose(bias, np.log(cfg.E * W.expert_popularity(cfg)), rtol=1e-6)
        np.testing.assert_allclose(gating.gate_logits(X, Wr, bias) - z0, np.broadcast_to(bias, z0.shape), atol=1e-9)
    else:
        assert bias is None
