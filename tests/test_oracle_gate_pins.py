"""Pins for the oracle's GatedMLP gate, Y = SiLU(gate) * up (no GPU needed).

The paper's GatedMLP benchmark runs two products of the same input, applies SiLU to one and
multiplies elementwise with the other.  oracle.silu_mul_f64 is pinned to closed forms worked out
by hand (tests/golden/hand_cases.txt, cases G1 and G2, written by make_hand_cases.py in 40-digit
decimals), to identities of SiLU, to float64 library sigmoids, and the pins are shown to catch
planted mistakes.
"""
import math

import numpy as np
import pytest

import oracle
import workloads
from test_oracle_pins import H1, _store

LN3, LN7 = math.log(3.0), math.log(7.0)
G1_Z = [[0.0, LN3, -LN3, LN7, 5.0, 2.0, 4.0, -1.0]]


def test_gate_closed_forms(golden_hand_cases):
    Y = oracle.silu_mul_f64(np.array(G1_Z))
    for (i, j), v in golden_hand_cases["G1"].items():
        assert Y[i, j] == pytest.approx(v, rel=4e-16, abs=1e-300), (i, j)
    assert Y[0, 0] == 0.0


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_gated_block_hand_case(golden_hand_cases, dtype):
    """H1's inputs through the whole gated block, H = 1 (gate = column 0, up = column 1)."""
    X, g, W = _store(H1, dtype)
    Y = oracle.rmsnorm_gated_mlp(X, g, W, dtype, 0.0)
    assert Y.shape == (2, 1)
    for (i, j), v in golden_hand_cases["G2"].items():
        assert Y[i, j] == pytest.approx(v, rel=4e-15), (i, j)


def test_silu_odd_part_identity():
    """SiLU(v) - SiLU(-v) = v  (1/(1+e^-v) + 1/(1+e^v) = 1)."""
    rng = np.random.default_rng(11)
    v = rng.standard_normal(4096) * 4.0
    ones = np.ones_like(v)
    a = oracle.silu_mul_f64(np.stack([v, ones], 1).reshape(-1, 2))[:, 0]
    b = oracle.silu_mul_f64(np.stack([-v, ones], 1).reshape(-1, 2))[:, 0]
    np.testing.assert_allclose(a - b, v, rtol=0, atol=4e-15)


def test_silu_limits_and_sign():
    z = np.array([[40.0, 1.0], [-40.0, 1.0], [1e-9, 1.0], [3.0, -2.0], [3.0, 0.0]])
    y = oracle.silu_mul_f64(z)[:, 0]
    assert y[0] == pytest.approx(40.0, rel=1e-15)            # SiLU(v) -> v
    assert abs(y[1]) < 1e-15 and y[1] < 0                    # SiLU(v) -> v e^v, below zero
    assert y[2] == pytest.approx(0.5e-9, rel=1e-8)           # SiLU(v) ~ v/2 near 0
    assert y[3] == pytest.approx(-2.0 * 3.0 / (1.0 + math.exp(-3.0)), rel=1e-15)
    assert y[4] == 0.0


def test_gate_is_linear_in_the_up_half():
    rng = np.random.default_rng(5)
    gate, u1, u2 = (rng.standard_normal((7, 33)) for _ in range(3))
    y = lambda u: oracle.silu_mul_f64(np.concatenate([gate, u], 1))
    np.testing.assert_allclose(y(2.5 * u1 - 0.75 * u2), 2.5 * y(u1) - 0.75 * y(u2), rtol=0, atol=1e-14)
    assert np.all(y(np.zeros_like(u1)) == 0.0)


def test_gate_against_library_sigmoids():
    torch = pytest.importorskip("torch")
    from scipy.special import expit
    rng = np.random.default_rng(9)
    z = rng.standard_normal((64, 512)) * 3.0
    want_np = z[:, :256] * expit(z[:, :256]) * z[:, 256:]
    zt = torch.from_numpy(z)
    want_t = (torch.nn.functional.silu(zt[:, :256]) * zt[:, 256:]).numpy()
    got = oracle.silu_mul_f64(z)
    np.testing.assert_allclose(got, want_np, rtol=1e-14, atol=1e-300)
    np.testing.assert_allclose(got, want_t, rtol=1e-14, atol=1e-300)


def test_gated_block_against_numpy_on_a_config():
    w = workloads.make(16, 1024, 512, "bf16", 1e-5, 77)
    x, g, W = (workloads.to_f32(a, "bf16").astype(np.float64) for a in (w.X, w.g, w.W))
    zn = (x / np.sqrt((x * x).mean(-1, keepdims=True) + np.float64(np.float32(1e-5)))) * g @ W
    want = zn[:, :256] / (1.0 + np.exp(-zn[:, :256])) * zn[:, 256:]
    got = oracle.rmsnorm_gated_mlp(w.X, w.g, w.W, "bf16", w.eps)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


def test_scale_invariance_of_the_gated_block():
    """eps = 0: the gated block inherits Y(cX) = Y(X) for c > 0 (powers of two keep inputs exact)."""
    w = workloads.make(4, 256, 64, "f16", 0.0, 3)
    X2 = (w.X.astype(np.float32) * 4.0).astype(np.float16)
    a = oracle.rmsnorm_gated_mlp(w.X, w.g, w.W, "f16", 0.0)
    b = oracle.rmsnorm_gated_mlp(X2, w.g, w.W, "f16", 0.0)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-15)


def _gate_definition(z, mistake=None):
    H = z.shape[1] // 2
    gate, up = (z[:, H:], z[:, :H]) if mistake == "halves_swapped" else (z[:, :H], z[:, H:])
    if mistake == "sigmoid_only":
        return 1.0 / (1.0 + np.exp(-gate)) * up
    if mistake == "exp_sign":
        return gate / (1.0 + np.exp(gate)) * up
    if mistake == "no_up":
        return gate / (1.0 + np.exp(-gate))
    if mistake == "silu_on_both":
        return gate / (1.0 + np.exp(-gate)) * (up / (1.0 + np.exp(-up)))
    if mistake == "interleaved_halves":
        return z[:, 0::2] / (1.0 + np.exp(-z[:, 0::2])) * z[:, 1::2]
    return gate / (1.0 + np.exp(-gate)) * up


@pytest.mark.parametrize("mistake", ["halves_swapped", "sigmoid_only", "exp_sign", "no_up", "silu_on_both",
                                     "interleaved_halves"])
def test_gate_pins_catch_planted_mistakes(golden_hand_cases, mistake):
    Y = _gate_definition(np.array(G1_Z), mistake)
    assert any(abs(Y[i, j] - v) > 1e-9 for (i, j), v in golden_hand_cases["G1"].items()), mistake
    Y = _gate_definition(np.array(G1_Z))
    assert all(abs(Y[i, j] - v) < 1e-14 for (i, j), v in golden_hand_cases["G1"].items())
