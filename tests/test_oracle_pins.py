"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle (oracle/rmsnorm_linear_oracle.c) is pinned to things other than
itself: hand-computed cases, exact rational arithmetic, algebraic invariants
of Eq. 1 + MatMul, and float64 library routines.  The last block plants
typical mistakes in a copy of the definition and checks that the pins catch
each of them.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads

H1 = dict(X=[[3, 4, 0], [1, 2, 2]], g=[1, 2, 0.5], W=[[1, 0], [0, 1], [2, -2]], eps=0.0)
H3 = dict(X=[[2, 2, 2], [-1, 0, 1]], g=[1, 1, 1], W=[[1, 0], [0, 1], [1, 1]], eps=5.0)


def _store(case, dtype):
    return (workloads.to_storage(np.array(case["X"], np.float32), dtype),
            workloads.to_storage(np.array(case["g"], np.float32), dtype),
            workloads.to_storage(np.array(case["W"], np.float32), dtype))


def _wide(a, dtype):
    return workloads.to_f32(a, dtype).astype(np.float64)


# ---------------------------------------------------------------- decoders
def test_f16_decoder_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = oracle.decode(bits.view(np.float16), "f16")
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_bf16_decoder_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = oracle.decode(bits, "bf16")
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_decoder_spot_values():
    assert oracle.decode_f16_scalar(0x3C00) == 1.0
    assert oracle.decode_f16_scalar(0xC000) == -2.0
    assert oracle.decode_f16_scalar(0x0001) == 2.0 ** -24
    assert oracle.decode_f16_scalar(0x7BFF) == 65504.0
    assert oracle.decode_bf16_scalar(0x3F80) == 1.0
    assert oracle.decode_bf16_scalar(0x4049) == 3.140625
    assert oracle.decode_bf16_scalar(0x0001) == 2.0 ** -133


# ---------------------------------------------------------------- hand cases
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("case_name,case", [("H1", H1), ("H3", H3)])
def test_hand_cases(golden_hand_cases, case_name, case, dtype):
    X, g, W = _store(case, dtype)          # all entries are exact in every storage type
    Z = oracle.rmsnorm_linear(X, g, W, dtype, case["eps"])
    want = golden_hand_cases[case_name]
    for (i, j), v in want.items():
        assert Z[i, j] == pytest.approx(v, rel=2e-15, abs=1e-300), (case_name, i, j)


def test_eps_placement_is_under_the_root(golden_hand_cases):
    """Row 0 of H3 is 4/3 with eps under the root; 4/7 if it were added to the RMS."""
    X, g, W = _store(H3, "f32")
    Z = oracle.rmsnorm_linear(X, g, W, "f32", 5.0)
    assert abs(Z[0, 0] - 4.0 / 3.0) < 1e-15
    assert abs(Z[0, 0] - 4.0 / 7.0) > 0.5


# ---------------------------------------------------------------- exact brute force
def test_exact_rational_brute_force():
    """Small integer inputs: Z^2 * (sum x^2 / K + eps) == B^2 exactly, B = (X*g) @ W in rationals."""
    rng = np.random.default_rng(7)
    for trial in range(20):
        M, K, N = rng.integers(1, 5), rng.integers(1, 7), rng.integers(1, 5)
        X = rng.integers(-4, 5, (M, K))
        X[X.sum(axis=1) == 0, 0] = 3                 # avoid all-zero rows (some may remain: add eps)
        g = rng.integers(1, 4, K)
        W = rng.integers(-3, 4, (K, N))
        eps = Fraction(int(rng.integers(0, 3)), 4) + Fraction(1, 8)   # exact in binary
        Z = oracle.rmsnorm_linear(X.astype(np.float32), g.astype(np.float32),
                                  W.astype(np.float32), "f32", float(eps))
        for i in range(M):
            ms = Fraction(int((X[i] ** 2).sum()), int(K)) + eps
            for n in range(N):
                B = sum(Fraction(int(X[i, k] * g[k] * W[k, n])) for k in range(K))
                z = Fraction(Z[i, n])
                # sign and magnitude, with no square root taken on the exact side
                assert (z > 0) == (B > 0) and (z < 0) == (B < 0)
                if B != 0:
                    rel = abs(z * z * ms - B * B) / (B * B)
                    assert rel < Fraction(1, 10 ** 14), (trial, i, n, float(rel))


# ---------------------------------------------------------------- invariants
def _rand(M, K, N, dtype, seed):
    w = workloads.make(M, K, N, dtype, 0.0, seed)
    return w.X, w.g, w.W


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_scale_invariance_eps0(dtype):
    """Y(cX) = Y(X) for c > 0 when eps = 0; powers of two keep the inputs exact."""
    X, g, W = _rand(5, 96, 17, dtype, 11)
    Z = oracle.rmsnorm_linear(X, g, W, dtype, 0.0)
    for c in (0.25, 4.0):
        Xc = workloads.to_storage(_wide(X, dtype) * c, dtype)
        assert np.array_equal(_wide(Xc, dtype), _wide(X, dtype) * c)
        Zc = oracle.rmsnorm_linear(Xc, g, W, dtype, 0.0)
        np.testing.assert_allclose(Zc, Z, rtol=1e-13, atol=1e-15)


def test_scale_invariance_breaks_with_eps():
    X, g, W = _rand(3, 64, 9, "f32", 12)
    Z = oracle.rmsnorm_linear(X, g, W, "f32", 1.0)
    Z4 = oracle.rmsnorm_linear(X * 4, g, W, "f32", 1.0)
    assert np.abs(Z4 - Z).max() > 1e-2


def test_unit_rms_rows_identity_weight():
    """g = 1, W = I, eps = 0: every output row has RMS exactly 1."""
    K = 64
    X = workloads.make(7, K, K, "bf16", 0.0, 13).X
    g = workloads.to_storage(np.ones(K, np.float32), "bf16")
    W = workloads.to_storage(np.eye(K, dtype=np.float32), "bf16")
    Z = oracle.rmsnorm_linear(X, g, W, "bf16", 0.0)
    np.testing.assert_allclose(np.sqrt((Z ** 2).mean(axis=1)), 1.0, rtol=1e-14)
    # and each row is the input row divided by its RMS
    x = _wide(X, "bf16")
    np.testing.assert_allclose(Z, x / np.sqrt((x * x).mean(axis=1, keepdims=True)), rtol=1e-14)


def test_linearity_homogeneity_permutations():
    rng = np.random.default_rng(14)
    X, g, W1 = _rand(4, 48, 10, "f32", 15)
    W2 = rng.standard_normal(W1.shape).astype(np.float32)
    eps = 1e-3
    f = lambda X_, g_, W_: oracle.rmsnorm_linear(np.ascontiguousarray(X_, np.float32),
                                                  np.ascontiguousarray(g_, np.float32),
                                                  np.ascontiguousarray(W_, np.float32), "f32", eps)
    Z1, Z2 = f(X, g, W1), f(X, g, W2)
    # additive in W up to the float32 rounding of W1 + W2: use exactly representable halves
    Ws = (W1.astype(np.float64) + W2.astype(np.float64))
    Zs = oracle.matmul_f64(oracle.rmsnorm_f64(X, g, eps), Ws)
    np.testing.assert_allclose(Zs, Z1 + Z2, rtol=1e-12, atol=1e-13)
    # homogeneous in g (factor 2 is exact)
    np.testing.assert_allclose(f(X, 2 * g, W1), 2 * Z1, rtol=1e-14)
    # column permutation of W permutes the columns of Z
    P = rng.permutation(W1.shape[1])
    np.testing.assert_array_equal(f(X, g, W1[:, P]), Z1[:, P])
    # joint permutation of the reduction index leaves Z unchanged up to summation order
    Q = rng.permutation(X.shape[1])
    np.testing.assert_allclose(f(X[:, Q], g[Q], W1[Q, :]), Z1, rtol=1e-11, atol=1e-13)
    # rows are independent: a permutation of rows permutes the rows of Z
    R = rng.permutation(X.shape[0])
    np.testing.assert_array_equal(f(X[R], g, W1), Z1[R])


def test_not_symmetric_in_operands():
    """Catches a transposed W or swapped g/X roles: a non-square case with distinct values."""
    X = np.array([[1, 2, 3]], np.float32)
    g = np.array([1, 1, 1], np.float32)
    W = np.array([[1, 2], [3, 4], [5, 6]], np.float32)
    Z = oracle.rmsnorm_linear(X, g, W, "f32", 0.0)
    r = np.sqrt(14.0 / 3.0)
    np.testing.assert_allclose(Z, [[22 / r, 28 / r]], rtol=1e-15)


# ---------------------------------------------------------------- the paper's rewrite is an identity
def test_reordered_division_identity():
    """B = (X*g) @ W, A = sum x^2 (case study: the form with the division moved behind the product): Z = B / sqrt(A/K + eps)."""
    for dtype, seed in (("f16", 21), ("bf16", 22), ("f32", 23)):
        w = workloads.make(9, 200, 33, dtype, 1e-5, seed, outlier_frac=0.2)
        Z = oracle.rmsnorm_linear(w.X, w.g, w.W, dtype, w.eps)
        x, g, W = _wide(w.X, dtype), _wide(w.g, dtype), _wide(w.W, dtype)
        B = (x * g) @ W
        A = (x * x).sum(axis=1, keepdims=True)
        np.testing.assert_allclose(Z, B / np.sqrt(A / x.shape[1] + w.eps), rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- library routines
@pytest.mark.parametrize("name", ["tiny", "decode", "qkv"])
def test_against_float64_library(name):
    import torch
    w = workloads.config(name)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    x, g, W = _wide(w.X, w.dtype), _wide(w.g, w.dtype), _wide(w.W, w.dtype)
    ref_np = ((x / np.sqrt((x * x).mean(-1, keepdims=True) + w.eps)) * g) @ W
    scale = np.sqrt((ref_np ** 2).mean())
    assert np.abs(Z - ref_np).max() <= 1e-12 * scale
    xt = torch.from_numpy(x)
    ref_t = torch.nn.functional.rms_norm(xt, (x.shape[1],), torch.from_numpy(g), eps=w.eps) @ torch.from_numpy(W)
    assert np.abs(Z - ref_t.numpy()).max() <= 1e-12 * scale
    assert 0.9 < scale < 1.2           # W ~ N(0, 1/K) in variance: rms(Y) ~ sqrt(E g^2) ~ 1.04


def test_row_subset_equals_full_rows():
    w = workloads.make(40, 128, 24, "bf16", 1e-5, 31)
    full = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    rows = np.array([3, 17, 39, 0])
    sub = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=rows)
    np.testing.assert_array_equal(sub, full[rows])


def test_unfused_pair_composes():
    w = workloads.make(6, 80, 12, "f16", 1e-6, 32)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Yn = oracle.rmsnorm(w.X, w.g, w.dtype, w.eps)
    np.testing.assert_allclose(oracle.matmul_f64(Yn, _wide(w.W, w.dtype)), Z, rtol=1e-15, atol=0)


def test_matmul_f64_against_exact_integers():
    rng = np.random.default_rng(33)
    a = rng.integers(-9, 10, (5, 13)).astype(np.float64)
    b = rng.integers(-9, 10, (13, 4)).astype(np.float64)
    want = [[sum(int(a[i, k]) * int(b[k, n]) for k in range(13)) for n in range(4)] for i in range(5)]
    np.testing.assert_array_equal(oracle.matmul_f64(a, b), np.array(want, np.float64))


def test_zero_row():
    X = np.zeros((2, 8), np.float32)
    X[1] = 1
    g = np.ones(8, np.float32)
    W = np.ones((8, 3), np.float32)
    Z = oracle.rmsnorm_linear(X, g, W, "f32", 1e-6)
    assert np.all(Z[0] == 0.0)
    with np.errstate(all="ignore"):
        Z0 = oracle.rmsnorm_linear(X, g, W, "f32", 0.0)
    assert np.all(np.isnan(Z0[0])) and np.allclose(Z0[1], 8.0)


def test_bad_arguments_rejected():
    X = np.zeros((2, 8), np.float32)
    g = np.ones(8, np.float32)
    W = np.ones((8, 3), np.float32)
    with pytest.raises(RuntimeError):
        oracle.rmsnorm_linear(X, g, W, "f32", 0.0, rows=np.array([2]))
    with pytest.raises(TypeError):
        oracle.rmsnorm_linear(X.astype(np.float64), g, W, "f32", 0.0)


# ---------------------------------------------------------------- the pins have teeth
def _definition(x, g, W, eps, mistake=None):
    """Eq. 1 + MatMul in numpy float64 with one planted mistake (CPU only, never the oracle)."""
    K = x.shape[1]
    ms = (x * x).mean(-1, keepdims=True)
    if mistake == "eps_outside_root":
        r = np.sqrt(ms) + eps
    elif mistake == "no_eps":
        r = np.sqrt(ms)
    elif mistake == "rms_of_xg":
        r = np.sqrt(((x * g) ** 2).mean(-1, keepdims=True) + eps)
    elif mistake == "sum_not_mean":
        r = np.sqrt(ms * K + eps)
    elif mistake == "no_root":
        r = ms + eps
    else:
        r = np.sqrt(ms + eps)
    y = x / r if mistake == "drop_g" else x * g / r
    if mistake == "w_read_transposed":
        # read W's buffer as if it were stored [N][K]
        return y @ W.reshape(W.shape[1], W.shape[0]).T
    return y @ W


@pytest.mark.parametrize("mistake", ["eps_outside_root", "no_eps", "rms_of_xg", "sum_not_mean",
                                     "no_root", "drop_g", "w_read_transposed"])
def test_pins_catch_planted_mistakes(golden_hand_cases, mistake):
    caught = False
    for name, case in (("H1", H1), ("H3", H3)):
        x, g, W = (np.array(case[k], np.float64) for k in ("X", "g", "W"))
        Z = _definition(x, g, W, case["eps"], mistake)
        for (i, j), v in golden_hand_cases[name].items():
            if abs(Z[i, j] - v) > 1e-9:
                caught = True
    assert caught, mistake
    # and the unmutated definition passes the same pins
    for name, case in (("H1", H1), ("H3", H3)):
        x, g, W = (np.array(case[k], np.float64) for k in ("X", "g", "W"))
        Z = _definition(x, g, W, case["eps"])
        for (i, j), v in golden_hand_cases[name].items():
            assert abs(Z[i, j] - v) < 1e-14
