"""The nTrans chain y = Norm(x + alpha (.) Norm(h - x)): oracle pins (CPU) and GPU parity.

Norm is read as Eq. 1 without a gain (v / sqrt(mean v^2 + eps)); the paper does not say which
normalisation its nTrans benchmark uses.  Bar on the GPU: the plain block's, max |err| <=
2e-2 rms(Y) for 16-bit types (rows of Y have unit RMS), 1e-5 for fp32.
"""
import numpy as np
import pytest

import oracle
import workloads
from util import compare, to_device, to_host_f64


def _make(M, D, dtype, seed, alpha_scale=0.3):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, D), dtype=np.float32)
    h = rng.standard_normal((M, D), dtype=np.float32)
    a = (rng.uniform(0.0, 1.0, D) * alpha_scale).astype(np.float32)
    return tuple(workloads.to_storage(v, dtype) for v in (x, h, a))


def _wide(a, dtype):
    return workloads.to_f32(a, dtype).astype(np.float64)


def test_hand_case(golden_hand_cases):
    x = np.array([[1, 2, 2]], np.float32); h = np.array([[4, 6, 2]], np.float32); a = np.array([1, 0.5, 3], np.float32)
    for dtype in ("f32", "f16", "bf16"):                 # every entry is exact in every storage type
        Y = oracle.ntrans(*(workloads.to_storage(v, dtype) for v in (x, h, a)), dtype, 0.0)
        for (i, j), v in golden_hand_cases["N1"].items():
            assert Y[i, j] == pytest.approx(v, rel=4e-15)


def test_rows_have_unit_rms_and_special_cases():
    x, h, a = _make(9, 520, "bf16", 1)
    Y = oracle.ntrans(x, h, a, "bf16", 0.0)
    np.testing.assert_allclose(np.sqrt((Y ** 2).mean(1)), 1.0, rtol=1e-14)
    xw = _wide(x, "bf16")
    normx = xw / np.sqrt((xw ** 2).mean(1, keepdims=True))
    np.testing.assert_allclose(oracle.ntrans(x, h, np.zeros_like(a), "bf16", 0.0), normx, rtol=1e-14)   # alpha = 0
    eps = 1e-3                                                                                           # h = x: inner norm of 0 is 0
    np.testing.assert_allclose(oracle.ntrans(x, x, a, "bf16", eps),
                               xw / np.sqrt((xw ** 2).mean(1, keepdims=True) + eps), rtol=1e-14)
    neg = lambda b: (b ^ np.uint16(0x8000))                                                              # bf16 sign flip
    np.testing.assert_allclose(oracle.ntrans(neg(x), neg(h), a, "bf16", 0.0), -Y, rtol=1e-15)            # odd in (x, h)


def test_against_library_float64():
    torch = pytest.importorskip("torch")
    x, h, a = _make(17, 1032, "f16", 2)
    xw, hw, aw = (_wide(v, "f16") for v in (x, h, a))
    eps = float(np.float32(1e-6))
    norm = lambda v: v / np.sqrt((v * v).mean(-1, keepdims=True) + eps)
    np.testing.assert_allclose(oracle.ntrans(x, h, a, "f16", eps), norm(xw + aw * norm(hw - xw)), rtol=1e-13)
    F = torch.nn.functional
    xt, ht, at = (torch.from_numpy(v) for v in (xw, hw, aw))
    want = F.rms_norm(xt + at * F.rms_norm(ht - xt, (1032,), eps=eps), (1032,), eps=eps).numpy()
    np.testing.assert_allclose(oracle.ntrans(x, h, a, "f16", eps), want, rtol=1e-12)


@pytest.mark.parametrize("mistake", ["h_plus_x", "norm_h_minus_x", "no_outer_norm", "alpha_outside", "sum_not_mean"])
def test_hand_case_catches_planted_mistakes(golden_hand_cases, mistake):
    x = np.array([[1, 2, 2]], np.float64); h = np.array([[4, 6, 2]], np.float64); a = np.array([1, 0.5, 3], np.float64)
    norm = (lambda v: v / np.sqrt((v * v).sum(-1, keepdims=True))) if mistake == "sum_not_mean" else \
           (lambda v: v / np.sqrt((v * v).mean(-1, keepdims=True)))
    if mistake == "h_plus_x":
        y = norm(x + a * norm(h + x))
    elif mistake == "norm_h_minus_x":
        y = norm(x + a * (norm(h) - x))
    elif mistake == "no_outer_norm":
        y = x + a * norm(h - x)
    elif mistake == "alpha_outside":
        y = a * norm(x + norm(h - x))
    else:
        y = norm(x + a * norm(h - x))
    assert any(abs(y[i, j] - v) > 1e-9 for (i, j), v in golden_hand_cases["N1"].items())
    good = lambda v: v / np.sqrt((v * v).mean(-1, keepdims=True))
    y = good(x + a * good(h - x))
    assert all(abs(y[i, j] - v) < 1e-14 for (i, j), v in golden_hand_cases["N1"].items())


# ------------------------------------------------------------------------------------ GPU parity
@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("M,D", [(1, 8), (3, 100), (5, 520), (16, 2048), (7, 4096), (33, 8192), (4, 8200), (2, 20000),
                                 (1000, 2048)])
def test_gpu_parity(M, D, dtype):
    import torch
    import paper_2405_05751_amd as rl
    x, h, a = _make(M, D, dtype, 8000 + M + D)
    eps = float(np.float32(1e-6))
    Y = rl.rl_ntrans(to_device(x, dtype), to_device(h, dtype), to_device(a, dtype), eps)
    torch.cuda.synchronize()
    compare(to_host_f64(Y, dtype), oracle.ntrans(x, h, a, dtype, eps), dtype, f"ntrans {M}x{D} {dtype}")


@pytest.mark.gpu
def test_gpu_zero_difference_rows_and_canaries():
    import torch
    import paper_2405_05751_amd as rl
    x, h, a = _make(6, 1032, "bf16", 8100)
    h[2] = x[2]                                          # inner norm of a zero row
    eps = float(np.float32(1e-5))
    pad, n = 512, 6 * 1032
    buf = torch.full((pad + n + pad,), 99.0, dtype=torch.bfloat16, device="cuda")
    Y = buf[pad:pad + n].view(6, 1032)
    rl.rl_ntrans(to_device(x, "bf16"), to_device(h, "bf16"), to_device(a, "bf16"), eps, Y)
    torch.cuda.synchronize()
    assert torch.all(buf[:pad] == 99.0) and torch.all(buf[pad + n:] == 99.0)
    compare(to_host_f64(Y, "bf16"), oracle.ntrans(x, h, a, "bf16", eps), "bf16", "ntrans zero difference")
    with np.errstate(all="ignore"):
        want = oracle.ntrans(x, h, a, "bf16", 0.0)       # eps = 0: that row is NaN (0/0) on both sides
    Y0 = rl.rl_ntrans(to_device(x, "bf16"), to_device(h, "bf16"), to_device(a, "bf16"), 0.0)
    torch.cuda.synchronize()
    compare(to_host_f64(Y0, "bf16"), want, "bf16", "ntrans eps=0")
