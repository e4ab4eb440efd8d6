"""Parity of the fp32 path (matrix cores on fp32 operands, two levels of accumulators) against the fp64
oracle, through the C ABI.  Needs an MI355X.

Bar: max |err| <= 1e-5 * rms(Y), per row and overall (the tolerance the benchmark spec states for fp32).  What the
arithmetic gives: products are exact in fp32, a first-level sum takes 128 terms, the second level K / 512
per wave, then 4 waves and up to 16 slabs: a few ulps of 6e-8, measured 2e-7 to 6e-7."""
import numpy as np
import pytest

import oracle
import workloads
from util import compare, compare_gated, to_device, to_host_f64, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rl():
    import torch
    import paper_2405_05751_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


def _run(rl, w, variant="auto", slabs=0, rows=None):
    import torch
    X, g, W = upload(w)
    Y = torch.empty(w.M, w.N, dtype=torch.float32, device="cuda")
    rl.rmsnorm_linear_ex(X, g, W, w.eps, Y, variant=variant, slabs=slabs)
    torch.cuda.synchronize()
    used = rl.rl_last_variant()
    if rows is not None:
        Y = Y[torch.from_numpy(np.asarray(rows)).cuda()]
    return to_host_f64(Y, "f32"), used


# row counts around the 16-row blocks and the 64-row row blocks; K around the 64-row runs, the ring of
# three and the 8-run chunks; N around the 64-column tiles (multiples of 4)
@pytest.mark.parametrize("M,K,N", [(1, 4, 4), (1, 64, 64), (1, 4096, 4096), (2, 68, 60), (15, 520, 132), (16, 1024, 4096),
                                   (17, 196, 68), (33, 2052, 516), (48, 512, 1000), (64, 4096, 1028), (65, 260, 64),
                                   (100, 1000, 200), (128, 8192, 256), (300, 516, 520), (1000, 772, 1284)])
def test_fp32_shapes(rl, M, K, N):
    w = workloads.make(M, K, N, "f32", 1e-6, 4100 + M + K + N, outlier_frac=0.02 if M >= 48 else 0.0)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w)
    assert used == "f32", used
    ratio, _ = compare(Y, Z, "f32", f"fp32 {M}x{K}x{N}")
    print(f"fp32 {M}x{K}x{N}: max|err|/rms(Y) = {ratio:.3e}")
    assert ratio <= 2e-6, ratio


@pytest.mark.parametrize("slabs", [1, 2, 3, 5, 8, 16])
@pytest.mark.parametrize("M,K,N", [(5, 4100, 328), (64, 2048, 192), (130, 1028, 132)])
def test_fp32_every_slab_count(rl, M, K, N, slabs):
    """Forced slab counts, ragged last slabs included; a launch shape gives the same bits twice."""
    import torch
    w = workloads.make(M, K, N, "f32", 1e-5, 4200 + M + slabs)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "f32", slabs)
    assert used == "f32"
    compare(Y, Z, "f32", f"fp32 {M}x{K}x{N}, {slabs} slabs")
    Y2, _ = _run(rl, w, "f32", slabs)
    assert np.array_equal(Y, Y2), "same launch shape, different bits"


def test_fp32_long_k_keeps_the_margin(rl):
    """K = 65536: the two levels of accumulators keep the error at a few ulps, where one running fp32 sum
    per output would use up the tolerance."""
    w = workloads.make(4, 65536, 256, "f32", 1e-6, 4300)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w)
    assert used == "f32"
    ratio, _ = compare(Y, Z, "f32", "fp32 4x65536x256")
    print(f"fp32 4x65536x256: max|err|/rms(Y) = {ratio:.3e}")
    assert ratio <= 2e-6, ratio


def test_fp32_large_m_sampled_rows(rl):
    w = workloads.make(2048, 1024, 2048, "f32", 1e-5, 4400, outlier_frac=0.01, n_check_rows=64)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
    Y, used = _run(rl, w, rows=w.check_rows)
    assert used == "f32"
    compare(Y, Z, "f32", "fp32 2048x1024x2048")


def test_fp32_plain_product_and_fallbacks(rl):
    """matmul in fp32 takes the same kernel without the norm; sizes it does not run (not multiples of 4) go to
    the plain kernel; forcing it on a 16-bit type is refused."""
    import torch
    w = workloads.make(70, 516, 260, "f32", 1e-5, 4500)
    X, g, W = upload(w)
    Y = rl.matmul(X, W)
    torch.cuda.synchronize()
    assert rl.rl_last_variant() == "f32"
    want = w.X.astype(np.float64) @ w.W.astype(np.float64)
    compare(to_host_f64(Y, "f32"), want, "f32", "fp32 matmul")
    w2 = workloads.make(9, 130, 1027, "f32", 1e-5, 4501)
    Z2 = oracle.rmsnorm_linear(w2.X, w2.g, w2.W, "f32", w2.eps)
    Y2, used = _run(rl, w2)
    assert used == "naive"
    compare(Y2, Z2, "f32", "fp32 odd sizes")
    wb = workloads.make(8, 64, 64, "bf16", 1e-5, 4502)
    Xb, gb, Wb = upload(wb)
    with pytest.raises(rl.RmsnlError) as ei:
        rl.rmsnorm_linear_ex(Xb, gb, Wb, wb.eps, torch.empty(8, 64, dtype=torch.bfloat16, device="cuda"), variant="f32")
    assert ei.value.status == 2


@pytest.mark.parametrize("M,K,H", [(1, 64, 4), (3, 516, 36), (16, 1024, 512), (50, 260, 100), (64, 2048, 192),
                                   (70, 516, 64), (200, 1028, 320)])
def test_fp32_gated_block(rl, M, K, H):
    """The gated block in fp32 on the same kernel: a tile is 32 gate and 32 up columns; both layouts of W."""
    import torch
    w = workloads.make(M, K, 2 * H, "f32", 1e-5, 4800 + M + H)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, "f32", w.eps)
    X, g, W = upload(w)
    Y = rl.rmsnorm_gated_mlp(X, g, W, w.eps)
    torch.cuda.synchronize()
    assert rl.rl_last_variant() == "f32"
    worst = compare_gated(to_host_f64(Y, "f32"), Z, "f32", f"fp32 gated {M}x{K}x2*{H}")
    print(f"fp32 gated {M}x{K}x2*{H}: worst err/bound {worst:.3f}")
    for slabs in (2, 5):
        Ys = rl.rmsnorm_gated_mlp_ex(X, g, W, w.eps, variant="f32", slabs=slabs)
        torch.cuda.synchronize()
        compare_gated(to_host_f64(Ys, "f32"), Z, "f32", f"fp32 gated, {slabs} slabs")
    if H % 64 == 0:
        Wi = rl.rl_interleave_gate_up(W)
        Yi = rl.rmsnorm_gated_mlp_interleaved(X, g, Wi, w.eps)
        torch.cuda.synchronize()
        assert rl.rl_last_variant() == "f32"
        assert torch.equal(Yi, Y), "the interleaved layout reads other addresses, not other values"


def test_fp32_eps_zero_and_zero_row(rl):
    """eps = 0 gives Eq. 1 exactly; an all-zero row then yields NaN as the definition does, other rows are untouched."""
    w = workloads.make(20, 256, 128, "f32", 0.0, 4600)
    w.X[7] = 0.0
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, "f32", 0.0)
    Y, used = _run(rl, w)
    assert used == "f32"
    assert np.isnan(Y[7]).all()
    compare(Y, Z, "f32", "fp32 eps = 0 with a zero row")


def test_fp32_tuner_and_workspace(rl):
    import torch
    w = workloads.make(8, 2048, 512, "f32", 1e-5, 4700)
    X, g, W = upload(w)
    Y = torch.empty(8, 512, dtype=torch.float32, device="cuda")
    try:
        us = rl.rl_autotune(X, g, W, w.eps, Y, reps=5)
        variant, nt, ks = rl.rl_autotune_get(8, 2048, 512, torch.float32)
        assert us > 0 and variant == "f32", (us, variant)
        Z = oracle.rmsnorm_linear(w.X, w.g, w.W, "f32", w.eps)
        Y2, used = _run(rl, w)
        assert used == "f32"
        compare(Y2, Z, "f32", "fp32 after tuning")
    finally:
        rl.rl_autotune_clear()
    assert rl.rl_workspace_bytes(8, 2048, 512, torch.float32) > 0
