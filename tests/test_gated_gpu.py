"""Parity of the gated block (RMSNorm, the two products, SiLU(gate) * up in one kernel) against the
fp64 oracle, through the C ABI.  Needs an MI355X.

Bar: see util.compare_gated (the plain block's tolerance propagated through the gate, plus the
output rounding).  Inputs are seeded and synthetic; W is [K][2H] = [gate | up], or the same columns interleaved in
groups of 64 for rmsnorm_gated_mlp_interleaved.
"""
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
    yield pkg
    pkg.rl_set_variant("auto")
    pkg.rl_set_tuning(0, 0)


def _run(rl, w, variant="auto", tuning=(0, 0), rows=None):
    import torch
    rl.rl_set_variant(variant)
    rl.rl_set_tuning(*tuning)
    try:
        X, g, W = upload(w)
        Y = rl.rmsnorm_gated_mlp(X, g, W, w.eps)
        torch.cuda.synchronize()
        used = rl.rl_last_variant()
    finally:
        rl.rl_set_variant("auto")
        rl.rl_set_tuning(0, 0)
    if rows is not None:
        Y = Y[torch.from_numpy(np.asarray(rows)).cuda()]
    return to_host_f64(Y, w.dtype), used


def test_gateup_config(rl):
    """Config 4 read as the gated MLP it comes from: X 64x4096, W 4096x(2*14336)."""
    w = workloads.config("gateup")
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
    Y, used = _run(rl, w, rows=w.check_rows)
    assert used == "skinny"
    worst = compare_gated(Y, Z, w.dtype, "gateup gated")
    print(f"gateup gated: variant {used}, worst err/bound {worst:.3f}")


SHAPES = [
    # M, K, H
    (1, 64, 8), (2, 72, 136), (5, 264, 40), (8, 512, 256), (16, 1024, 2048), (17, 520, 200),
    (33, 1032, 392), (64, 264, 584), (65, 256, 128), (100, 520, 392), (130, 1544, 264),
    (257, 264, 136), (300, 776, 648), (512, 512, 512),
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("variant", ["auto", "gemv", "skinny", "tile", "tile_pre", "naive"])
@pytest.mark.parametrize("M,K,H", SHAPES)
def test_gated_shapes(rl, M, K, H, variant, dtype):
    if variant == "tile_pre" and M <= 64:
        pytest.skip("the two-kernel form is for large M")
    if variant == "gemv" and M > 16:
        pytest.skip("gemv needs M <= 16")
    w = workloads.make(M, K, 2 * H, dtype, 1e-5, 7000 + M * 3 + K + H, outlier_frac=0.1 if M > 8 else 0.0)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, variant)
    if variant != "auto":
        assert used == variant
    compare_gated(Y, Z, dtype, f"gated {M}x{K}x2*{H} {dtype}/{variant}->{used}")


@pytest.mark.parametrize("n_tile,k_split", [(128, 2), (128, 4), (64, 3), (32, 8), (16, 2)])
def test_gated_split_k(rl, n_tile, k_split):
    """The cross-workgroup exchange with the gated epilogue in the last arriver."""
    w = workloads.make(16, 4096, 2 * 1096, "bf16", 1e-5, 7100 + n_tile + k_split)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "skinny", tuning=(n_tile, k_split))
    assert used == "skinny"
    compare_gated(Y, Z, "bf16", f"gated split n_tile={n_tile} k_split={k_split}")


@pytest.mark.parametrize("M,K,H", [(1, 1, 1), (3, 100, 7), (4, 513, 33), (9, 130, 12), (70, 77, 50)])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_gated_any_shape_falls_back(rl, M, K, H, dtype):
    w = workloads.make(M, K, 2 * H, dtype, 1e-5, 7200 + M + K + H)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "auto")
    compare_gated(Y, Z, dtype, f"gated odd {M}x{K}x2*{H} {dtype}->{used}")


@pytest.mark.parametrize("n_tile,waves", [(256, 4), (512, 4), (512, 8)])
def test_gated_tile_launch_shapes(rl, n_tile, waves):
    w = workloads.make(300, 776, 2 * 648, "bf16", 1e-5, 7250 + n_tile + waves)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "tile", tuning=(n_tile, waves))
    assert used == "tile"
    compare_gated(Y, Z, "bf16", f"gated tile shape={n_tile} waves={waves}")


def test_gated_prefill_sized_tile(rl):
    """A tile-kernel shape with several tiles each way and ragged edges, on sampled rows."""
    w = workloads.make(1000, 2048, 2 * 1160, "bf16", 1e-5, 7300)
    rows = np.arange(0, 1000, 37)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=rows)
    Y, used = _run(rl, w, rows=rows)
    assert used in ("tile", "tile_pre", "skinny")
    compare_gated(Y, Z, "bf16", f"gated 1000x2048x2*1160 auto->{used}")
    Y, used = _run(rl, w, "tile", rows=rows)
    assert used == "tile"
    compare_gated(Y, Z, "bf16", "gated 1000x2048x2*1160, fused tile kernel")
    for tuning in ((0, 0), (1, 1), (1, 4)):          # the library's own split, none, four slabs
        Y, used = _run(rl, w, "tile_pre", tuning=tuning, rows=rows)
        assert used == "tile_pre"
        compare_gated(Y, Z, "bf16", f"gated 1000x2048x2*1160, two kernels {tuning}")


def test_gated_hand_case(rl, golden_hand_cases):
    """H1's inputs through the gated block (G2 of the golden file); tiny, so it runs on the fallback."""
    w = workloads.Workload("H1", 2, 3, 2, "f32", 0.0,
                           workloads.to_storage(np.array([[3, 4, 0], [1, 2, 2]], np.float32), "f32"),
                           workloads.to_storage(np.array([1, 2, 0.5], np.float32), "f32"),
                           workloads.to_storage(np.array([[1, 0], [0, 1], [2, -2]], np.float32), "f32"),
                           np.arange(2), np.zeros(0, np.int64))
    Y, _ = _run(rl, w)
    for (i, j), v in golden_hand_cases["G2"].items():
        assert Y[i, j] == pytest.approx(v, rel=2e-6)


def test_gated_matches_unfused_pair(rl):
    """A/B: the library's own rmsnorm_linear followed by silu_mul agrees with the fused call."""
    import torch
    w = workloads.make(32, 1024, 2 * 512, "bf16", 1e-5, 7400)
    X, g, W = upload(w)
    Zg = rl.rmsnorm_linear(X, g, W, w.eps)
    Yp = rl.silu_mul(Zg)
    Yf = rl.rmsnorm_gated_mlp(X, g, W, w.eps)
    torch.cuda.synchronize()
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    compare_gated(to_host_f64(Yf, "bf16"), Z, "bf16", "fused")
    # the pair rounds Z to bf16 before the gate: one more rounding of each factor
    H = 512
    Zr = to_host_f64(Zg, "bf16")
    want = Zr[:, :H] / (1.0 + np.exp(-Zr[:, :H])) * Zr[:, H:]
    np.testing.assert_allclose(to_host_f64(Yp, "bf16"), want, rtol=2.0 ** -7, atol=1e-6)


def test_gated_zero_row_and_canaries(rl):
    import torch
    w = workloads.make(6, 256, 2 * 136, "bf16", 0.0, 7500)
    w.X[3] = 0
    with np.errstate(all="ignore"):
        Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, 0.0)
    X, g, W = upload(w)
    pad, H = 1024, 136
    buf = torch.full((pad + 6 * H + pad,), 123.0, dtype=torch.bfloat16, device="cuda")
    Y = buf[pad:pad + 6 * H].view(6, H)
    for variant in ("skinny", "naive"):
        Y.fill_(7.0)
        rl.rl_set_variant(variant)
        try:
            rl.rmsnorm_gated_mlp(X, g, W, 0.0, Y)
            torch.cuda.synchronize()
        finally:
            rl.rl_set_variant("auto")
        assert torch.all(buf[:pad] == 123.0) and torch.all(buf[pad + 6 * H:] == 123.0)
        compare_gated(to_host_f64(Y, "bf16"), Z, "bf16", f"gated zero row/{variant}")


@pytest.mark.parametrize("n_tile,k_split", [(128, 1), (128, 5), (256, 2), (256, 16), (512, 4)])
def test_gated_gemv_launch_shapes(rl, n_tile, k_split):
    w = workloads.make(3, 2056, 2 * 776, "bf16", 1e-5, 7600 + n_tile + k_split)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "gemv", tuning=(n_tile, k_split))
    assert used == "gemv"
    compare_gated(Y, Z, "bf16", f"gated gemv n_tile={n_tile} k_split={k_split}")


def test_fast_variants_refuse_odd_halves(rl):
    w = workloads.make(1, 256, 2 * 12, "bf16", 1e-5, 7601)           # H % 8 != 0
    for variant in ("gemv", "skinny", "tile"):
        with pytest.raises(rl.RmsnlError):
            _run(rl, w, variant)


# ------------------------------------------------------------------ W interleaved in groups of 64
def _interleave_host(W: np.ndarray, H: int) -> np.ndarray:
    """[gate | up] -> groups of 64 gate columns alternating with the same outputs' 64 up columns."""
    K = W.shape[0]
    return np.ascontiguousarray(
        np.stack([W[:, :H].reshape(K, H // 64, 64), W[:, H:].reshape(K, H // 64, 64)], axis=2).reshape(K, 2 * H))


def _run_interleaved(rl, w, variant="auto", tuning=(0, 0), repack_on_device=False):
    import torch
    H = w.N // 2
    X, g, W = upload(w)
    if repack_on_device:
        Wi = rl.rl_interleave_gate_up(W)
    else:
        Wi = to_device(_interleave_host(w.W, H), w.dtype)
    rl.rl_set_variant(variant)
    rl.rl_set_tuning(*tuning)
    try:
        Y = rl.rmsnorm_gated_mlp_interleaved(X, g, Wi, w.eps)
        torch.cuda.synchronize()
        used = rl.rl_last_variant()
        Y2 = rl.rmsnorm_gated_mlp(X, g, W, w.eps)          # the two-halves layout, same variant and launch shape
        torch.cuda.synchronize()
    finally:
        rl.rl_set_variant("auto")
        rl.rl_set_tuning(0, 0)
    return to_host_f64(Y, w.dtype), used, to_host_f64(Y2, w.dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("K,H", [(1, 64), (37, 192), (520, 4096)])
def test_interleave_kernel_is_the_permutation(rl, K, H, dtype):
    import torch
    w = workloads.make(1, K, 2 * H, dtype, 1e-5, 7650 + K + H)
    _, _, W = upload(w)
    Wi = rl.rl_interleave_gate_up(W)
    torch.cuda.synchronize()
    want = to_device(_interleave_host(w.W, H), dtype)
    assert torch.equal(Wi.view(torch.uint8), want.view(torch.uint8))


ISHAPES = [
    # M, K, H with H % 64 == 0
    (1, 64, 64), (2, 72, 192), (5, 264, 128), (8, 512, 256), (16, 1024, 2048), (17, 520, 448),
    (33, 1032, 384), (64, 264, 576), (65, 256, 128), (100, 520, 320), (130, 1544, 256),
    (257, 264, 192), (300, 776, 640), (512, 512, 512),
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("variant", ["auto", "gemv", "skinny", "tile", "tile_pre", "naive"])
@pytest.mark.parametrize("M,K,H", ISHAPES)
def test_gated_interleaved_shapes(rl, M, K, H, variant, dtype):
    """Against the oracle on the de-interleaved W, and bit for bit against the two-halves call (the
    arithmetic is the same, only the column a lane fetches differs)."""
    if variant == "tile_pre" and M <= 64:
        pytest.skip("the two-kernel form is for large M")
    if variant == "gemv" and M > 16:
        pytest.skip("gemv needs M <= 16")
    w = workloads.make(M, K, 2 * H, dtype, 1e-5, 7660 + M * 3 + K + H, outlier_frac=0.1 if M > 8 else 0.0)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used, Y2 = _run_interleaved(rl, w, variant, repack_on_device=(M % 2 == 0))
    if variant != "auto":
        assert used == variant
    compare_gated(Y, Z, dtype, f"gated interleaved {M}x{K}x2*{H} {dtype}/{variant}->{used}")
    assert np.array_equal(Y, Y2), f"interleaved and two-halves results differ ({variant}->{used})"


@pytest.mark.parametrize("variant,tuning", [("skinny", (128, 2)), ("skinny", (64, 3)), ("skinny", (32, 8)),
                                            ("gemv", (128, 5)), ("gemv", (256, 2)), ("gemv", (512, 4)),
                                            ("tile", (256, 4)), ("tile", (512, 8)),
                                            ("tile_pre", (1, 1)), ("tile_pre", (1, 4))])
def test_gated_interleaved_launch_shapes(rl, variant, tuning):
    M = 3 if variant == "gemv" else 16 if variant == "skinny" else 300
    w = workloads.make(M, 2056, 2 * 1088, "bf16", 1e-5, 7680 + sum(tuning))
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used, Y2 = _run_interleaved(rl, w, variant, tuning=tuning)
    assert used == variant
    compare_gated(Y, Z, "bf16", f"gated interleaved {variant} {tuning}")
    assert np.array_equal(Y, Y2)


def test_gated_interleaved_f32_and_bad_h(rl):
    for K, expect in ((100, "f32"), (102, "naive")):       # the fp32 kernel, and the plain one where K % 4 != 0
        w = workloads.make(7, K, 2 * 64, "f32", 1e-5, 7690)
        Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
        Y, used, _ = _run_interleaved(rl, w)
        assert used == expect
        compare_gated(Y, Z, "f32", f"gated interleaved f32, K = {K}")
    w = workloads.make(2, 64, 2 * 96, "bf16", 1e-5, 7691)            # H % 64 != 0
    X, g, W = upload(w)
    with pytest.raises(rl.RmsnlError):
        rl.rmsnorm_gated_mlp_interleaved(X, g, W, w.eps)
    with pytest.raises(rl.RmsnlError):
        rl.rl_interleave_gate_up(W)


def test_gateup_config_interleaved(rl):
    """Config 4 as the gated MLP with interleaved weights, at full size, on sampled rows."""
    import torch
    w = workloads.config("gateup")
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
    X, g, W = upload(w)
    Wi = rl.rl_interleave_gate_up(W)
    Y = rl.rmsnorm_gated_mlp_interleaved(X, g, Wi, w.eps)
    torch.cuda.synchronize()
    assert rl.rl_last_variant() == "skinny"
    Yr = to_host_f64(Y[torch.from_numpy(np.asarray(w.check_rows)).cuda()], w.dtype)
    compare_gated(Yr, Z, w.dtype, "gateup gated interleaved")


# ------------------------------------------------------------------ the launch-shape tuner
@pytest.mark.parametrize("M,K,N,gated", [(1, 2048, 1024, False), (16, 1024, 2048, False), (48, 512, 1024, True),
                                         (200, 512, 768, False), (3, 100, 7, False)])
def test_autotune_picks_a_runnable_shape_and_auto_uses_it(rl, M, K, N, gated):
    import torch
    w = workloads.make(M, K, N, "bf16", 1e-5, 7700 + M + K + N)
    X, g, W = upload(w)
    Y = torch.empty((M, N // 2 if gated else N), dtype=torch.bfloat16, device="cuda")
    rl.rl_autotune_clear()
    try:
        us = rl.rl_autotune(X, g, W, w.eps, Y, gated=gated, reps=5)
        variant, n_tile, k_split = rl.rl_autotune_get(M, K, N, torch.bfloat16, gated)
        assert us > 0 and variant in ("gemv", "skinny", "tile", "tile_pre", "naive")
        print(f"{M}x{K}x{N} gated={gated}: {variant} n_tile={n_tile} k_split={k_split}, {us:.2f} us")
        rl.rl_set_variant("auto")
        Y.fill_(float("nan"))
        (rl.rmsnorm_gated_mlp if gated else rl.rmsnorm_linear)(X, g, W, w.eps, Y)
        torch.cuda.synchronize()
        assert rl.rl_last_variant() == variant
        Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
        if gated:
            compare_gated(to_host_f64(Y, "bf16"), Z, "bf16", "tuned gated")
        else:
            compare(to_host_f64(Y, "bf16"), Z, "bf16", "tuned")
    finally:
        rl.rl_autotune_clear()
    assert rl.rl_autotune_get(M, K, N, torch.bfloat16, gated) == ("auto", 0, 0)
