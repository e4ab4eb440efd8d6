"""Parity of the HIP library against the fp64 oracle, through the C ABI.  Needs an MI355X.

Bar: max |err| <= 2e-2 * rms(Y) for f16/bf16 and <= 1e-5 * rms(Y) for f32, per checked row and
over all checked rows; NaN positions must agree.  Inputs are the seeded synthetic workloads.
"""
import numpy as np
import pytest

import oracle
import workloads
from util import TOL, compare, to_device, to_host_f64, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rl():
    import torch
    import paper_2405_05751_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    yield pkg
    pkg.rl_set_variant("auto")
    pkg.rl_set_tuning(0, 0)


_cache = {}


def _workload(name):
    if name not in _cache:
        w = workloads.config(name)
        Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
        _cache[name] = (w, Z)
    return _cache[name]


def _run(rl, w, variant="auto", tuning=(0, 0), rows=None):
    import torch
    rl.rl_set_variant(variant)
    rl.rl_set_tuning(*tuning)
    X, g, W = upload(w)
    Y = rl.rmsnorm_linear(X, g, W, w.eps)
    torch.cuda.synchronize()
    used = rl.rl_last_variant()
    rl.rl_set_variant("auto")
    rl.rl_set_tuning(0, 0)
    if rows is not None:
        Y = Y[torch.from_numpy(np.asarray(rows)).cuda()]
    return to_host_f64(Y, w.dtype), used


def _supported(variant, w):
    if variant == "auto":
        return True
    if variant == "naive":
        return w.M <= 4096
    if w.dtype == "f32" or w.N % 8 or w.K % 8:
        return False
    if variant == "gemv":
        return w.M <= 16
    if variant == "skinny":
        return w.M <= 1024
    if variant == "tile_pre":
        return w.M > 64
    return True


# ------------------------------------------------------------------ the five configurations
@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_config_auto(rl, name):
    w, Z = _workload(name)
    Y, used = _run(rl, w, "auto", rows=w.check_rows)
    ratio, rms = compare(Y, Z, w.dtype, f"{name}/auto->{used}")
    print(f"{name}: variant {used}, max|err|/rms(Y) = {ratio:.3e}, rms(Y) = {rms:.4f}")
    # a correct 16-bit kernel sits at the output-rounding floor, far above fp64 agreement
    if w.dtype == "bf16":
        assert ratio > 1e-3, "suspiciously small error: is the comparison against a rounded oracle?"


@pytest.mark.parametrize("variant", ["naive", "gemv", "skinny", "tile", "tile_pre"])
@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_config_forced_variant(rl, name, variant):
    shape = workloads.config_shape(name)
    probe = workloads.Workload(name, shape[1], shape[2], shape[3], shape[4], shape[5],
                               None, None, None, None, None)
    if variant == "naive" and name == "prefill":
        pytest.skip("the slow fallback would take minutes at 8192^3")
    if not _supported(variant, probe):
        pytest.skip(f"{variant} does not cover {name}")
    w, Z = _workload(name)
    Y, used = _run(rl, w, variant, rows=w.check_rows)
    assert used == variant
    ratio, _ = compare(Y, Z, w.dtype, f"{name}/{variant}")
    print(f"{name}/{variant}: max|err|/rms(Y) = {ratio:.3e}")


# ------------------------------------------------------------------ the paper's own shape
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("variant", ["auto", "naive", "gemv", "skinny", "tile"])
def test_paper_shape(rl, dtype, variant):
    """X[16,1024], G[1024], W[1024,4096] -> Z[16,4096] (shapes of the case-study figure)."""
    w = workloads.make(16, 1024, 4096, dtype, 1e-6, 901)
    if not _supported(variant, w):
        pytest.skip(f"{variant} does not cover the shape")
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, variant)
    compare(Y, Z, dtype, f"paper-shape/{variant}->{used}")


# ------------------------------------------------------------------ ragged and edge shapes
RAGGED = [
    # M, K, N
    (1, 8, 8), (1, 64, 8), (2, 72, 264), (3, 1000, 520), (5, 4104, 1032), (7, 136, 4096),
    (15, 2048, 776), (16, 520, 256), (17, 512, 512), (33, 1032, 392), (64, 264, 1160),
    (65, 256, 256), (100, 520, 776), (130, 1544, 520), (257, 264, 264), (300, 776, 1288),
]


@pytest.mark.parametrize("variant", ["auto", "gemv", "skinny", "tile"])
@pytest.mark.parametrize("M,K,N", RAGGED)
def test_ragged_shapes(rl, M, K, N, variant):
    w = workloads.make(M, K, N, "bf16", 1e-5, 1000 + M * 7 + K + N, outlier_frac=0.1 if M > 8 else 0.0)
    if not _supported(variant, w):
        pytest.skip(f"{variant} does not cover M={M}")
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, variant)
    compare(Y, Z, w.dtype, f"ragged {M}x{K}x{N}/{variant}->{used}")


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (2, 3, 2), (3, 7, 5), (4, 513, 33), (9, 130, 1027), (70, 77, 99)])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_any_shape_falls_back(rl, M, K, N, dtype):
    """Sizes that are not multiples of 8 are served (by the fallback) rather than refused."""
    w = workloads.make(M, K, N, dtype, 1e-5, 2000 + M + K + N)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "auto")
    compare(Y, Z, dtype, f"odd {M}x{K}x{N} {dtype}->{used}")


@pytest.mark.parametrize("n_tile,k_split", [(128, 1), (128, 3), (256, 1), (256, 2), (256, 7), (512, 4), (256, 64)])
def test_gemv_launch_shapes(rl, n_tile, k_split):
    """Every tile width and slab count of the split-K variant gives the same answer (to tolerance)."""
    w = workloads.make(4, 2056, 1544, "bf16", 1e-5, 3000 + n_tile + k_split)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "gemv", tuning=(n_tile, k_split))
    assert used == "gemv"
    compare(Y, Z, w.dtype, f"gemv n_tile={n_tile} k_split={k_split}")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("M,K,N", [(2048, 1024, 4096), (1100, 520, 2056), (300, 4104, 264), (512, 776, 14336),
                                   (257, 264, 8200)])
def test_two_slabs_of_the_split_product(rl, M, K, N, dtype):
    """Two slabs of the split product with ragged edges, the fused block and the plain product, twice in a
    row bit for bit."""
    import torch
    w = workloads.make(M, K, N, dtype, 1e-5, 4950 + M + K + N, outlier_frac=0.05, n_check_rows=24)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
    X, g, W = upload(w)
    rows = torch.from_numpy(w.check_rows).cuda()
    rl.rl_set_variant("tile_pre")
    rl.rl_set_tuning(1, 2)
    try:
        Y1 = rl.rmsnorm_linear(X, g, W, w.eps)
        Y2 = rl.rmsnorm_linear(X, g, W, w.eps)
        Xn = rl.rmsnorm(X, g, w.eps)
        P1 = rl.matmul(Xn, W)
        torch.cuda.synchronize()
        assert rl.rl_last_variant() == "tile_pre"
    finally:
        rl.rl_set_variant("auto")
        rl.rl_set_tuning(0, 0)
    assert torch.equal(Y1.view(torch.int16), Y2.view(torch.int16))
    compare(to_host_f64(Y1[rows], dtype), Z, dtype, f"two slabs {M}x{K}x{N} {dtype}")
    # the plain product of the rounded normalised rows: one more rounding than the fused block
    Zp = oracle.matmul_f64(to_host_f64(Xn[rows], dtype), oracle.decode(w.W, dtype))
    compare(to_host_f64(P1[rows], dtype), Zp, dtype, f"two slabs, plain product {M}x{K}x{N} {dtype}")


@pytest.mark.parametrize("gated", [False, True])
@pytest.mark.parametrize("variant,M", [("gemv", 1), ("gemv", 3), ("gemv", 16), ("skinny", 5), ("skinny", 40)])
@pytest.mark.parametrize("k_split", [2, 3, 4, 5, 8, 9, 16, 17, 32])
def test_every_slab_count_of_the_split_k_epilogue(rl, variant, M, k_split, gated):
    """The last arriver fetches the slabs' partials in batches sized to the slab count (2, 4, 8, 16 per
    batch, several batches beyond): every size, with ragged tiles, and twice in a row (the arrival
    counters must be back at zero)."""
    import torch
    K = 128 * 33 if variant == "gemv" else 256 * 33
    N = 1544 if not gated else 2 * 776
    w = workloads.make(M, K, N, "bf16", 1e-5, 3100 + M + k_split, n_check_rows=min(M, 8))
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
    X, g, W = upload(w)
    call = rl.rmsnorm_gated_mlp if gated else rl.rmsnorm_linear
    rl.rl_set_variant(variant)
    rl.rl_set_tuning(128, k_split)
    try:
        Y1 = call(X, g, W, w.eps)
        Y2 = call(X, g, W, w.eps)
        torch.cuda.synchronize()
        assert rl.rl_last_variant() == variant
    finally:
        rl.rl_set_variant("auto")
        rl.rl_set_tuning(0, 0)
    assert torch.equal(Y1.view(torch.int16), Y2.view(torch.int16)), "same launch shape, different bits"
    Yh = to_host_f64(Y1[torch.from_numpy(w.check_rows).cuda()], w.dtype)
    if gated:
        from util import compare_gated
        compare_gated(Yh, Z, w.dtype, f"{variant} gated M={M} k_split={k_split}")
    else:
        compare(Yh, Z, w.dtype, f"{variant} M={M} k_split={k_split}")


@pytest.mark.parametrize("n_tile,waves", [(256, 4), (256, 8), (512, 4), (512, 8)])
@pytest.mark.parametrize("M,K,N", [(130, 1544, 520), (257, 264, 264), (300, 776, 1288), (512, 512, 1024)])
def test_tile_launch_shapes(rl, M, K, N, n_tile, waves):
    """Both tile shapes (256x256 and 128x512) and both wave counts of the tile variant."""
    w = workloads.make(M, K, N, "bf16", 1e-5, 3500 + M + K + N, outlier_frac=0.05)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "tile", tuning=(n_tile, waves))
    assert used == "tile"
    compare(Y, Z, w.dtype, f"tile {M}x{K}x{N} shape={n_tile} waves={waves}")


# ------------------------------------------------------------------ seeded random shapes
def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        M = int(rng.choice([1, 2, 3, 5, 9, 16, 17, 40, 64, 65, 100, 129, 255, 256, 257, 400, 700]))
        K = int(rng.integers(1, 400)) * 8
        N = int(rng.integers(1, 400)) * 8
        shapes.append((M, K, N))
    return shapes


@pytest.mark.parametrize("gated", [False, True])
@pytest.mark.parametrize("M,K,N", _random_shapes(36, 20240517))
def test_random_shapes_automatic_choice(rl, M, K, N, gated):
    """Whatever the automatic choice picks for a shape (GEMV, skinny, tile kernels with and without
    the K split) agrees with the oracle on sampled rows."""
    import torch
    if gated:
        N = (N + 15) // 16 * 16
    dtype = "bf16" if (M + K + N) % 3 else "f16"
    w = workloads.make(M, K, N, dtype, 1e-5, 6000 + M + 3 * K + 7 * N, outlier_frac=0.05 if M > 16 else 0.0,
                       n_check_rows=min(M, 24))
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
    X, g, W = upload(w)
    Y = (rl.rmsnorm_gated_mlp if gated else rl.rmsnorm_linear)(X, g, W, w.eps)
    torch.cuda.synchronize()
    used = rl.rl_last_variant()
    assert used != "naive"
    Yh = to_host_f64(Y[torch.from_numpy(w.check_rows).cuda()], dtype)
    if gated:
        from util import compare_gated
        compare_gated(Yh, Z, dtype, f"random gated {M}x{K}x{N} {dtype}->{used}")
    else:
        compare(Yh, Z, dtype, f"random {M}x{K}x{N} {dtype}->{used}")


# ------------------------------------------------------------------ skinny kernel, block after block
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("M,K,N", [(65, 264, 136), (128, 1032, 520), (200, 4096, 1024), (1024, 520, 264)])
def test_skinny_runs_larger_m_in_blocks_of_64_rows(rl, M, K, N, dtype):
    w = workloads.make(M, K, N, dtype, 1e-5, 4800 + M + K + N, outlier_frac=0.05)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "skinny")
    assert used == "skinny"
    compare(Y, Z, w.dtype, f"skinny in blocks {M}x{K}x{N} {dtype}")


def test_mid_m_automatic_choice(rl):
    """Above 64 rows: row blocks of the skinny kernel while (row blocks) x K x N is small, the tile
    kernels (two-kernel form, split over K) beyond; from two rows the skinny kernel, unless W is small."""
    w = workloads.make(128, 2048, 2048, "bf16", 1e-5, 4900)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "auto")
    assert used == "skinny"
    compare(Y, Z, w.dtype, "auto -> skinny at 128x2048x2048")
    w = workloads.make(640, 4096, 8192, "bf16", 1e-5, 4902, n_check_rows=32)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
    Y, used = _run(rl, w, "auto", rows=w.check_rows)
    assert used == "tile_pre"
    compare(Y, Z, w.dtype, "auto -> tile_pre at 640x4096x8192")
    w = workloads.make(2, 4096, 4096, "bf16", 1e-5, 4901)
    Y, used = _run(rl, w, "auto")
    assert used == "skinny"
    compare(Y, oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps), w.dtype, "auto -> skinny at M = 2")
    for M, K, N, want in [(2, 1024, 2048, "gemv"), (4, 2048, 2048, "gemv"), (4, 3072, 3072, "skinny"),
                          (1, 1024, 10240, "skinny"), (1, 1024, 8192, "gemv")]:
        w = workloads.make(M, K, N, "bf16", 1e-5, 4903 + M + N)
        Y, used = _run(rl, w, "auto")
        assert used == want, (M, K, N, used)
        compare(Y, oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps), w.dtype, f"auto -> {want} at {M}x{K}x{N}")


# ------------------------------------------------------------------ two-kernel tile variant
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("tuning", [(0, 0), (1, 1), (1, 3), (1, 16)])
@pytest.mark.parametrize("M,K,N", [(65, 8, 8), (130, 1544, 520), (257, 2056, 264), (300, 4104, 1288),
                                   (70, 16392, 264), (1100, 520, 4104)])
def test_tile_pre_variant(rl, M, K, N, dtype, tuning):
    """X-hat and 1/rms written by a first kernel, then the tile kernel as a scaled product: every
    prepass form (1, 2, 4, 8 chunks per thread and the loop), ragged K and N, several tiles; the
    product unsplit (1, 1), split over K by the library's own rule (0, 0) or as told (1, slabs)."""
    w = workloads.make(M, K, N, dtype, 1e-5, 4600 + M + K + N, outlier_frac=0.05)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "tile_pre", tuning=tuning)
    assert used == "tile_pre"
    compare(Y, Z, w.dtype, f"tile_pre {M}x{K}x{N} {dtype} {tuning}")
    Yt, _ = _run(rl, w, "tile")
    # same X-hat rounding and the same product kernel: only the order of the sum of squares differs
    compare(Y, Yt, w.dtype, "tile_pre against tile")


@pytest.mark.parametrize("tuning", [(0, 0), (2, 1), (2, 3)])
@pytest.mark.parametrize("M,K,N", [(300, 1024, 33280), (4100, 2056, 4096), (2048, 520, 8448)])
def test_tile_pre_splits_the_last_partial_round(rl, M, K, N, tuning):
    """More than 256 tiles with a few left over (4, 16, 8 here): full rounds unsplit, the rest split over
    K with compact partial tiles; both tile orders (8 | tile rows or not); (2, 1) switches the split off."""
    w = workloads.make(M, K, N, "bf16", 1e-5, 4650 + M + K + N, outlier_frac=0.02, n_check_rows=48)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=w.check_rows)
    Y, used = _run(rl, w, "tile_pre", tuning=tuning, rows=w.check_rows)
    assert used == "tile_pre"
    compare(Y, Z, w.dtype, f"tile_pre {M}x{K}x{N} remainder split {tuning}")


def test_tile_pre_is_the_automatic_choice_for_large_shapes(rl):
    import torch
    w = workloads.make(1100, 264, 4096, "bf16", 1e-5, 4700)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "auto")
    assert used == "tile_pre"
    compare(Y, Z, w.dtype, "auto -> tile_pre")
    # a lent workspace without room for X-hat: the fused tile kernel runs instead, no error
    small = torch.zeros(1400 * 1024 // 4, dtype=torch.float32, device="cuda")     # head fits, X-hat does not
    try:
        rl.rl_set_workspace(small)
        Y, used = _run(rl, w, "auto")
        assert used == "tile"
        compare(Y, Z, w.dtype, "auto -> tile with a small lent workspace")
        rl.rl_set_variant("tile_pre")
        X, g, W = upload(w)
        with pytest.raises(rl.RmsnlError) as ei:
            rl.rmsnorm_linear(X, g, W, w.eps)
        assert ei.value.status == 4
    finally:
        rl.rl_set_variant("auto")
        rl.rl_set_workspace(None)
    need = rl.rl_workspace_bytes(w.M, w.K, w.N, torch.bfloat16)
    assert need >= 2 * w.M * w.K + 4 * w.M


# ------------------------------------------------------------------ fp32 path
@pytest.mark.parametrize("M,K,N", [(8, 512, 512), (3, 4096, 1000), (16, 1024, 4096)])
def test_fp32_path(rl, M, K, N):
    w = workloads.make(M, K, N, "f32", 1e-6, 4000 + M)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, used = _run(rl, w, "auto")
    ratio, _ = compare(Y, Z, "f32", f"fp32 {M}x{K}x{N}->{used}")
    print(f"fp32 {M}x{K}x{N}: max|err|/rms(Y) = {ratio:.3e}")


# ------------------------------------------------------------------ hand cases through the GPU
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_hand_cases_on_gpu(rl, golden_hand_cases, dtype):
    cases = {
        "H1": ([[3, 4, 0], [1, 2, 2]], [1, 2, 0.5], [[1, 0], [0, 1], [2, -2]], 0.0),
        "H3": ([[2, 2, 2], [-1, 0, 1]], [1, 1, 1], [[1, 0], [0, 1], [1, 1]], 5.0),
    }
    for name, (X, g, W, eps) in cases.items():
        w = workloads.Workload(name, 2, 3, 2, dtype, eps,
                               workloads.to_storage(np.array(X, np.float32), dtype),
                               workloads.to_storage(np.array(g, np.float32), dtype),
                               workloads.to_storage(np.array(W, np.float32), dtype),
                               np.arange(2), np.zeros(0, np.int64))
        Y, _ = _run(rl, w, "auto")
        want = np.array([[golden_hand_cases[name][(i, j)] for j in range(2)] for i in range(2)])
        compare(Y, want, dtype, f"{name} {dtype}")


# ------------------------------------------------------------------ invariants on the GPU
@pytest.mark.parametrize("variant", ["gemv", "skinny", "tile", "naive"])
def test_scale_invariance_on_gpu(rl, variant):
    """eps = 0: Y(cX) = Y(X); with c a power of two the inputs stay exact and so do the outputs."""
    w = workloads.make(8, 512, 512, "bf16", 0.0, 5001)
    if not _supported(variant, w):
        pytest.skip("variant does not cover the shape")
    Y1, _ = _run(rl, w, variant)
    x4 = workloads.to_storage(workloads.to_f32(w.X, "bf16") * 4.0, "bf16")
    w4 = workloads.Workload("x4", w.M, w.K, w.N, w.dtype, 0.0, x4, w.g, w.W, w.check_rows, w.outlier_rows)
    Y4, _ = _run(rl, w4, variant)
    # scaling X by 4 scales A by 16 and B by 4 exactly in binary floating point
    np.testing.assert_array_equal(Y1, Y4)


def test_unit_rms_on_gpu(rl):
    K = 512
    X = workloads.make(8, K, K, "f16", 0.0, 5002).X
    w = workloads.Workload("unit", 8, K, K, "f16", 0.0, X,
                           workloads.to_storage(np.ones(K, np.float32), "f16"),
                           workloads.to_storage(np.eye(K, dtype=np.float32), "f16"),
                           np.arange(8), np.zeros(0, np.int64))
    for variant in ("gemv", "naive"):
        Y, _ = _run(rl, w, variant)
        np.testing.assert_allclose(np.sqrt((Y ** 2).mean(axis=1)), 1.0, rtol=2e-3)


def test_zero_row_nan_positions(rl):
    w = workloads.make(4, 256, 256, "bf16", 0.0, 5003)
    w.X[2] = 0
    with np.errstate(all="ignore"):
        Z0 = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, 0.0)
    assert np.isnan(Z0[2]).all()
    for variant in ("gemv", "naive", "skinny"):
        if _supported(variant, w):
            Y, _ = _run(rl, w, variant)
            compare(Y, Z0, w.dtype, f"zero row eps=0/{variant}")
    w.eps = float(np.float32(1e-6))
    Z1 = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y, _ = _run(rl, w, "auto")
    assert np.all(Y[2] == 0.0)
    compare(Y, Z1, w.dtype, "zero row eps>0")


# ------------------------------------------------------------------ determinism and memory safety
@pytest.mark.parametrize("name,variant", [("decode", "gemv"), ("qkv", "gemv"), ("qkv", "skinny"),
                                          ("gateup", "skinny"), ("tiny", "tile"), ("tiny", "tile_pre")])
def test_bit_reproducible(rl, name, variant):
    w, _ = _workload(name)
    Y1, _ = _run(rl, w, variant)
    for _ in range(3):
        Y2, _ = _run(rl, w, variant)
        assert np.array_equal(Y1, Y2), f"{name}/{variant} differs between runs"


@pytest.mark.parametrize("variant", ["auto", "gemv", "skinny", "tile", "naive"])
def test_output_canaries(rl, variant):
    """Y sits inside a larger buffer filled with a sentinel: nothing outside Y may change."""
    import torch
    w = workloads.make(5, 520, 776, "bf16", 1e-5, 6001)
    if not _supported(variant, w):
        pytest.skip("variant does not cover the shape")
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    X, g, W = upload(w)
    pad = 4096
    buf = torch.full((pad + w.M * w.N + pad,), 123.0, dtype=torch.bfloat16, device="cuda")
    Y = buf[pad:pad + w.M * w.N].view(w.M, w.N)
    Y.fill_(float("nan"))
    rl.rl_set_variant(variant)
    rl.rmsnorm_linear(X, g, W, w.eps, Y)
    torch.cuda.synchronize()
    rl.rl_set_variant("auto")
    assert torch.all(buf[:pad] == 123.0) and torch.all(buf[pad + w.M * w.N:] == 123.0)
    compare(to_host_f64(Y, w.dtype), Z, w.dtype, f"canary/{variant}")


# ------------------------------------------------------------------ the unfused A/B pair
@pytest.mark.parametrize("name", ["tiny", "decode", "qkv", "gateup"])
def test_unfused_pair(rl, name):
    import torch
    w, Z = _workload(name)
    X, g, W = upload(w)
    Xn = rl.rmsnorm(X, g, w.eps)
    torch.cuda.synchronize()
    Yn_oracle = oracle.rmsnorm(w.X, w.g, w.dtype, w.eps)
    compare(to_host_f64(Xn, w.dtype), Yn_oracle, w.dtype, f"{name}/rmsnorm")
    Y = rl.matmul(Xn, W)
    torch.cuda.synchronize()
    # the product alone, against the oracle's product of the very same rounded intermediate
    Xn_bits = Xn.view(torch.uint16).cpu().numpy() if w.dtype == "bf16" else Xn.cpu().numpy()
    Zp = oracle.matmul(Xn_bits, w.W, w.dtype)
    compare(to_host_f64(Y, w.dtype), Zp, w.dtype, f"{name}/matmul")
    # and the pair end to end against the fused definition (one extra 16-bit rounding of Xn)
    ratio, _ = compare(to_host_f64(Y, w.dtype), Z, w.dtype, f"{name}/pair")
    print(f"{name}: unfused pair max|err|/rms(Y) = {ratio:.3e}")


@pytest.mark.parametrize("M,K,N", [(65, 1032, 264), (130, 1544, 520), (300, 4104, 1288), (1100, 520, 4104)])
def test_plain_product_with_few_tiles_is_split_over_k(rl, M, K, N):
    """matmul through the tile kernels (forced: the automatic choice may prefer the skinny kernel
    at these sizes) takes the K split when its tiles are few, and through the automatic choice."""
    import torch
    w = workloads.make(M, K, N, "bf16", 1e-5, 5100 + M + K + N)
    X, _, W = upload(w)
    Zp = oracle.matmul(w.X, w.W, "bf16")
    rl.rl_set_variant("tile_pre")
    try:
        Y = rl.matmul(X, W)
        torch.cuda.synchronize()
        assert rl.rl_last_variant() == "tile_pre"
    finally:
        rl.rl_set_variant("auto")
    compare(to_host_f64(Y, "bf16"), Zp, "bf16", f"matmul {M}x{K}x{N}, tile kernels")
    Y = rl.matmul(X, W)
    torch.cuda.synchronize()
    compare(to_host_f64(Y, "bf16"), Zp, "bf16", f"matmul {M}x{K}x{N}, auto -> {rl.rl_last_variant()}")


@pytest.mark.parametrize("M,K", [(1, 8), (3, 100), (5, 4096), (2, 16384), (4, 20000)])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_rmsnorm_shapes(rl, M, K, dtype):
    import torch
    w = workloads.make(M, K, 8, dtype, 1e-5, 7000 + M + K)
    X, g, _ = upload(w)
    Xn = rl.rmsnorm(X, g, w.eps)
    torch.cuda.synchronize()
    compare(to_host_f64(Xn, dtype), oracle.rmsnorm(w.X, w.g, dtype, w.eps), dtype, f"rmsnorm {M}x{K} {dtype}")


# ------------------------------------------------------------------ error paths that need a device
def test_forced_variant_refuses_unsupported_shape(rl):
    import torch
    w = workloads.make(32, 64, 64, "bf16", 1e-5, 8001)
    X, g, W = upload(w)
    rl.rl_set_variant("gemv")
    try:
        with pytest.raises(rl.RmsnlError) as ei:
            rl.rmsnorm_linear(X, g, W, w.eps)
        assert ei.value.status == 2
    finally:
        rl.rl_set_variant("auto")
    torch.cuda.synchronize()


def test_lent_workspace(rl):
    import torch
    w, Z = _workload("decode")
    need = rl.rl_workspace_bytes(w.M, w.K, w.N, torch.bfloat16)
    assert need > 0
    small = torch.zeros((need - 8192) // 4, dtype=torch.float32, device="cuda")   # head fits, partials do not
    big = torch.zeros(need // 4 + 16, dtype=torch.float32, device="cuda")
    X, g, W = upload(w)
    try:
        rl.rl_set_workspace(small)
        with pytest.raises(rl.RmsnlError) as ei:
            rl.rmsnorm_linear(X, g, W, w.eps)
        assert ei.value.status == 4
        rl.rl_set_workspace(big)
        Y = rl.rmsnorm_linear(X, g, W, w.eps)
        torch.cuda.synchronize()
        compare(to_host_f64(Y, w.dtype), Z, w.dtype, "decode with lent workspace")
        assert big[: 256 * 1024 // 4].abs().sum().item() == 0      # counters returned to zero
    finally:
        rl.rl_set_workspace(None)


def test_workspace_growth_keeps_captured_graphs_valid(rl):
    """A graph captured while the library workspace was small still works after a larger shape has
    made the library switch to a bigger one (the old allocation stays alive)."""
    import torch
    w, Z = _workload("decode")
    X, g, W = upload(w)
    Y = torch.empty((w.M, w.N), dtype=torch.bfloat16, device="cuda")
    rl.rmsnorm_linear(X, g, W, w.eps, Y)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rl.rmsnorm_linear(X, g, W, w.eps, Y)
    Xb = torch.randn((8192, 16384), device="cuda").to(torch.bfloat16)        # X-hat alone needs 256 MiB
    gb = torch.ones(16384, dtype=torch.bfloat16, device="cuda")
    Wb = torch.randn((16384, 256), device="cuda").to(torch.bfloat16)
    rl.rmsnorm_linear(Xb, gb, Wb, 1e-5)
    assert rl.rl_last_variant() == "tile_pre"
    torch.cuda.synchronize()
    for _ in range(2):
        Y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        compare(to_host_f64(Y, w.dtype), Z, w.dtype, "replay after workspace growth")
    Y2 = rl.rmsnorm_linear(X, g, W, w.eps)                                   # and the new workspace serves split-K too
    torch.cuda.synchronize()
    compare(to_host_f64(Y2, w.dtype), Z, w.dtype, "decode after workspace growth")


def test_probes_run(rl):
    import torch
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    rl.rl_probe_copy(dst, src)
    sink = torch.zeros(rl.lib().rl_probe_mfma_sink_floats(), dtype=torch.float32, device="cuda")
    rl.rl_probe_read(src, sink)
    flops = rl.rl_probe_mfma(sink, 8)
    torch.cuda.synchronize()
    assert torch.equal(dst, src) and flops > 0
