"""Shapes past the fast kernels' old limits run on the fast kernels, not on the fallback.  Needs an MI355X.

A W of 16640 x 131072 bf16 (4 GiB: a vocabulary-sized projection) used to send every call to the
fp32-arithmetic fallback, silently and a hundred times slower, because the tile kernels addressed W
with 32-bit offsets from its first byte and the skinny kernel priced its workspace before it sized
its slabs.  Also here: more rows than a grid's second dimension holds, and the fp32 path at long K.
"""
import numpy as np
import pytest

import oracle
import workloads
from util import compare, to_device, to_host_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rl():
    import torch
    import paper_2405_05751_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.rl_set_variant("auto")
    pkg.rl_set_tuning(0, 0)
    yield pkg
    pkg.rl_set_variant("auto")
    pkg.rl_set_tuning(0, 0)


K_BIG, N_BIG, BLOCK = 16640, 131072, 4096       # W: 4.06 GiB of bf16, byte offsets beyond 2^32


@pytest.fixture(scope="module")
def big_w():
    """g and W [16640][131072] bf16, seeded.  One block of 4096 columns is drawn; block j of W is that
    block with its columns rotated by 17 j and, for odd j, negated (exact in bf16), so every column is
    N(0, 1/K) as in the configurations and no two blocks agree column for column: a kernel that fetched
    a wrong column or row would show.  Only column subsets ever go to the oracle."""
    rng = np.random.default_rng(workloads.SEED + 9000)
    g = workloads.to_storage(rng.uniform(0.5, 1.5, K_BIG).astype(np.float32), "bf16")
    base = workloads.to_storage(rng.standard_normal((K_BIG, BLOCK), dtype=np.float32) * np.float32(K_BIG ** -0.5), "bf16")

    def columns(cols):
        cols = np.asarray(cols)
        j, c = cols // BLOCK, cols % BLOCK
        out = base[:, (c + 17 * j) % BLOCK]
        return out ^ np.where(j % 2 == 1, 0x8000, 0).astype(np.uint16)[None, :]

    import torch
    Wd = torch.empty((K_BIG, N_BIG), dtype=torch.bfloat16, device="cuda")
    for j in range(N_BIG // BLOCK):
        Wd[:, j * BLOCK:(j + 1) * BLOCK] = to_device(columns(np.arange(j * BLOCK, (j + 1) * BLOCK)), "bf16")
    return g, columns, to_device(g, "bf16"), Wd


# columns the oracle evaluates: the first and last of W, and those on either side of byte offset 2^32 in the last rows
CHECK_COLS = np.concatenate([np.arange(0, 384), np.arange(65536 - 192, 65536 + 192), np.arange(N_BIG - 384, N_BIG)])


@pytest.mark.parametrize("M,expect", [(64, "skinny"), (1, ("gemv", "skinny")), (256, "tile_pre"), (200, "tile_pre")])
def test_four_gib_w_runs_on_a_fast_kernel(rl, big_w, M, expect):
    import torch
    g, columns, gd, Wd = big_w
    print(f"large shape {M}x{K_BIG}x{N_BIG}", flush=True)
    rng = np.random.default_rng(workloads.SEED + 9100 + M)
    X = workloads.to_storage(rng.standard_normal((M, K_BIG), dtype=np.float32), "bf16")
    Y = rl.rmsnorm_linear(to_device(X, "bf16"), gd, Wd, 1e-5)
    torch.cuda.synchronize()
    used = rl.rl_last_variant()
    assert used in (expect if isinstance(expect, tuple) else (expect,)), used
    rows = np.unique(np.array([0, M // 3, M - 1]))
    Z = oracle.rmsnorm_linear(X, g, columns(CHECK_COLS), "bf16", 1e-5, rows=rows)
    got = Y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(CHECK_COLS).cuda()]
    ratio, _ = compare(to_host_f64(got, "bf16"), Z, "bf16", f"{M}x{K_BIG}x{N_BIG}->{used}")
    print(f"  variant {used}, max|err|/rms(Y) = {ratio:.3e}", flush=True)


def test_four_gib_w_one_fused_tile_kernel_and_plain_product(rl, big_w):
    """The fused tile kernel and the plain matmul on the same W (forced, ragged M)."""
    import torch
    g, columns, gd, Wd = big_w
    M = 130
    rng = np.random.default_rng(workloads.SEED + 9200)
    X = workloads.to_storage(rng.standard_normal((M, K_BIG), dtype=np.float32), "bf16")
    Xd = to_device(X, "bf16")
    rows = np.array([0, 77, 129])
    sel_r, sel_c = torch.from_numpy(rows).cuda(), torch.from_numpy(CHECK_COLS).cuda()
    Wsub = columns(CHECK_COLS)
    Z = oracle.rmsnorm_linear(X, g, Wsub, "bf16", 1e-5, rows=rows)
    Y = rl.rmsnorm_linear_ex(Xd, gd, Wd, 1e-5, variant="tile")
    torch.cuda.synchronize()
    assert rl.rl_last_variant() == "tile"
    compare(to_host_f64(Y[sel_r][:, sel_c], "bf16"), Z, "bf16", "fused tile kernel, 4 GiB W")
    P = rl.matmul(Xd, Wd)
    torch.cuda.synchronize()
    assert rl.rl_last_variant() != "naive"
    compare(to_host_f64(P[sel_r][:, sel_c], "bf16"), oracle.matmul(X[rows], Wsub, "bf16"), "bf16", "plain product, 4 GiB W")


def test_more_rows_than_a_grid_dimension(rl):
    """M > 65535 on the fp32 kernel (a row block per 64 rows), on the fallback (fp32, N not a multiple of 4) and on
    the tile kernels (bf16)."""
    import torch
    for dt, K, N in (("f32", 24, 40), ("f32", 24, 42), ("bf16", 64, 256)):
        M = 70001
        w = workloads.make(M, K, N, dt, 1e-5, 9300, n_check_rows=48)
        X, g, W = to_device(w.X, dt), to_device(w.g, dt), to_device(w.W, dt)
        Y = rl.rmsnorm_linear(X, g, W, w.eps)
        torch.cuda.synchronize()
        used = rl.rl_last_variant()
        rows = np.concatenate([w.check_rows, [M - 1]])
        Z = oracle.rmsnorm_linear(w.X, w.g, w.W, dt, w.eps, rows=rows)
        compare(to_host_f64(Y[torch.from_numpy(rows).cuda()], dt), Z, dt, f"{M} rows {dt}->{used}")
        assert used == ("tile_pre" if dt == "bf16" else "f32" if N % 4 == 0 else "naive"), used


@pytest.mark.parametrize("M,K,N", [(4, 16384, 256), (3, 28672, 264), (2, 65536, 64)])
def test_fp32_path_at_long_k(rl, M, K, N):
    """The 1e-5 bar of the fp32 path holds at the long reductions of the configurations (and beyond)."""
    import torch
    w = workloads.make(M, K, N, "f32", 1e-6, 9400 + M)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, "f32", w.eps)
    Y = rl.rmsnorm_linear(to_device(w.X, "f32"), to_device(w.g, "f32"), to_device(w.W, "f32"), w.eps)
    torch.cuda.synchronize()
    ratio, _ = compare(to_host_f64(Y, "f32"), Z, "f32", f"fp32 {M}x{K}x{N}")
    print(f"fp32 {M}x{K}x{N}: max|err|/rms(Y) = {ratio:.3e}")
    assert ratio <= 2e-6, "fp64 accumulation should leave little more than the output rounding"
