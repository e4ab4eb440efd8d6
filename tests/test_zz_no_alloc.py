"""The entry point that allocates nothing (rmsnorm_linear_noalloc), through the C ABI.  Needs an MI355X.

Its kernels keep their split-K counters and partial sums in a fixed device array instead of an
allocated workspace; everything else is rmsnorm_linear.  So the bar is: bit for bit the output of
rmsnorm_linear on the same inputs (same kernels, same launch shape, fixed summation order), and the
plain block's tolerance against the fp64 oracle.  Every case is two calls in a row on the one shared
array, the second on a smaller input, so that nothing the first call left behind may leak into it.
"""
import numpy as np
import pytest

import oracle
import workloads
from util import compare, to_host_f64, upload

pytestmark = pytest.mark.gpu

ERR_WORKSPACE = 4


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


def _both(rl, w, oracle_rows=None):
    """Run the existing and the new entry point on w; returns (Y_existing, Y_noalloc, variant, oracle Z)."""
    import torch
    X, g, W = upload(w)
    Y_ref = rl.rmsnorm_linear(X, g, W, w.eps)
    torch.cuda.synchronize()
    used_ref = rl.rl_last_variant()
    Y = torch.full((w.M, w.N), float("nan"), dtype=Y_ref.dtype, device="cuda")
    st = rl.lib().rmsnorm_linear_noalloc(X.data_ptr(), g.data_ptr(), W.data_ptr(), float(w.eps), Y.data_ptr(),
                                         w.M, w.K, w.N, {"f16": 0, "bf16": 1, "f32": 2}[w.dtype],
                                         torch.cuda.current_stream().cuda_stream)
    assert st == 0, rl.rl_last_error()
    torch.cuda.synchronize()
    used = rl.rl_last_variant()
    rows = np.arange(w.M) if oracle_rows is None else oracle_rows
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps, rows=rows)
    sel = torch.from_numpy(rows).cuda()
    return Y_ref, Y, used_ref, used, to_host_f64(Y[sel], w.dtype), Z


# (first call, second and smaller call): GEMV split over K; skinny split over K; fp16; a ragged shape;
# the fp32 kernel split over K
PAIRS = [
    ((1, 4096, 4096, "bf16"), (1, 1024, 2048, "bf16")),
    ((16, 4096, 6144, "bf16"), (8, 2048, 2048, "f16")),
    ((64, 2048, 4096, "f16"), (3, 520, 264, "bf16")),
    ((130, 1024, 2056, "bf16"), (33, 4096, 1024, "bf16")),
    ((8, 512, 512, "f16"), (5, 264, 520, "f32")),
    ((2, 4096, 2048, "f32"), (70, 1028, 132, "f32")),
]


@pytest.mark.parametrize("first,second", PAIRS)
def test_noalloc_matches_existing_entry_point_twice_in_a_row(rl, first, second):
    import torch
    for n, (M, K, N, dt) in enumerate((first, second)):
        print(f"noalloc case {M}x{K}x{N} {dt} (call {n + 1})", flush=True)
        w = workloads.make(M, K, N, dt, 1e-5, 9100 + M + N + n)
        Y_ref, Y, used_ref, used, Yh, Z = _both(rl, w)
        assert used == used_ref, (used, used_ref)
        assert torch.equal(Y.view(torch.int16), Y_ref.view(torch.int16)), f"{M}x{K}x{N}: differs from rmsnorm_linear"
        ratio, _ = compare(Yh, Z, w.dtype, f"noalloc {M}x{K}x{N}")
        print(f"  variant {used}, max|err|/rms(Y) = {ratio:.3e}", flush=True)


def test_noalloc_uses_the_scratch_array_and_needs_no_workspace(rl):
    """With a lent workspace too small for anything, the existing entry point fails on a split-K shape;
    the new one does not look at it."""
    import torch
    w = workloads.make(1, 4096, 4096, "bf16", 1e-6, 9201)
    X, g, W = upload(w)
    assert rl.rl_workspace_bytes(w.M, w.K, w.N, torch.bfloat16) > 0            # the shape is split over K
    lent = torch.zeros((1280 * 1024 + 16) // 4, dtype=torch.int32, device="cuda")
    rl.rl_set_workspace(lent)
    try:
        with pytest.raises(rl.RmsnlError) as ei:
            rl.rmsnorm_linear(X, g, W, w.eps)
        assert ei.value.status == ERR_WORKSPACE
        Y = torch.empty((w.M, w.N), dtype=torch.bfloat16, device="cuda")
        rl.rmsnorm_linear_noalloc(X, g, W, w.eps, Y)
        torch.cuda.synchronize()
    finally:
        rl.rl_set_workspace(None)
    Y_ref = rl.rmsnorm_linear(X, g, W, w.eps)
    torch.cuda.synchronize()
    assert torch.equal(Y.view(torch.int16), Y_ref.view(torch.int16))


def test_noalloc_large_m_runs_the_one_fused_tile_kernel(rl):
    """X-hat of the two-kernel tile form (2 M K bytes) does not fit the array: the fused tile kernel runs."""
    import torch
    w = workloads.make(2304, 2048, 1024, "bf16", 1e-5, 9301, n_check_rows=64)
    assert 2 * w.M * w.K > rl.rl_noalloc_scratch_bytes()
    _, _, used_ref, used, Yh, Z = _both(rl, w, oracle_rows=w.check_rows)
    assert used == "tile" and used_ref == "tile_pre", (used, used_ref)
    compare(Yh, Z, w.dtype, "noalloc large M")
    # and a small problem right after it on the same array
    w2 = workloads.make(2, 2048, 2048, "bf16", 1e-5, 9302)
    Y_ref, Y, _, _, Yh2, Z2 = _both(rl, w2)
    assert torch.equal(Y.view(torch.int16), Y_ref.view(torch.int16))
    compare(Yh2, Z2, w2.dtype, "noalloc after large M")


def test_noalloc_rejects_what_does_not_fit(rl):
    """Partials beyond the array: a clear error, nothing launched, Y untouched; the next call still works."""
    import torch
    M, K, N = 64, 4096, 28672
    X = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    g = torch.ones(K, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((K, N), dtype=torch.bfloat16, device="cuda")
    Y = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    rl.rl_set_variant("skinny")
    rl.rl_set_tuning(128, 16)                    # 16 slabs of 64 x 28672 fp32 partials = 117 MB
    try:
        st = rl.lib().rmsnorm_linear_noalloc(X.data_ptr(), g.data_ptr(), W.data_ptr(), 1e-5, Y.data_ptr(), M, K, N, 1,
                                             torch.cuda.current_stream().cuda_stream)
        assert st == ERR_WORKSPACE
        assert "scratch" in rl.rl_last_error()
    finally:
        rl.rl_set_variant("auto")
        rl.rl_set_tuning(0, 0)
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())
    w = workloads.make(1, 2048, 1024, "bf16", 1e-6, 9401)
    Y_ref, Y2, _, _, Yh, Z = _both(rl, w)
    assert torch.equal(Y2.view(torch.int16), Y_ref.view(torch.int16))
    compare(Yh, Z, w.dtype, "noalloc after a rejected call")


def test_noalloc_under_graph_capture_replays_bit_for_bit(rl):
    """What the entry point is for: captured in a HIP graph (after one eager call has looked the array up),
    replayed with eager work of the ordinary entry point in between; every replay gives the eager bits."""
    import torch
    dts = {"bf16": 1, "f32": 2}
    for M, K, N, dt in ((1, 4096, 4096, "bf16"), (16, 4096, 1024, "bf16"), (2, 4096, 2048, "f32")):
        w = workloads.make(M, K, N, dt, 1e-5, 9900 + M)
        X, g, W = upload(w)
        Y_ref = rl.rmsnorm_linear(X, g, W, w.eps)
        Y = torch.zeros_like(Y_ref)
        call = lambda: rl.lib().rmsnorm_linear_noalloc(X.data_ptr(), g.data_ptr(), W.data_ptr(), float(w.eps), Y.data_ptr(),
                                                       M, K, N, dts[dt], torch.cuda.current_stream().cuda_stream)
        assert call() == 0, rl.rl_last_error()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            assert call() == 0, rl.rl_last_error()
        for n in range(3):
            Y.zero_()
            other = rl.rmsnorm_linear(X, g, W, w.eps)            # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(Y.view(torch.int16), Y_ref.view(torch.int16)), f"replay {n} of {M}x{K}x{N} {dt} differs"
            assert torch.equal(other.view(torch.int16), Y_ref.view(torch.int16))
