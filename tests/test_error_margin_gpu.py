"""How much of the 2e-2 bar the kernels use, over several seeds.  Needs an MI355X.

A bf16 output in [4, 8) is rounded by up to 2^-6 = 0.0156, and outputs of that size occur as soon as
a tensor has a few hundred thousand elements of unit variance: max |err| / rms(Y) of a PERFECT kernel
(the fp64 result rounded once to bf16) is then 1.5e-2 already.  So the test splits the error in two:
the floor (rounding the oracle's own result to bf16, no kernel involved) and what the kernel adds on
top, and bounds the second part.  Up to 32 rows the small-M kernel feeds X (.) g to the matrix cores
as two operands and adds next to nothing; the other kernels round X (.) g once to bf16 first.
"""
import numpy as np
import pytest

import oracle
import workloads
from util import compare, to_host_f64, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rl():
    import torch
    import paper_2405_05751_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.rl_set_variant("auto")
    pkg.rl_set_tuning(0, 0)
    return pkg


def _bf16_rne(z):
    """float64 -> nearest bf16 (ties to even), back in float64."""
    bits = workloads.f32_to_bf16_bits(z.astype(np.float32))
    return workloads.bf16_bits_to_f32(bits).astype(np.float64)


# shape, outlier fraction, checked rows, bound on what the kernel may add to the floor
CASES = [
    ((16, 4096, 6144), 0.0, None, 2.5e-3),       # fused QKV: two-operand X-hat
    ((64, 4096, 28672), 0.01, None, 5e-3),       # gate+up: X-hat rounded once
    ((256, 8192, 8192), 0.0, 32, 5e-3),          # a 256-row slice of the prefill shape: tile kernels
]


@pytest.mark.parametrize("shape,outliers,n_rows,own_bound", CASES)
def test_error_over_five_seeds(rl, shape, outliers, n_rows, own_bound):
    import torch
    M, K, N = shape
    worst_total, worst_floor, worst_own = 0.0, 0.0, 0.0
    for seed in range(5):
        print(f"error margin {M}x{K}x{N} seed {seed}", flush=True)
        w = workloads.make(M, K, N, "bf16", 1e-5, 99000 + 17 * seed + M, outlier_frac=outliers, n_check_rows=n_rows)
        X, g, W = upload(w)
        Y = rl.rmsnorm_linear(X, g, W, w.eps)
        torch.cuda.synchronize()
        rows = w.check_rows
        Z = oracle.rmsnorm_linear(w.X, w.g, w.W, "bf16", w.eps, rows=rows)
        Yh = to_host_f64(Y[torch.from_numpy(rows).cuda()], "bf16")
        total, rms = compare(Yh, Z, "bf16", f"{shape} seed {seed}")             # the bar itself: <= 2e-2
        floor = float(np.abs(_bf16_rne(Z) - Z).max() / rms)
        # the kernel's own part, measured before the output rounding hides or doubles it: distance of Y from
        # the correctly rounded result, less the half ulp by which a nearby fp32 value may round the other way
        own = float(max(0.0, total - floor))
        worst_total, worst_floor, worst_own = max(worst_total, total), max(worst_floor, floor), max(worst_own, own)
        print(f"  {rl.rl_last_variant()}: max|err|/rms(Y) = {total:.3e}, perfect kernel {floor:.3e}, above it {own:.2e}", flush=True)
    assert worst_own <= own_bound, (worst_own, own_bound)
    assert worst_total <= 1.95e-2
