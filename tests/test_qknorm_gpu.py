"""Parity of rl_qknorm_attention (layer normalisation of query and keys fused with decode attention)
against the fp64 oracle, through the C ABI.  Needs an MI355X.

Bar: per (sample, head) output vector, max |err| <= tol * rms(vector) with tol = 2e-2 for f16/bf16
(one rounding of the output to the storage type, fp32 arithmetic before it) and 1e-4 for f32 (the
fp32 error of a score, about 1e-6 relative on values up to 10, goes through the exponential)."""
import numpy as np
import pytest

import oracle
import workloads
from util import to_device, to_host_f64

pytestmark = pytest.mark.gpu
TOL = {"f16": 2e-2, "bf16": 2e-2, "f32": 1e-4}


@pytest.fixture(scope="module")
def rl():
    import torch
    import paper_2405_05751_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


def _check(rl, c, dtype, eps, what):
    import torch
    dev = {k: to_device(v, dtype) for k, v in c.items()}
    O = rl.rl_qknorm_attention(dev["Q"], dev["K"], dev["V"], dev["gq"], dev["bq"], dev["gk"], dev["bk"], eps)
    torch.cuda.synchronize()
    got = to_host_f64(O, dtype)
    want = oracle.qknorm_attention(c["Q"], c["K"], c["V"], c["gq"], c["bq"], c["gk"], c["bk"], dtype, eps)
    assert got.shape == want.shape
    assert np.isfinite(got).all(), what
    err = np.abs(got - want).max(axis=-1)
    rms = np.sqrt((want ** 2).mean(axis=-1))
    worst = float((err / rms).max())
    assert worst <= TOL[dtype], f"{what}: max|err|/rms = {worst:.3e} > {TOL[dtype]}"
    return worst


# fast path: D = 128, 16-bit; sequence lengths around the 16-position iteration, the ring of six
# iterations, split boundaries; few and many heads (one split, many splits)
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("B,H,S", [(1, 1, 1), (1, 2, 15), (1, 3, 16), (2, 2, 17), (1, 1, 97), (1, 4, 1000),
                                   (2, 3, 1031), (1, 32, 4096), (8, 32, 512), (3, 5, 4100), (1, 1, 8192),
                                   (64, 16, 130)])
def test_fast_path(rl, B, H, S, dtype):
    c = workloads.make_attention(B, H, S, 128, dtype, 9100 + B * 7 + H * 3 + S)
    worst = _check(rl, c, dtype, 1e-5, f"qknorm attention {B}x{H}x{S}x128 {dtype}")
    print(f"{B}x{H}x{S}x128 {dtype}: max|err|/rms = {worst:.3e}")


# the same kernel with 8 and with 32 lanes to a key (D = 64: 32 positions per iteration, D = 256: 8):
# lengths around one iteration, around the ring of six, ragged splits, one and many splits
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("D", [64, 256])
@pytest.mark.parametrize("B,H,S", [(1, 1, 1), (1, 2, 7), (1, 3, 8), (2, 2, 9), (1, 2, 31), (1, 1, 32), (2, 1, 33),
                                   (1, 1, 191), (1, 3, 193), (1, 4, 1000), (2, 3, 1031), (1, 32, 4096), (8, 32, 300),
                                   (3, 5, 4100), (1, 1, 8192)])
def test_fast_path_other_head_sizes(rl, B, H, S, D, dtype):
    c = workloads.make_attention(B, H, S, D, dtype, 9200 + B * 7 + H * 3 + S + D)
    worst = _check(rl, c, dtype, 1e-5, f"qknorm attention {B}x{H}x{S}x{D} {dtype}")
    print(f"{B}x{H}x{S}x{D} {dtype}: max|err|/rms = {worst:.3e}")


@pytest.mark.parametrize("D", [64, 256])
def test_fast_path_forced_splits(rl, D):
    """Every split count the tuning knob allows, on a length that leaves a ragged last split."""
    c = workloads.make_attention(1, 2, 1500, D, "bf16", 9250 + D)
    try:
        for splits in (1, 2, 3, 7, 16, 23):
            rl.rl_set_tuning(0, splits)
            _check(rl, c, "bf16", 1e-5, f"D = {D}, {splits} splits")
    finally:
        rl.rl_set_tuning(0, 0)


@pytest.mark.parametrize("dtype,D", [("f32", 128), ("f32", 64), ("bf16", 96), ("f16", 80), ("bf16", 512), ("f32", 7)])
@pytest.mark.parametrize("B,H,S", [(1, 1, 1), (2, 3, 300), (1, 2, 1025)])
def test_plain_path(rl, B, H, S, D, dtype):
    c = workloads.make_attention(B, H, S, D, dtype, 9300 + B + H + S + D)
    _check(rl, c, dtype, 1e-5, f"qknorm attention {B}x{H}x{S}x{D} {dtype}")


def test_split_tuner(rl):
    """The tuner over sequence splits: it picks a count, later calls of that shape run it and still match
    the oracle; a shape of the plain kernel has nothing to search."""
    import torch
    for D, B, H, S in ((128, 1, 8, 2048), (64, 2, 3, 1100), (256, 1, 2, 640)):
        c = workloads.make_attention(B, H, S, D, "bf16", 9800 + D)
        dev = {k: to_device(v, "bf16") for k, v in c.items()}
        Ks = [dev["K"], dev["K"].clone()]
        Vs = [dev["V"], dev["V"].clone()]
        O = torch.empty_like(dev["Q"])
        try:
            splits, us = rl.rl_autotune_qknorm(dev["Q"], Ks, Vs, dev["gq"], dev["bq"], dev["gk"], dev["bk"], 1e-5, O, reps=5)
            assert 1 <= splits <= max(1, S // 64) and us > 0, (splits, us)
            print(f"D = {D}, {B}x{H}x{S}: {splits} splits, {us:.1f} us")
            _check(rl, c, "bf16", 1e-5, f"after tuning, D = {D}")
        finally:
            rl.rl_autotune_clear()
        _check(rl, c, "bf16", 1e-5, f"after forgetting, D = {D}")
    c = workloads.make_attention(1, 2, 100, 80, "f16", 9810)
    dev = {k: to_device(v, "f16") for k, v in c.items()}
    O = torch.empty_like(dev["Q"])
    assert rl.rl_autotune_qknorm(dev["Q"], [dev["K"]], [dev["V"]], dev["gq"], dev["bq"], dev["gk"], dev["bk"], 1e-5, O)[0] == 0
    with pytest.raises(rl.RmsnlError):
        rl.rl_autotune_qknorm(dev["Q"], [dev["K"]], [dev["V"]], dev["gq"], dev["bq"], dev["gk"], dev["bk"], 1e-5, O, reps=0)


def test_eps_zero_and_peaked_scores(rl):
    """eps = 0, and keys whose gain makes the scores span a wide range (a sharply peaked softmax)."""
    c = workloads.make_attention(2, 4, 777, 128, "bf16", 9500)
    _check(rl, c, "bf16", 0.0, "eps = 0")
    big = workloads.to_storage(workloads.to_f32(c["gk"], "bf16") * np.float32(6.0), "bf16")
    _check(rl, dict(c, gk=big), "bf16", 1e-5, "peaked softmax")


def test_output_canaries_and_reuse(rl):
    """Nothing is written outside O, and a second call with a shorter sequence is not disturbed by
    what the first left in the workspace."""
    import torch
    c = workloads.make_attention(2, 8, 2048, 128, "bf16", 9600)
    dev = {k: to_device(v, "bf16") for k, v in c.items()}
    buf = torch.full((2 * 8 * 128 + 512,), 7.0, dtype=torch.bfloat16, device="cuda")
    O = buf[256:256 + 2 * 8 * 128].view(2, 8, 128)
    rl.rl_qknorm_attention(dev["Q"], dev["K"], dev["V"], dev["gq"], dev["bq"], dev["gk"], dev["bk"], 1e-5, O)
    torch.cuda.synchronize()
    assert (buf[:256] == 7.0).all() and (buf[256 + 2 * 8 * 128:] == 7.0).all()
    want = oracle.qknorm_attention(c["Q"], c["K"], c["V"], c["gq"], c["bq"], c["gk"], c["bk"], "bf16", 1e-5)
    got = to_host_f64(O.contiguous(), "bf16")
    assert (np.abs(got - want).max(-1) / np.sqrt((want ** 2).mean(-1))).max() <= 2e-2
    c2 = workloads.make_attention(1, 3, 100, 128, "bf16", 9601)
    _check(rl, c2, "bf16", 1e-5, "second, smaller call")


def test_hand_case_q1_on_gpu(rl, golden_hand_cases):
    """The D = 2 closed form through the plain kernel, in all three types."""
    import torch
    w = lambda a: np.asarray(a, dtype=np.float32)
    arrs = (w([[[3.0, 1.0]]]), w([[[[2.0, 0.0], [0.0, 5.0]]]]), w([[[[1.0, 0.0], [0.0, 1.0]]]]),
            w([1, 1]), w([0.5, 0.0]), w([1, 1]), w([0, 0]))
    want = np.array([golden_hand_cases["Q1"][(0, j)] for j in range(2)])
    for dtype, tol in (("f32", 1e-6), ("f16", 2e-3), ("bf16", 1e-2)):
        # 16-byte alignment: every operand in its own allocation
        dev = [to_device(workloads.to_storage(a, dtype), dtype) for a in arrs]
        O = rl.rl_qknorm_attention(*dev, 0.0)
        torch.cuda.synchronize()
        np.testing.assert_allclose(to_host_f64(O, dtype)[0, 0], want, rtol=tol)


def test_argument_checks(rl):
    import torch
    c = workloads.make_attention(1, 2, 32, 128, "bf16", 9700)
    dev = {k: to_device(v, "bf16") for k, v in c.items()}
    with pytest.raises(ValueError):
        rl.rl_qknorm_attention(dev["Q"], dev["K"][:, :, :16], dev["V"], dev["gq"], dev["bq"], dev["gk"], dev["bk"], 1e-5)
    with pytest.raises(rl.RmsnlError) as ei:
        rl.rl_qknorm_attention(dev["Q"], dev["K"], dev["V"], dev["gq"], dev["bq"], dev["gk"], dev["bk"], -1.0)
    assert ei.value.status == 1
    torch.cuda.synchronize()
