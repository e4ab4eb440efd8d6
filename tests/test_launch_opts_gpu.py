"""Per-call launch options and workspace (rmsnorm_linear_ex), the stage trace and the read probes.  Needs an MI355X."""
import numpy as np
import pytest

import oracle
import workloads
from util import compare, compare_gated, to_host_f64, upload

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
    pkg.rl_set_trace(None)


def test_ex_without_options_is_the_plain_call(rl):
    import torch
    for shape in [(1, 2048, 1024), (16, 1024, 2048), (300, 512, 520)]:
        w = workloads.make(*shape, "bf16", 1e-5, 9500 + shape[0])
        X, g, W = upload(w)
        Y0 = rl.rmsnorm_linear(X, g, W, w.eps)
        torch.cuda.synchronize()
        v0 = rl.rl_last_launch()
        Y1 = torch.empty_like(Y0)
        assert rl.lib().rmsnorm_linear_ex(X.data_ptr(), g.data_ptr(), W.data_ptr(), float(w.eps), Y1.data_ptr(),
                                          w.M, w.K, w.N, 1, None, torch.cuda.current_stream().cuda_stream) == 0
        torch.cuda.synchronize()
        assert rl.rl_last_launch() == v0
        assert torch.equal(Y0.view(torch.int16), Y1.view(torch.int16))


@pytest.mark.parametrize("variant,opts", [
    ("gemv", dict(columns=256, slabs=4)), ("gemv", dict(columns=128, slabs=6)),
    ("skinny", dict(columns=128, slabs=3)), ("skinny", dict(columns=64, slabs=5)), ("skinny", dict(slabs=1)),
    ("tile", dict(columns=512, waves=4)), ("tile", dict(waves=8)), ("naive", {}),
])
def test_ex_forces_variant_and_shape_per_call(rl, variant, opts):
    """The options of the call win over the process-wide settings, which stay as they were."""
    import torch
    w = workloads.make(12, 1536, 1024, "bf16", 1e-5, 9600)
    X, g, W = upload(w)
    rl.rl_set_variant("naive")                   # process-wide setting that the call must not follow
    rl.rl_set_tuning(0, 0)
    try:
        Y = rl.rmsnorm_linear_ex(X, g, W, w.eps, variant=variant, **opts)
        torch.cuda.synchronize()
        used, cols, slabs, wgs = rl.rl_last_launch()
    finally:
        rl.rl_set_variant("auto")
    assert used == variant
    if "columns" in opts:
        assert cols == opts["columns"]
    if "slabs" in opts:
        assert slabs == opts["slabs"]
    if "waves" in opts:
        assert slabs == opts["waves"]
    assert rl.rl_get_variant() == "auto"
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    compare(to_host_f64(Y, w.dtype), Z, w.dtype, f"ex {variant} {opts}")


def test_ex_rejects_bad_options(rl):
    import ctypes
    import torch
    w = workloads.make(4, 512, 512, "bf16", 1e-5, 9601)
    X, g, W = upload(w)
    Y = torch.empty((4, 512), dtype=torch.bfloat16, device="cuda")
    args = (X.data_ptr(), g.data_ptr(), W.data_ptr(), float(w.eps), Y.data_ptr(), 4, 512, 512, 1)
    o = rl.LaunchOpts()
    o.struct_size = 8                                        # wrong size
    assert rl.lib().rmsnorm_linear_ex(*args, ctypes.byref(o), None) == 1
    o.struct_size = ctypes.sizeof(rl.LaunchOpts)
    o.variant = 17
    assert rl.lib().rmsnorm_linear_ex(*args, ctypes.byref(o), None) == 1
    o.variant = 2
    o.slabs = -1
    assert rl.lib().rmsnorm_linear_ex(*args, ctypes.byref(o), None) == 1
    o.slabs = 0
    o.columns = 12                                           # skinny: not a multiple of 8
    assert rl.lib().rmsnorm_linear_ex(*args, ctypes.byref(o), None) == 2
    o.columns = 0
    o.workspace = X.data_ptr()
    o.workspace_bytes = 1024                                 # smaller than the head
    assert rl.lib().rmsnorm_linear_ex(*args, ctypes.byref(o), None) == 1


def test_ex_own_workspace_and_two_streams(rl):
    """Two split-K calls in flight at once on two streams, each with its own workspace: both results
    equal those of the same calls run one after the other."""
    import torch
    wa = workloads.make(1, 4096, 4096, "bf16", 1e-6, 9701)
    wb = workloads.make(16, 4096, 3072, "bf16", 1e-5, 9702)
    Xa, ga, Wa = upload(wa)
    Xb, gb, Wb = upload(wb)
    Ya0 = rl.rmsnorm_linear(Xa, ga, Wa, wa.eps)
    Yb0 = rl.rmsnorm_linear(Xb, gb, Wb, wb.eps)
    torch.cuda.synchronize()
    need = max(rl.rl_workspace_bytes(1, 4096, 4096, torch.bfloat16), rl.rl_workspace_bytes(16, 4096, 3072, torch.bfloat16))
    assert need > 0
    ws_a = torch.zeros(need // 4 + 64, dtype=torch.int32, device="cuda")
    ws_b = torch.zeros(need // 4 + 64, dtype=torch.int32, device="cuda")
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    Ya = torch.empty_like(Ya0)
    Yb = torch.empty_like(Yb0)
    torch.cuda.synchronize()
    for rep in range(20):
        rl.rmsnorm_linear_ex(Xa, ga, Wa, wa.eps, Ya, stream=sa, workspace=ws_a)
        rl.rmsnorm_linear_ex(Xb, gb, Wb, wb.eps, Yb, stream=sb, workspace=ws_b)
    torch.cuda.synchronize()
    assert torch.equal(Ya.view(torch.int16), Ya0.view(torch.int16))
    assert torch.equal(Yb.view(torch.int16), Yb0.view(torch.int16))
    # the kernels left the arrival counters (the first 256 KiB) at zero
    assert int(ws_a[: 65536].abs().sum()) == 0 and int(ws_b[: 65536].abs().sum()) == 0
    # too small a workspace for a split call: a clear error, nothing written
    small = torch.zeros((1280 * 1024 + 64) // 4, dtype=torch.int32, device="cuda")
    with pytest.raises(rl.RmsnlError) as ei:
        rl.rmsnorm_linear_ex(Xa, ga, Wa, wa.eps, Ya, workspace=small)
    assert ei.value.status == 4


def test_gated_ex_variants(rl):
    import torch
    w = workloads.make(12, 1024, 2 * 640, "bf16", 1e-5, 9802)
    X, g, W = upload(w)
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    Y0 = rl.rmsnorm_gated_mlp(X, g, W, w.eps)
    Y1 = rl.rmsnorm_gated_mlp_ex(X, g, W, w.eps)
    torch.cuda.synchronize()
    assert torch.equal(Y0.view(torch.int16), Y1.view(torch.int16))
    Wi = rl.rl_interleave_gate_up(W)
    for kw in (dict(variant="gemv"), dict(variant="skinny", slabs=2), dict(variant="tile")):
        Y = rl.rmsnorm_gated_mlp_ex(X, g, W, w.eps, **kw)
        Yi = rl.rmsnorm_gated_mlp_ex(X, g, Wi, w.eps, interleaved=True, **kw)
        torch.cuda.synchronize()
        assert rl.rl_last_launch()[0] == kw["variant"]
        assert torch.equal(Y.view(torch.int16), Yi.view(torch.int16)), kw
        compare_gated(to_host_f64(Y, w.dtype), Z, w.dtype, f"gated ex {kw}")


def test_stage_trace_stamps(rl):
    """rl_set_trace: every traced workgroup's stamps rise from stage to stage, untraced workgroups and
    the rest of the buffer stay untouched, and NULL switches it off."""
    import torch
    slots = rl.rl_trace_slots()
    w = workloads.make(1, 4096, 4096, "bf16", 1e-6, 9901)       # 512 workgroups, 16 slabs
    X, g, W = upload(w)
    Y = rl.rmsnorm_linear(X, g, W, w.eps)
    torch.cuda.synchronize()
    _, _, slabs, wgs = rl.rl_last_launch()
    assert wgs == 512 and slabs == 16
    room = 300                                                   # fewer than the launch has
    buf = torch.full(((room + 8) * slots,), -1, dtype=torch.int64, device="cuda")
    rl.rl_set_trace(buf[: room * slots])
    try:
        Y2 = rl.rmsnorm_linear(X, g, W, w.eps)
        torch.cuda.synchronize()
    finally:
        rl.rl_set_trace(None)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))
    t = buf.cpu().numpy().reshape(-1, slots)
    assert (t[room:] == -1).all(), "stamps beyond the registered bytes"
    assert (t[:room, 8:] == -1).all(), "only stages 0 to 7 exist"
    tr = t[:room, :8]
    assert (tr[:, :6] > 0).all(), "every traced workgroup passes stages 0 to 5"
    assert (np.diff(tr[:, :6], axis=1) >= 0).all(), "stamps must not go back in time"
    last = tr[:, 6] > 0                                          # the last arrivers of their tiles
    assert 0 < last.sum() <= 32
    assert (tr[last, 7] >= tr[last, 6]).all() and (tr[last, 6] >= tr[last, 5]).all()
    assert (tr[~last, 6:] == -1).all()
    span_us = (tr[:, :6].max() - tr[:, 0].min()) / 100.0         # 100 MHz clock
    assert 1.0 < span_us < 200.0, span_us
    buf.fill_(-1)
    rl.rmsnorm_linear(X, g, W, w.eps)                            # switched off: nothing is written
    torch.cuda.synchronize()
    assert bool((buf == -1).all())


def test_read_probes_run_and_reject(rl):
    import torch
    src = torch.randint(0, 1 << 30, (4096 * 8192 // 4,), dtype=torch.int32, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    for parts in (1, 3, 16):
        rl.rl_probe_read_strips(src, 4096, 8192, parts, sink)
    rl.rl_probe_read_strips(src, 1000, 8192, 7, sink)           # ragged rows
    for wgs in (1, 256, 1000):
        rl.rl_probe_read_flat(src, src.numel() * 4, wgs, sink)
    rl.rl_probe_read_flat(src, 16 * 1000, 3, sink)
    torch.cuda.synchronize()
    L = rl.lib()
    assert L.rl_probe_read_strips(src.data_ptr(), 4096, 8200, 1, sink.data_ptr(), None) == 1     # not a multiple of 256
    assert L.rl_probe_read_strips(src.data_ptr(), 4096, 8192, 0, sink.data_ptr(), None) == 1
    assert L.rl_probe_read_strips(src.data_ptr(), 1 << 20, 8192, 1, sink.data_ptr(), None) == 1   # beyond 2^31 bytes
    assert L.rl_probe_read_flat(src.data_ptr(), 24, 1, sink.data_ptr(), None) == 1
    assert L.rl_probe_read_flat(src.data_ptr(), 1024, 0, sink.data_ptr(), None) == 1


def test_autotune_on_rotating_copies_and_the_interleaved_layout(rl):
    """rl_autotune_rotating: the search runs on copies of W in rotation, remembers its pick per layout,
    RL_AUTO then launches exactly that shape, and the result is still the block."""
    import torch
    w = workloads.make(16, 1024, 2 * 640, "bf16", 1e-5, 9950)
    X, g, W = upload(w)
    Ws = [W] + [W.clone() for _ in range(3)]
    Wis = [rl.rl_interleave_gate_up(v) for v in Ws]
    Z = oracle.rmsnorm_linear(w.X, w.g, w.W, w.dtype, w.eps)
    rl.rl_autotune_clear()
    try:
        Y = torch.empty((w.M, w.N), dtype=torch.bfloat16, device="cuda")
        us = rl.rl_autotune_rotating(X, g, Ws, w.eps, Y, reps=8)
        assert 1.0 < us < 1000.0
        v, nt, ks = rl.rl_autotune_get(w.M, w.K, w.N, torch.bfloat16)
        assert v in ("gemv", "skinny", "tile")
        assert rl.rl_autotune_get(w.M, w.K, w.N, torch.bfloat16, gated=True) == ("auto", 0, 0)     # other layouts untouched
        Y = rl.rmsnorm_linear(X, g, W, w.eps)
        torch.cuda.synchronize()
        used, cols, slabs, _ = rl.rl_last_launch()
        assert used == v and (nt == 0 or cols == nt) and (ks == 0 or slabs == ks)
        compare(to_host_f64(Y, w.dtype), Z, w.dtype, "tuned plain block")
        Yg = torch.empty((w.M, w.N // 2), dtype=torch.bfloat16, device="cuda")
        rl.rl_autotune_rotating(X, g, Wis, w.eps, Yg, gated=True, interleaved=True, reps=8)
        vi, nti, ksi = rl.rl_autotune_get(w.M, w.K, w.N, torch.bfloat16, gated=True, interleaved=True)
        assert vi in ("gemv", "skinny", "tile")
        assert rl.rl_autotune_get(w.M, w.K, w.N, torch.bfloat16, gated=True) == ("auto", 0, 0)
        Yi = rl.rmsnorm_gated_mlp_interleaved(X, g, Wis[0], w.eps)
        torch.cuda.synchronize()
        assert rl.rl_last_launch()[0] == vi
        compare_gated(to_host_f64(Yi, w.dtype), Z, w.dtype, "tuned interleaved gated block")
    finally:
        rl.rl_autotune_clear()
    with pytest.raises(rl.RmsnlError):
        rl.rl_autotune_rotating(X, g, Ws, w.eps, Y, interleaved=True, reps=4)        # interleaved is the gated block's
