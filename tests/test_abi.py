"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments before touching the GPU.  Runs without a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def rl():
    import paper_2405_05751_amd as pkg
    from paper_2405_05751_amd import build
    if not os.path.exists(pkg.LIB_PATH):
        build.build()
    return pkg


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "rmsnl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([A-Za-z_][A-Za-z0-9_]*)\s*\([^;{}]*\)\s*;", text)
    return sorted(set(names))


def test_header_symbols_exported(rl):
    declared = _declared_functions()
    assert {"rmsnorm_linear", "rmsnorm", "matmul"} <= set(declared)
    handle = ctypes.CDLL(rl.LIB_PATH)
    for name in declared:
        assert hasattr(handle, name), f"{name} declared in rmsnl.h but not exported"


def test_binding_covers_header(rl):
    from paper_2405_05751_amd import binding
    assert sorted(binding.EXPORTS) == _declared_functions()
    for name in ("rmsnorm_linear", "rmsnorm", "matmul"):
        assert callable(getattr(rl, name))


def test_version_and_defaults(rl):
    assert "gfx950" in rl.rl_version()
    assert rl.rl_workspace_default_bytes() >= 32 << 20


ERR_INVALID = 1


@pytest.mark.parametrize("args,frag", [
    ((None, 16, 16, 0.0, 16, 1, 8, 8, 1, None), "null"),
    ((16, 16, 16, 0.0, None, 1, 8, 8, 1, None), "null"),
    ((16, 16, 16, 0.0, 16, 0, 8, 8, 1, None), "M, K, N"),
    ((16, 16, 16, 0.0, 16, 1, 8, 1 << 31, 1, None), "M, K, N"),
    ((16, 16, 16, 0.0, 16, 1, -3, 8, 1, None), "M, K, N"),
    ((16, 16, 16, 0.0, 16, 1, 8, 8, 7, None), "dtype"),
    ((16, 16, 16, float("nan"), 16, 1, 8, 8, 1, None), "eps"),
    ((16, 16, 16, float("inf"), 16, 1, 8, 8, 1, None), "eps"),
    ((16, 16, 16, -1.0, 16, 1, 8, 8, 1, None), "eps"),
    ((16, 16, 24, 0.0, 16, 1, 8, 8, 1, None), "aligned"),
    ((16, 8, 16, 0.0, 16, 1, 8, 8, 1, None), "aligned"),
])
def test_rmsnorm_linear_rejects_bad_arguments(rl, args, frag):
    st = rl.lib().rmsnorm_linear(*args)
    assert st == ERR_INVALID
    assert frag in rl.rl_last_error()


def test_pair_rejects_bad_arguments(rl):
    L = rl.lib()
    assert L.rmsnorm(None, 16, 0.0, 16, 1, 8, 1, None) == ERR_INVALID
    assert L.rmsnorm(16, 16, -0.5, 16, 1, 8, 1, None) == ERR_INVALID
    assert L.rmsnorm(16, 16, 0.0, 16, 1, 0, 1, None) == ERR_INVALID
    assert L.matmul(16, None, 16, 1, 8, 8, 1, None) == ERR_INVALID
    assert L.matmul(16, 16, 16, 1, 8, 8, 3, None) == ERR_INVALID
    assert L.matmul(16, 20, 16, 1, 8, 8, 1, None) == ERR_INVALID


def test_variant_and_tuning_setters(rl):
    L = rl.lib()
    assert L.rl_set_variant(9) == ERR_INVALID
    assert L.rl_set_variant(-1) == ERR_INVALID
    for name in ("gemv", "skinny", "tile", "naive", "auto"):
        rl.rl_set_variant(name)
        assert rl.rl_get_variant() == name
    assert L.rl_set_tuning(-1, 0) == ERR_INVALID
    rl.rl_set_tuning(0, 0)
    assert L.rl_probe_copy(None, 16, 16, None) == ERR_INVALID
    assert L.rl_probe_copy(16, 16, 8, None) == ERR_INVALID
    assert L.rl_probe_mfma(None, 1, 1, None) == ERR_INVALID
    assert L.rl_probe_mfma(16, 1, 2, None) == ERR_INVALID


def test_workspace_bytes_queries(rl):
    import torch
    rl.rl_set_variant("auto")
    assert rl.rl_workspace_bytes(0, 8, 8, torch.bfloat16) == 0
    assert rl.rl_workspace_bytes(1, 4097, 4099, torch.float32) == 0      # plain kernel: no workspace
    # the fp32 kernel splits this shape over K: 4 slabs of M x N fp32 partials behind the 1280 KiB head
    assert rl.rl_workspace_bytes(1, 4096, 4096, torch.float32) == 1280 * 1024 + 4 * 1 * 4096 * 4
    need = rl.rl_workspace_bytes(1, 4096, 4096, torch.bfloat16)
    assert 0 < need <= rl.rl_workspace_default_bytes()


def test_product_does_not_import_oracle():
    """The HIP package must not reach into the oracle (or any CPU fallback)."""
    pkg_dir = os.path.join(ROOT, "paper_2405_05751_amd")
    for dirpath, _, files in os.walk(pkg_dir):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "liboracle" not in text, f


def test_gated_and_tuner_reject_bad_arguments(rl):
    L = rl.lib()
    assert L.rmsnorm_gated_mlp(None, 16, 16, 0.0, 16, 1, 8, 8, 1, None) == ERR_INVALID
    assert L.rmsnorm_gated_mlp(16, 16, 16, 0.0, 16, 1, 8, 0, 1, None) == ERR_INVALID
    assert L.rmsnorm_gated_mlp(16, 16, 16, -1.0, 16, 1, 8, 8, 1, None) == ERR_INVALID
    assert L.silu_mul(None, 16, 1, 8, 1, None) == ERR_INVALID
    assert L.rmsnorm_gated_mlp_interleaved(16, 16, None, 0.0, 16, 1, 8, 64, 1, None) == ERR_INVALID
    assert L.rmsnorm_gated_mlp_interleaved(16, 16, 16, 0.0, 16, 1, 8, 96, 1, None) == ERR_INVALID    # H % 64 != 0
    assert "H % 64" in rl.rl_last_error()
    assert L.rl_interleave_gate_up(16, 16, 8, 64, 1, None) == ERR_INVALID                            # same buffer
    assert L.rl_interleave_gate_up(16, 32, 8, 32, 1, None) == ERR_INVALID
    assert L.rl_interleave_gate_up(16, 32, 0, 64, 1, None) == ERR_INVALID
    assert L.silu_mul(16, 24, 1, 8, 1, None) == ERR_INVALID
    assert L.rl_autotune(None, 16, 16, 0.0, 16, 1, 8, 8, 1, 0, 5, None, None) == ERR_INVALID
    assert L.rl_autotune(16, 16, 16, 0.0, 16, 1, 8, 7, 1, 1, 5, None, None) == ERR_INVALID      # gated needs even N
    assert L.rl_autotune(16, 16, 16, 0.0, 16, 1, 8, 8, 1, 0, 0, None, None) == ERR_INVALID      # reps
    import torch
    rl.rl_autotune_clear()
    assert rl.rl_autotune_get(4, 64, 64, torch.bfloat16) == ("auto", 0, 0)


def test_tile_order_visits_every_tile_once(rl):
    """Host logic of the tile kernels: the launch order is a one-to-one map of positions onto tiles,
    for grids with and without full rounds of 256, band-divisible rows, ragged panels and remainders."""
    for M, N in [(8192, 8192), (2048, 8192), (4096, 14336), (2304, 8192), (1280, 4352), (1100, 264),
                 (300, 256 * 37), (256 * 19, 256 * 23), (256 * 64, 256 * 3), (1, 8)]:
        tm, tn = -(-M // 256), -(-N // 256)
        seen = set()
        for b in range(tm * tn):
            r, c = rl.rl_tile_order(M, N, b)
            assert 0 <= r < tm and 0 <= c < tn, (M, N, b, r, c)
            seen.add((r, c))
        assert len(seen) == tm * tn, (M, N)
    # the 32 workgroups one XCD runs together (positions 8 i + x, 32 consecutive i) form a 4 x 8 block
    for M, N in [(8192, 8192), (2048, 8192), (4096, 14336)]:
        for x in (0, 5):
            tiles = [rl.rl_tile_order(M, N, 8 * i + x) for i in range(32)]
            assert len({r for r, _ in tiles}) <= 4 and len({c for _, c in tiles}) <= 9, (M, N, x, tiles)
    with pytest.raises(rl.RmsnlError):
        rl.rl_tile_order(512, 512, 4)
