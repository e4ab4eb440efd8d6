"""ctypes binding of librmsnl.so: argument marshalling only.

Every function has the name and meaning of its C entry point in include/rmsnl.h.
Tensors are torch CUDA(HIP) tensors used purely as device buffers; the stream is
torch's current stream unless one is given.  There is no CPU fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("RMSNL_LIB") or os.path.join(_HERE, "librmsnl.so")

RL_OK, RL_ERR_INVALID_ARG, RL_ERR_UNSUPPORTED, RL_ERR_HIP, RL_ERR_WORKSPACE = range(5)
RL_F16, RL_BF16, RL_F32 = range(3)
RL_AUTO, RL_GEMV_SPLITK, RL_MFMA_SKINNY, RL_MFMA_TILE, RL_NAIVE, RL_MFMA_TILE_PRE, RL_MFMA_F32 = range(7)
VARIANTS = {"auto": RL_AUTO, "gemv": RL_GEMV_SPLITK, "skinny": RL_MFMA_SKINNY,
            "tile": RL_MFMA_TILE, "naive": RL_NAIVE, "tile_pre": RL_MFMA_TILE_PRE, "f32": RL_MFMA_F32}
VARIANT_NAMES = {v: k for k, v in VARIANTS.items()}
_DTYPES = {torch.float16: RL_F16, torch.bfloat16: RL_BF16, torch.float32: RL_F32}

EXPORTS = {
    # name: (restype, argtypes)
    "rmsnorm_linear": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                      ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                      ctypes.c_int, ctypes.c_void_p]),
    "rmsnorm_linear_noalloc": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                              ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                              ctypes.c_int, ctypes.c_void_p]),
    "rl_noalloc_scratch_bytes": (ctypes.c_size_t, []),
    "rmsnorm": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p,
                               ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]),
    "matmul": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                              ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]),
    "rmsnorm_gated_mlp": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                         ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                         ctypes.c_int, ctypes.c_void_p]),
    "rmsnorm_gated_mlp_interleaved": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                                     ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                                     ctypes.c_int, ctypes.c_void_p]),
    "rl_interleave_gate_up": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                             ctypes.c_int, ctypes.c_void_p]),
    "rl_qknorm_attention": (ctypes.c_int, [ctypes.c_void_p] * 7 + [ctypes.c_float, ctypes.c_void_p] +
                            [ctypes.c_int64] * 4 + [ctypes.c_int, ctypes.c_void_p]),
    "rl_autotune_qknorm": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int] +
                           [ctypes.c_void_p] * 4 + [ctypes.c_float, ctypes.c_void_p] + [ctypes.c_int64] * 4 +
                           [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int),
                            ctypes.POINTER(ctypes.c_float)]),
    "silu_mul": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                ctypes.c_int, ctypes.c_void_p]),
    "rl_autotune": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p,
                                   ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_float)]),
    "rl_autotune_get": (ctypes.c_int, [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                       ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int),
                                       ctypes.POINTER(ctypes.c_int)]),
    "rl_autotune_clear": (None, []),
    "rl_ntrans": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p,
                                 ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]),
    "rl_ff_rmsnorm_linear": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_uint32,
                                            ctypes.c_int, ctypes.c_void_p]),
    "rl_set_variant": (ctypes.c_int, [ctypes.c_int]),
    "rl_get_variant": (ctypes.c_int, []),
    "rl_last_variant": (ctypes.c_int, []),
    "rl_set_tuning": (ctypes.c_int, [ctypes.c_int, ctypes.c_int]),
    "rl_set_workspace": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t]),
    "rl_set_trace": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t]),
    "rl_trace_slots": (ctypes.c_size_t, []),
    "rl_tile_order": (ctypes.c_int, [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                     ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]),
    "rl_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]),
    "rl_workspace_default_bytes": (ctypes.c_size_t, []),
    "rl_probe_copy": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "rl_probe_read": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]),
    "rl_probe_mfma": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]),
    "rl_probe_mfma_operands": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]),
    "rl_probe_mfma_sink_floats": (ctypes.c_size_t, []),
    "rl_probe_mfma_flops": (ctypes.c_double, [ctypes.c_int]),
    "rl_last_error": (ctypes.c_char_p, []),
    "rl_version": (ctypes.c_char_p, []),
}


class LaunchOpts(ctypes.Structure):
    """rl_launch_opts of include/rmsnl.h."""
    _fields_ = [("struct_size", ctypes.c_size_t), ("variant", ctypes.c_int), ("columns", ctypes.c_int),
                ("slabs", ctypes.c_int), ("waves", ctypes.c_int), ("rem_slabs", ctypes.c_int),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


EXPORTS.update({
    "rmsnorm_linear_ex": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                         ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                         ctypes.c_int, ctypes.POINTER(LaunchOpts), ctypes.c_void_p]),
    "rmsnorm_gated_mlp_ex": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                            ctypes.c_int, ctypes.c_int, ctypes.POINTER(LaunchOpts), ctypes.c_void_p]),
    "rl_last_launch": (ctypes.c_int, [ctypes.POINTER(ctypes.c_int)] * 4),
    "rl_autotune_rotating": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                                            ctypes.c_float, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                            ctypes.POINTER(ctypes.c_float)]),
    "rl_ff_pairs": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                   ctypes.c_int64, ctypes.c_int64, ctypes.c_uint32, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_void_p]),
    "rl_probe_read_strips": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                            ctypes.c_void_p, ctypes.c_void_p]),
    "rl_probe_read_flat": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p,
                                          ctypes.c_void_p]),
})


class RmsnlError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"rmsnl status {status}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` (or "
                              "paper_2405_05751_amd/build.py) to compile the HIP library")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _check(status: int) -> None:
    if status != RL_OK:
        raise RmsnlError(status, lib().rl_last_error().decode())


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def rmsnorm_linear(X: torch.Tensor, g: torch.Tensor, W: torch.Tensor, eps: float,
                   Y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or g.shape != (K,) or X.dtype != W.dtype or X.dtype != g.dtype:
        raise ValueError("shape or dtype mismatch")
    if Y is None:
        Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    elif Y.shape != (M, N) or Y.dtype != X.dtype:
        raise ValueError("Y has the wrong shape or dtype")
    _check(lib().rmsnorm_linear(_dev(X, "X"), _dev(g, "g"), _dev(W, "W"), float(eps), _dev(Y, "Y"),
                                M, K, N, _DTYPES[X.dtype], _stream(stream)))
    return Y


def rmsnorm_linear_noalloc(X: torch.Tensor, g: torch.Tensor, W: torch.Tensor, eps: float, Y: torch.Tensor,
                           stream=None) -> torch.Tensor:
    """rmsnorm_linear through the entry point that allocates nothing; the caller brings Y."""
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or g.shape != (K,) or X.dtype != W.dtype or X.dtype != g.dtype:
        raise ValueError("shape or dtype mismatch")
    if Y.shape != (M, N) or Y.dtype != X.dtype:
        raise ValueError("Y has the wrong shape or dtype")
    _check(lib().rmsnorm_linear_noalloc(_dev(X, "X"), _dev(g, "g"), _dev(W, "W"), float(eps), _dev(Y, "Y"),
                                        M, K, N, _DTYPES[X.dtype], _stream(stream)))
    return Y


def _opts(variant="auto", columns=0, slabs=0, waves=0, rem_slabs=0, workspace: Optional[torch.Tensor] = None):
    o = LaunchOpts()
    o.struct_size = ctypes.sizeof(LaunchOpts)
    o.variant = VARIANTS[variant] if isinstance(variant, str) else int(variant)
    o.columns, o.slabs, o.waves, o.rem_slabs = int(columns), int(slabs), int(waves), int(rem_slabs)
    if workspace is not None:
        o.workspace = _dev(workspace, "workspace")
        o.workspace_bytes = workspace.numel() * workspace.element_size()
    return o


def rmsnorm_linear_ex(X: torch.Tensor, g: torch.Tensor, W: torch.Tensor, eps: float, Y: Optional[torch.Tensor] = None,
                      stream=None, **opts) -> torch.Tensor:
    """rmsnorm_linear with this call's own launch options (variant, columns, slabs, waves, rem_slabs, workspace)."""
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or g.shape != (K,) or X.dtype != W.dtype or X.dtype != g.dtype:
        raise ValueError("shape or dtype mismatch")
    if Y is None:
        Y = torch.empty((M, N), dtype=X.dtype, device=X.device)
    elif Y.shape != (M, N) or Y.dtype != X.dtype:
        raise ValueError("Y has the wrong shape or dtype")
    o = _opts(**opts)
    _check(lib().rmsnorm_linear_ex(_dev(X, "X"), _dev(g, "g"), _dev(W, "W"), float(eps), _dev(Y, "Y"),
                                   M, K, N, _DTYPES[X.dtype], ctypes.byref(o), _stream(stream)))
    return Y


def rmsnorm_gated_mlp_ex(X: torch.Tensor, g: torch.Tensor, W: torch.Tensor, eps: float, Y: Optional[torch.Tensor] = None,
                         interleaved: bool = False, stream=None, **opts) -> torch.Tensor:
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or N % 2 or g.shape != (K,) or X.dtype != W.dtype or X.dtype != g.dtype:
        raise ValueError("shape or dtype mismatch")
    H = N // 2
    if Y is None:
        Y = torch.empty((M, H), dtype=X.dtype, device=X.device)
    elif Y.shape != (M, H) or Y.dtype != X.dtype:
        raise ValueError("Y has the wrong shape or dtype")
    o = _opts(**opts)
    _check(lib().rmsnorm_gated_mlp_ex(_dev(X, "X"), _dev(g, "g"), _dev(W, "W"), float(eps), _dev(Y, "Y"),
                                      M, K, H, _DTYPES[X.dtype], int(bool(interleaved)), ctypes.byref(o), _stream(stream)))
    return Y


def rl_last_launch():
    """(variant name, columns, slabs, workgroups) of the most recent successful call on this thread."""
    v, c, s, w = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().rl_last_launch(ctypes.byref(v), ctypes.byref(c), ctypes.byref(s), ctypes.byref(w)))
    return VARIANT_NAMES[v.value], c.value, s.value, w.value


def rl_probe_read_strips(src: torch.Tensor, rows: int, row_bytes: int, parts: int, sink: torch.Tensor, stream=None) -> None:
    _check(lib().rl_probe_read_strips(_dev(src, "src"), rows, row_bytes, parts, _dev(sink, "sink"), _stream(stream)))


def rl_probe_read_flat(src: torch.Tensor, nbytes: int, workgroups: int, sink: torch.Tensor, stream=None) -> None:
    _check(lib().rl_probe_read_flat(_dev(src, "src"), nbytes, workgroups, _dev(sink, "sink"), _stream(stream)))


def rl_noalloc_scratch_bytes() -> int:
    return int(lib().rl_noalloc_scratch_bytes())


def rmsnorm(X: torch.Tensor, g: torch.Tensor, eps: float, Xn: Optional[torch.Tensor] = None,
            stream=None) -> torch.Tensor:
    M, K = X.shape
    if g.shape != (K,) or g.dtype != X.dtype:
        raise ValueError("shape or dtype mismatch")
    if Xn is None:
        Xn = torch.empty_like(X)
    _check(lib().rmsnorm(_dev(X, "X"), _dev(g, "g"), float(eps), _dev(Xn, "Xn"), M, K,
                         _DTYPES[X.dtype], _stream(stream)))
    return Xn


def matmul(A: torch.Tensor, W: torch.Tensor, Y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K = A.shape
    K2, N = W.shape
    if K2 != K or A.dtype != W.dtype:
        raise ValueError("shape or dtype mismatch")
    if Y is None:
        Y = torch.empty((M, N), dtype=A.dtype, device=A.device)
    _check(lib().matmul(_dev(A, "A"), _dev(W, "W"), _dev(Y, "Y"), M, K, N, _DTYPES[A.dtype],
                        _stream(stream)))
    return Y


def rmsnorm_gated_mlp(X: torch.Tensor, g: torch.Tensor, W: torch.Tensor, eps: float,
                      Y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or N % 2 or g.shape != (K,) or X.dtype != W.dtype or X.dtype != g.dtype:
        raise ValueError("shape or dtype mismatch")
    H = N // 2
    if Y is None:
        Y = torch.empty((M, H), dtype=X.dtype, device=X.device)
    elif Y.shape != (M, H) or Y.dtype != X.dtype:
        raise ValueError("Y has the wrong shape or dtype")
    _check(lib().rmsnorm_gated_mlp(_dev(X, "X"), _dev(g, "g"), _dev(W, "W"), float(eps), _dev(Y, "Y"),
                                   M, K, H, _DTYPES[X.dtype], _stream(stream)))
    return Y


def rmsnorm_gated_mlp_interleaved(X: torch.Tensor, g: torch.Tensor, Wi: torch.Tensor, eps: float,
                                  Y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """rmsnorm_gated_mlp on a W interleaved in groups of 64 columns (see rl_interleave_gate_up)."""
    M, K = X.shape
    K2, N = Wi.shape
    if K2 != K or N % 2 or g.shape != (K,) or X.dtype != Wi.dtype or X.dtype != g.dtype:
        raise ValueError("shape or dtype mismatch")
    H = N // 2
    if Y is None:
        Y = torch.empty((M, H), dtype=X.dtype, device=X.device)
    elif Y.shape != (M, H) or Y.dtype != X.dtype:
        raise ValueError("Y has the wrong shape or dtype")
    _check(lib().rmsnorm_gated_mlp_interleaved(_dev(X, "X"), _dev(g, "g"), _dev(Wi, "Wi"), float(eps), _dev(Y, "Y"),
                                               M, K, H, _DTYPES[X.dtype], _stream(stream)))
    return Y


def rl_interleave_gate_up(W: torch.Tensor, Wi: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """W [K][2H] = [gate | up] -> the layout rmsnorm_gated_mlp_interleaved reads."""
    K, N = W.shape
    if N % 2:
        raise ValueError("W needs an even number of columns")
    if Wi is None:
        Wi = torch.empty_like(W)
    elif Wi.shape != W.shape or Wi.dtype != W.dtype:
        raise ValueError("Wi has the wrong shape or dtype")
    _check(lib().rl_interleave_gate_up(_dev(W, "W"), _dev(Wi, "Wi"), K, N // 2, _DTYPES[W.dtype], _stream(stream)))
    return Wi


def silu_mul(Z: torch.Tensor, Y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, N = Z.shape
    if N % 2:
        raise ValueError("Z needs an even number of columns")
    if Y is None:
        Y = torch.empty((M, N // 2), dtype=Z.dtype, device=Z.device)
    _check(lib().silu_mul(_dev(Z, "Z"), _dev(Y, "Y"), M, N // 2, _DTYPES[Z.dtype], _stream(stream)))
    return Y


def rl_autotune(X: torch.Tensor, g: torch.Tensor, W: torch.Tensor, eps: float, Y: torch.Tensor,
                gated: bool = False, reps: int = 20, stream=None) -> float:
    """Time every launch shape for this call and remember the fastest; returns its microseconds per launch."""
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or g.shape != (K,) or Y.shape != (M, N // 2 if gated else N):
        raise ValueError("shape mismatch")
    best = ctypes.c_float(0.0)
    _check(lib().rl_autotune(_dev(X, "X"), _dev(g, "g"), _dev(W, "W"), float(eps), _dev(Y, "Y"), M, K, N,
                             _DTYPES[X.dtype], int(bool(gated)), int(reps), _stream(stream), ctypes.byref(best)))
    return float(best.value)


def rl_autotune_rotating(X: torch.Tensor, g: torch.Tensor, Ws, eps: float, Y: torch.Tensor, gated: bool = False,
                         interleaved: bool = False, reps: int = 20, stream=None) -> float:
    """rl_autotune on cold data: Ws is a list of device copies of W (of Wi when interleaved) to rotate through."""
    M, K = X.shape
    K2, N = Ws[0].shape
    if K2 != K or g.shape != (K,) or Y.shape != (M, N // 2 if gated else N) or any(w.shape != Ws[0].shape for w in Ws):
        raise ValueError("shape mismatch")
    ptrs = (ctypes.c_void_p * len(Ws))(*[_dev(w, "W copy") for w in Ws])
    best = ctypes.c_float(0.0)
    _check(lib().rl_autotune_rotating(_dev(X, "X"), _dev(g, "g"), ptrs, len(Ws), float(eps), _dev(Y, "Y"), M, K, N,
                                      _DTYPES[X.dtype], int(bool(gated)), int(bool(interleaved)), int(reps),
                                      _stream(stream), ctypes.byref(best)))
    return float(best.value)


def rl_autotune_get(M: int, K: int, N: int, dtype: torch.dtype, gated: bool = False, interleaved: bool = False):
    """(variant name, n_tile, k_split) remembered for the shape; variant "auto" if none."""
    v, nt, ks = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().rl_autotune_get(M, K, N, _DTYPES[dtype], int(bool(gated)) | (2 if interleaved else 0), ctypes.byref(v),
                                 ctypes.byref(nt), ctypes.byref(ks)))
    return VARIANT_NAMES[v.value], nt.value, ks.value


def rl_autotune_clear() -> None:
    lib().rl_autotune_clear()


def rl_ntrans(X: torch.Tensor, Hh: torch.Tensor, alpha: torch.Tensor, eps: float,
              Y: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, D = X.shape
    if Hh.shape != (M, D) or alpha.shape != (D,) or Hh.dtype != X.dtype or alpha.dtype != X.dtype:
        raise ValueError("shape or dtype mismatch")
    if Y is None:
        Y = torch.empty_like(X)
    _check(lib().rl_ntrans(_dev(X, "X"), _dev(Hh, "H"), _dev(alpha, "alpha"), float(eps), _dev(Y, "Y"), M, D,
                           _DTYPES[X.dtype], _stream(stream)))
    return Y


def rl_qknorm_attention(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, gq: torch.Tensor, bq: torch.Tensor,
                        gk: torch.Tensor, bk: torch.Tensor, eps: float, O: Optional[torch.Tensor] = None,
                        stream=None) -> torch.Tensor:
    """LayerNorm of the query and of every key, then attention: Q [B, H, D], K and V [B, H, S, D] -> O [B, H, D]."""
    B, H, D = Q.shape
    S = K.shape[2]
    if K.shape != (B, H, S, D) or V.shape != (B, H, S, D) or any(t.shape != (D,) for t in (gq, bq, gk, bk)) \
            or any(t.dtype != Q.dtype for t in (K, V, gq, bq, gk, bk)):
        raise ValueError("shape or dtype mismatch")
    if O is None:
        O = torch.empty_like(Q)
    _check(lib().rl_qknorm_attention(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(gq, "gq"), _dev(bq, "bq"),
                                     _dev(gk, "gk"), _dev(bk, "bk"), float(eps), _dev(O, "O"), B, H, S, D,
                                     _DTYPES[Q.dtype], _stream(stream)))
    return O


def rl_autotune_qknorm(Q: torch.Tensor, Ks, Vs, gq: torch.Tensor, bq: torch.Tensor, gk: torch.Tensor, bk: torch.Tensor,
                       eps: float, O: torch.Tensor, reps: int = 20, stream=None):
    """Search over the sequence splits of rl_qknorm_attention; Ks and Vs are lists of device copies of K and V
    to rotate through.  Returns (splits chosen, microseconds per launch); splits 0 = nothing to search."""
    B, H, D = Q.shape
    S = Ks[0].shape[2]
    if len(Ks) != len(Vs) or not Ks or any(t.shape != (B, H, S, D) or t.dtype != Q.dtype for t in list(Ks) + list(Vs)) \
            or any(t.shape != (D,) or t.dtype != Q.dtype for t in (gq, bq, gk, bk)) or O.shape != Q.shape:
        raise ValueError("shape or dtype mismatch")
    kp = (ctypes.c_void_p * len(Ks))(*[_dev(t, "K copy") for t in Ks])
    vp = (ctypes.c_void_p * len(Vs))(*[_dev(t, "V copy") for t in Vs])
    splits, best = ctypes.c_int(0), ctypes.c_float(0.0)
    _check(lib().rl_autotune_qknorm(_dev(Q, "Q"), kp, vp, len(Ks), _dev(gq, "gq"), _dev(bq, "bq"), _dev(gk, "gk"),
                                    _dev(bk, "bk"), float(eps), _dev(O, "O"), B, H, S, D, _DTYPES[Q.dtype], int(reps),
                                    _stream(stream), ctypes.byref(splits), ctypes.byref(best)))
    return splits.value, float(best.value)


def rl_ff_rmsnorm_linear(X: torch.Tensor, g: torch.Tensor, W: torch.Tensor, p: int, reordered: bool,
                         stream=None) -> torch.Tensor:
    """The block over Z_p on int32/uint32 device tensors with entries in [0, p); returns Y [M, N] (int32)."""
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or g.shape != (K,) or any(t.dtype != torch.int32 for t in (X, g, W)):
        raise ValueError("shape or dtype mismatch (int32 tensors expected)")
    Y = torch.empty((M, N), dtype=torch.int32, device=X.device)
    _check(lib().rl_ff_rmsnorm_linear(_dev(X, "X"), _dev(g, "g"), _dev(W, "W"), _dev(Y, "Y"), M, K, N, int(p),
                                      int(bool(reordered)), _stream(stream)))
    return Y


def rl_ff_pairs(X: torch.Tensor, g: torch.Tensor, W: torch.Tensor, omega: int, gated: bool, schedule: int,
                slabs: int = 0, stream=None) -> torch.Tensor:
    """The block (or the gated block) on pairs over Z_227 x Z_113: int16 device tensors holding x_p | x_q << 8."""
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or g.shape != (K,) or any(t.dtype != torch.int16 for t in (X, g, W)):
        raise ValueError("shape or dtype mismatch (int16 tensors expected)")
    Y = torch.empty((M, N // 2 if gated else N), dtype=torch.int16, device=X.device)
    _check(lib().rl_ff_pairs(_dev(X, "X"), _dev(g, "g"), _dev(W, "W"), _dev(Y, "Y"), M, K, N, int(omega),
                             int(bool(gated)), int(schedule), int(slabs), _stream(stream)))
    return Y


def rl_set_variant(v) -> None:
    _check(lib().rl_set_variant(VARIANTS[v] if isinstance(v, str) else int(v)))


def rl_get_variant() -> str:
    return VARIANT_NAMES[lib().rl_get_variant()]


def rl_last_variant() -> str:
    return VARIANT_NAMES[lib().rl_last_variant()]


def rl_set_tuning(n_tile: int = 0, k_split: int = 0) -> None:
    _check(lib().rl_set_tuning(int(n_tile), int(k_split)))


def rl_set_workspace(buf: Optional[torch.Tensor]) -> None:
    if buf is None:
        _check(lib().rl_set_workspace(None, 0))
    else:
        _check(lib().rl_set_workspace(_dev(buf, "workspace"), buf.numel() * buf.element_size()))


def rl_set_trace(buf: Optional[torch.Tensor]) -> None:
    """Register (or with None remove) a device int64 buffer for per-workgroup stage time stamps."""
    if buf is None:
        _check(lib().rl_set_trace(None, 0))
    else:
        _check(lib().rl_set_trace(_dev(buf, "trace"), buf.numel() * buf.element_size()))


def rl_trace_slots() -> int:
    return int(lib().rl_trace_slots())


def rl_tile_order(M: int, N: int, position: int):
    """(tile_row, tile_col) of the workgroup at `position` of a tile-kernel launch over an M x N output."""
    tm, tn = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().rl_tile_order(M, N, position, ctypes.byref(tm), ctypes.byref(tn)))
    return int(tm.value), int(tn.value)


def rl_workspace_bytes(M: int, K: int, N: int, dtype: torch.dtype) -> int:
    return int(lib().rl_workspace_bytes(M, K, N, _DTYPES[dtype]))


def rl_workspace_default_bytes() -> int:
    return int(lib().rl_workspace_default_bytes())


def rl_probe_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    _check(lib().rl_probe_copy(_dev(dst, "dst"), _dev(src, "src"), nbytes, _stream(stream)))


def rl_probe_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    _check(lib().rl_probe_read(_dev(src, "src"), nbytes, _dev(sink, "sink"), _stream(stream)))


def rl_probe_mfma(sink: torch.Tensor, iters: int, dtype: torch.dtype = torch.bfloat16, stream=None,
                  zero_operands: bool = False) -> float:
    """Enqueue the matrix-core loop (on pseudo-random operands, or on zeros); returns the flops one launch performs."""
    if sink.numel() < lib().rl_probe_mfma_sink_floats() or sink.dtype != torch.float32:
        raise ValueError("sink too small")
    _check(lib().rl_probe_mfma_operands(_dev(sink, "sink"), int(iters), _DTYPES[dtype], int(bool(zero_operands)),
                                        _stream(stream)))
    return float(lib().rl_probe_mfma_flops(int(iters)))


def rl_last_error() -> str:
    return lib().rl_last_error().decode()


def rl_version() -> str:
    return lib().rl_version().decode()
