"""Python face of the C oracle (oracle/rmsnorm_linear_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg, never by the HIP package.  Everything returned
is float64 and is never rounded to the 16-bit storage type.

Arrays use the storage conventions of the input generators: numpy float16
for "f16", numpy float32 for "f32", numpy uint16 (upper half of the float32
bit pattern) for "bf16".
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_DT = {"f16": 0, "bf16": 1, "f32": 2}
_NP = {"f16": np.float16, "bf16": np.uint16, "f32": np.float32}
_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        lib.oracle_decode_f16.restype = ctypes.c_double
        lib.oracle_decode_f16.argtypes = [ctypes.c_uint16]
        lib.oracle_decode_bf16.restype = ctypes.c_double
        lib.oracle_decode_bf16.argtypes = [ctypes.c_uint16]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_decode.restype = None
        lib.oracle_decode.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p]
        lib.oracle_rmsnorm_f64.restype = None
        lib.oracle_rmsnorm_f64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double,
                                           ctypes.c_long, ctypes.c_long, ctypes.c_void_p]
        lib.oracle_matmul_f64.restype = None
        lib.oracle_matmul_f64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_long,
                                          ctypes.c_long, ctypes.c_long, ctypes.c_void_p]
        lib.oracle_rmsnorm_linear.restype = ctypes.c_int
        lib.oracle_rmsnorm_linear.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_int, ctypes.c_double, ctypes.c_long,
                                              ctypes.c_long, ctypes.c_long, ctypes.c_void_p,
                                              ctypes.c_long, ctypes.c_void_p]
        lib.oracle_ntrans.restype = ctypes.c_int
        lib.oracle_ntrans.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                      ctypes.c_double, ctypes.c_long, ctypes.c_long, ctypes.c_void_p]
        lib.oracle_qknorm_attention.restype = ctypes.c_int
        lib.oracle_qknorm_attention.argtypes = [ctypes.c_void_p] * 7 + [ctypes.c_int, ctypes.c_double] + \
            [ctypes.c_long] * 4 + [ctypes.c_void_p]
        lib.oracle_silu_mul_f64.restype = None
        lib.oracle_silu_mul_f64.argtypes = [ctypes.c_void_p, ctypes.c_long, ctypes.c_long, ctypes.c_void_p]
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the oracle's OpenMP loops will use."""
    return int(_load().oracle_num_threads())


def _storage(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != _NP[dtype]:
        raise TypeError(f"{dtype} arrays must be numpy {_NP[dtype].__name__}, got {a.dtype}")
    return a


def decode(a, dtype: str) -> np.ndarray:
    """Widen a storage array to float64 with the oracle's own decoders."""
    a = _storage(a, dtype)
    out = np.empty(a.shape, dtype=np.float64)
    _load().oracle_decode(a.ctypes.data, _DT[dtype], a.size, out.ctypes.data)
    return out


def decode_f16_scalar(bits: int) -> float:
    return float(_load().oracle_decode_f16(int(bits) & 0xFFFF))


def decode_bf16_scalar(bits: int) -> float:
    return float(_load().oracle_decode_bf16(int(bits) & 0xFFFF))


def rmsnorm_f64(x, g, eps: float) -> np.ndarray:
    """Eq. 1 on float64 arrays: x [M,K], g [K] -> [M,K]."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float64)
    M, K = x.shape
    assert g.shape == (K,)
    out = np.empty((M, K), dtype=np.float64)
    _load().oracle_rmsnorm_f64(x.ctypes.data, g.ctypes.data, float(eps), M, K, out.ctypes.data)
    return out


def matmul_f64(a, w) -> np.ndarray:
    """Plain float64 product: a [M,K] @ w [K,N]."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    M, K = a.shape
    K2, N = w.shape
    assert K == K2
    z = np.empty((M, N), dtype=np.float64)
    _load().oracle_matmul_f64(a.ctypes.data, w.ctypes.data, M, K, N, z.ctypes.data)
    return z


def rmsnorm_linear(X, g, W, dtype: str, eps: float, rows=None) -> np.ndarray:
    """The whole block on storage-typed inputs; returns float64 [len(rows), N].

    `eps` is taken as given (pass the float32-rounded value the GPU receives).
    `rows` defaults to every row of X.
    """
    X = _storage(X, dtype)
    g = _storage(g, dtype)
    W = _storage(W, dtype)
    M, K = X.shape
    K2, N = W.shape
    if K2 != K or g.shape != (K,):
        raise ValueError("shape mismatch")
    rows = np.arange(M, dtype=np.int64) if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    Z = np.empty((len(rows), N), dtype=np.float64)
    rc = _load().oracle_rmsnorm_linear(X.ctypes.data, g.ctypes.data, W.ctypes.data, _DT[dtype],
                                       float(eps), M, K, N, rows.ctypes.data, len(rows),
                                       Z.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle_rmsnorm_linear rejected its arguments")
    return Z


def rmsnorm(X, g, dtype: str, eps: float) -> np.ndarray:
    """Eq. 1 on storage-typed inputs; float64 [M,K] (unfused A/B leg)."""
    return rmsnorm_f64(decode(X, dtype), decode(g, dtype), eps)


def matmul(A, W, dtype: str) -> np.ndarray:
    """Plain product on storage-typed inputs; float64 [M,N] (unfused A/B leg)."""
    return matmul_f64(decode(A, dtype), decode(W, dtype))


def silu_mul_f64(z) -> np.ndarray:
    """Gate of the GatedMLP block on float64: z [R, 2H] read as [gate | up] -> SiLU(gate) * up, [R, H]."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    R, N = z.shape
    if N % 2:
        raise ValueError("the gated block needs an even number of columns")
    y = np.empty((R, N // 2), dtype=np.float64)
    _load().oracle_silu_mul_f64(z.ctypes.data, R, N // 2, y.ctypes.data)
    return y


def rmsnorm_gated_mlp(X, g, W, dtype: str, eps: float, rows=None) -> np.ndarray:
    """RMSNorm, the two products (W = [gate | up], [K, 2H]), SiLU(gate) * up; float64 [len(rows), H].

    The block's fp64 output is not rounded before the gate.
    """
    return silu_mul_f64(rmsnorm_linear(X, g, W, dtype, eps, rows=rows))


def ntrans(X, Hh, alpha, dtype: str, eps: float) -> np.ndarray:
    """nTrans chain y = Norm(x + alpha * Norm(h - x)) on storage-typed inputs; float64 [M, D]."""
    X = _storage(X, dtype); Hh = _storage(Hh, dtype); alpha = _storage(alpha, dtype)
    M, D = X.shape
    if Hh.shape != (M, D) or alpha.shape != (D,):
        raise ValueError("shape mismatch")
    Y = np.empty((M, D), dtype=np.float64)
    if _load().oracle_ntrans(X.ctypes.data, Hh.ctypes.data, alpha.ctypes.data, _DT[dtype], float(eps), M, D,
                             Y.ctypes.data) != 0:
        raise RuntimeError("oracle_ntrans rejected its arguments")
    return Y


def qknorm_attention(Q, K, V, gq, bq, gk, bk, dtype: str, eps: float) -> np.ndarray:
    """LayerNorm of the query and of every key, then attention, one query per (sample, head), on
    storage-typed inputs: Q [B, H, D], K and V [B, H, S, D], gains and biases [D]; float64 [B, H, D]."""
    Q = _storage(Q, dtype); K = _storage(K, dtype); V = _storage(V, dtype)
    gq = _storage(gq, dtype); bq = _storage(bq, dtype); gk = _storage(gk, dtype); bk = _storage(bk, dtype)
    B, H, D = Q.shape
    S = K.shape[2]
    if K.shape != (B, H, S, D) or V.shape != (B, H, S, D) or any(v.shape != (D,) for v in (gq, bq, gk, bk)):
        raise ValueError("shape mismatch")
    O = np.empty((B, H, D), dtype=np.float64)
    if _load().oracle_qknorm_attention(Q.ctypes.data, K.ctypes.data, V.ctypes.data, gq.ctypes.data, bq.ctypes.data,
                                       gk.ctypes.data, bk.ctypes.data, _DT[dtype], float(eps), B, H, S, D,
                                       O.ctypes.data) != 0:
        raise RuntimeError("oracle_qknorm_attention rejected its arguments")
    return O


# ---------------------------------------------------------------------------------------------
# The block over a prime field (the paper's random tests over finite fields, Table 3): the same
# graph evaluated with modular arithmetic.  Python integers, one operation at a time.
# ---------------------------------------------------------------------------------------------
def ff_sqrt(x: int, p: int) -> int:
    """Canonical square root in Z_p: the smallest y with y*y = x; for a non-residue x, the smallest
    y with y*y = x*n, n the least non-residue (so the function is total, and non-zero for x != 0)."""
    x %= p
    squares = {}
    for y in range(p):
        squares.setdefault(y * y % p, y)
    if x in squares:
        return squares[x]
    n = next(v for v in range(2, p) if v not in squares)
    return squares[x * n % p]


def ff_rmsnorm_linear(X, g, W, p: int, reordered: bool):
    """Eq. 1 then the product over Z_p (reordered=False), or the rewritten form (division after the
    product, reordered=True).  X [M][K], g [K], W [K][N] integer arrays with entries in [0, p).
    A row whose mean square is 0 has no inverse root: its outputs are defined as 0 in both forms."""
    X = np.asarray(X, dtype=np.int64); g = np.asarray(g, dtype=np.int64); W = np.asarray(W, dtype=np.int64)
    M, K = X.shape
    N = W.shape[1]
    inv = lambda v: pow(int(v), p - 2, p)
    Y = np.zeros((M, N), dtype=np.int64)
    for i in range(M):
        a = 0
        for k in range(K):
            a = (a + int(X[i, k]) * int(X[i, k])) % p
        r = ff_sqrt(a * inv(K % p) % p, p)
        if r == 0:
            continue
        rinv = inv(r)
        for n in range(N):
            acc = 0
            for k in range(K):
                if reordered:
                    acc = (acc + (int(X[i, k]) * int(g[k]) % p) * int(W[k, n])) % p
                else:
                    acc = (acc + ((int(X[i, k]) * int(g[k]) % p) * rinv % p) * int(W[k, n])) % p
            Y[i, n] = acc * rinv % p if reordered else acc
    return Y


# ---------------------------------------------------------------------------------------------
# Random tests over TWO fields (Table 3 in full): every value is a pair (x_p, x_q) from Z_p x Z_q,
# q a prime that divides p - 1.  Add, Sub, Mul, Div and Sqrt act on the two components
# independently; Exp takes the q component into the exponent of a q-th root of unity omega of Z_p
# and yields a p component only: (omega^{x_q} mod p, -).  An exponential may occur once on a path.
# Arrays of pairs have a last axis of length 2, [..., 0] the p component and [..., 1] the q component.
# ---------------------------------------------------------------------------------------------
def ff_roots_of_unity(p: int, q: int):
    """The q-th roots of unity of Z_p (all w with w^q = 1; there are q of them when q divides p - 1)."""
    if (p - 1) % q:
        raise ValueError("q must divide p - 1")
    return [w for w in range(1, p) if pow(w, q, p) == 1]


def ff_exp(x_q: int, omega: int, p: int, q: int) -> int:
    """The Exp row of Table 3: omega^{x_q} mod p for x_q in Z_q."""
    return pow(int(omega), int(x_q) % q, p)


def ff_pair_rmsnorm_linear(X, g, W, p: int, q: int, reordered: bool):
    """The block on pairs: each component is the block over its own field (Add, Mul, Div, Sqrt rows)."""
    X = np.asarray(X, dtype=np.int64); g = np.asarray(g, dtype=np.int64); W = np.asarray(W, dtype=np.int64)
    Zp = ff_rmsnorm_linear(X[..., 0], g[..., 0], W[..., 0], p, reordered)
    Zq = ff_rmsnorm_linear(X[..., 1], g[..., 1], W[..., 1], q, reordered)
    return np.stack([Zp, Zq], axis=-1)


def ff_pair_gated_mlp(X, g, W, p: int, q: int, omega: int, reordered: bool):
    """The gated block on pairs: Z = the block on W = [gate | up]; Y = SiLU(G) * U with
    SiLU(v) = v / (1 + exp(-v)).  The exponential takes the q component of -G and leaves a p
    component (Exp row); everything after it is arithmetic in Z_p, so Y has a p component only.
    Where 1 + exp(-G) has no inverse (it is 0 in Z_p) the output is defined as 0.
    reordered selects the graph Z is evaluated with (Eq. 1 first, or division after the product)."""
    Z = ff_pair_rmsnorm_linear(X, g, W, p, q, reordered)
    M, N, _ = Z.shape
    H = N // 2
    Y = np.zeros((M, H), dtype=np.int64)
    for i in range(M):
        for h in range(H):
            G_p, G_q = int(Z[i, h, 0]), int(Z[i, h, 1])
            U_p = int(Z[i, H + h, 0])
            e = ff_exp((-G_q) % q, omega, p, q)
            den = (1 + e) % p
            if den == 0:
                continue
            Y[i, h] = G_p * pow(den, p - 2, p) % p * U_p % p
    return Y
