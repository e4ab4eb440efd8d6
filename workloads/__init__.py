"""Seeded synthetic inputs for the RMSNorm-then-linear block.

This module only draws random numbers, rounds them to the storage type and
names the shapes.  It contains none of the method's arithmetic (no norm, no
product), so the CPU oracle and the HIP library can both be fed from it
without sharing anything that could hide a common mistake.

The shapes stand in for the paper's "RMSNorm" benchmark (a LLaMA-style
normalisation followed by a projection, evaluation section, benchmark table):
the paper itself times random inputs because run time depends on shapes only.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

SEED = 240505751

# name, M, K, N, dtype, eps, fraction of rows scaled x20, checked-row count (None = all)
_CONFIGS = (
    ("tiny",    8,    512,  512,   "f16",  1e-6, 0.0,  None),
    ("decode",  1,    4096, 4096,  "bf16", 1e-6, 0.0,  None),
    ("qkv",     16,   4096, 6144,  "bf16", 1e-5, 0.0,  None),
    ("gateup",  64,   4096, 28672, "bf16", 1e-5, 0.01, None),
    ("prefill", 8192, 8192, 8192,  "bf16", 1e-5, 0.0,  256),
)
CONFIG_NAMES = tuple(c[0] for c in _CONFIGS)

ELEM_BYTES = {"f16": 2, "bf16": 2, "f32": 4}


@dataclasses.dataclass
class Workload:
    """One problem instance.  X, g, W hold the exact bits both sides consume.

    f16 -> numpy float16, f32 -> numpy float32, bf16 -> numpy uint16 holding
    the upper half of the float32 pattern.
    """
    name: str
    M: int
    K: int
    N: int
    dtype: str
    eps: float
    X: np.ndarray
    g: np.ndarray
    W: np.ndarray
    check_rows: np.ndarray          # sorted row indices the oracle evaluates
    outlier_rows: np.ndarray

    @property
    def algorithmic_bytes(self) -> int:
        """Read X, g, W once and write Y once."""
        b = ELEM_BYTES[self.dtype]
        return b * (self.M * self.K + self.K + self.K * self.N + self.M * self.N)

    @property
    def flops(self) -> int:
        """2*M*K*N: the contraction only, the norm's flops are not counted."""
        return 2 * self.M * self.K * self.N


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bits to float32."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float32/float64 array once to the storage type."""
    if dtype == "f16":
        return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError(f"unknown dtype {dtype!r}")


def to_f32(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a storage array to float32 (for display / marshalling)."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a)
    return a.astype(np.float32)


def make(M: int, K: int, N: int, dtype: str, eps: float, seed: int, *,
         name: str = "custom", outlier_frac: float = 0.0,
         n_check_rows: Optional[int] = None) -> Workload:
    """Draw X ~ N(0,1), g ~ U(0.5,1.5), W ~ N(0, 1/K) (variance), in that order."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K), dtype=np.float32)
    g = rng.uniform(0.5, 1.5, K).astype(np.float32)
    W = rng.standard_normal((K, N), dtype=np.float32)
    W *= np.float32(K ** -0.5)
    if outlier_frac > 0.0:
        n_out = max(1, int(round(outlier_frac * M)))
        outlier_rows = np.sort(rng.choice(M, size=n_out, replace=False))
        X[outlier_rows] *= np.float32(20.0)
    else:
        outlier_rows = np.zeros(0, dtype=np.int64)
    if n_check_rows is None or n_check_rows >= M:
        check_rows = np.arange(M, dtype=np.int64)
    else:
        # stratified: the same number of rows from each consecutive 256-row block
        blocks = max(1, M // 256)
        per = max(1, n_check_rows // blocks)
        rows = []
        for b in range(blocks):
            lo = b * (M // blocks)
            hi = (b + 1) * (M // blocks) if b < blocks - 1 else M
            rows.append(lo + rng.choice(hi - lo, size=min(per, hi - lo), replace=False))
        check_rows = np.sort(np.concatenate(rows)).astype(np.int64)
    return Workload(name, M, K, N, dtype, float(np.float32(eps)),
                    to_storage(X, dtype), to_storage(g, dtype), to_storage(W, dtype),
                    check_rows, outlier_rows.astype(np.int64))


def config(name_or_index) -> Workload:
    """One of the five benchmark configurations, by name or index."""
    if isinstance(name_or_index, str):
        idx = CONFIG_NAMES.index(name_or_index)
    else:
        idx = int(name_or_index)
    name, M, K, N, dtype, eps, frac, nrows = _CONFIGS[idx]
    return make(M, K, N, dtype, eps, SEED + idx, name=name,
                outlier_frac=frac, n_check_rows=nrows)


def config_shape(name_or_index):
    """(name, M, K, N, dtype, eps) without drawing anything."""
    idx = CONFIG_NAMES.index(name_or_index) if isinstance(name_or_index, str) else int(name_or_index)
    return _CONFIGS[idx][:6]


def make_attention(B: int, H: int, S: int, D: int, dtype: str, seed: int):
    """Inputs of the QKNorm-before-attention workload, one query per (sample, head): Q [B, H, D],
    K and V [B, H, S, D] (a key-value cache of S positions), LayerNorm gains ~ U(0.5, 1.5) and
    biases ~ N(0, 0.1) of length D for queries and keys.  Keys and queries get a per-vector offset
    and scale (N(0, 1) and U(0.5, 2)), so that the normalisation has something to remove.
    Returns a dict of storage-typed arrays; draws in the order Q, K, V, gq, bq, gk, bk."""
    rng = np.random.default_rng(seed)
    def vectors(*shape):
        v = rng.standard_normal(shape + (D,), dtype=np.float32)
        v *= rng.uniform(0.5, 2.0, shape + (1,)).astype(np.float32)
        v += rng.standard_normal(shape + (1,), dtype=np.float32)
        return v
    Q = vectors(B, H)
    K = vectors(B, H, S)
    V = rng.standard_normal((B, H, S, D), dtype=np.float32)
    gq = rng.uniform(0.5, 1.5, D).astype(np.float32)
    bq = (rng.standard_normal(D, dtype=np.float32) * np.float32(0.1))
    gk = rng.uniform(0.5, 1.5, D).astype(np.float32)
    bk = (rng.standard_normal(D, dtype=np.float32) * np.float32(0.1))
    arrays = dict(Q=Q, K=K, V=V, gq=gq, bq=bq, gk=gk, bk=bk)
    return {k: to_storage(v, dtype) for k, v in arrays.items()}

