"""Helpers shared by the GPU parity tests: upload, download, and the comparison rule."""
from __future__ import annotations

import numpy as np

import workloads

TOL = {"f16": 2e-2, "bf16": 2e-2, "f32": 1e-5}


def to_device(a: np.ndarray, dtype: str):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == "bf16":
        t = t.view(torch.bfloat16)
    return t.cuda()


def to_host_f64(t, dtype: str) -> np.ndarray:
    """Exact widening of a device result to float64."""
    import torch
    if dtype == "bf16":
        bits = t.contiguous().view(torch.uint16).cpu().numpy()
        return workloads.bf16_bits_to_f32(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def upload(w: workloads.Workload):
    return to_device(w.X, w.dtype), to_device(w.g, w.dtype), to_device(w.W, w.dtype)


def compare(Y_gpu: np.ndarray, Z_oracle: np.ndarray, dtype: str, what: str = ""):
    """max |err| <= tol * rms(Y), per row and over all checked rows.  Returns (max_err / rms, rms)."""
    tol = TOL[dtype]
    assert Y_gpu.shape == Z_oracle.shape, (what, Y_gpu.shape, Z_oracle.shape)
    nan_o, nan_g = np.isnan(Z_oracle), np.isnan(Y_gpu)
    assert np.array_equal(nan_o, nan_g), f"{what}: NaN positions differ"
    ok_rows = ~nan_o.any(axis=1)
    Zo, Yg = Z_oracle[ok_rows], Y_gpu[ok_rows]
    if Zo.size == 0:
        return 0.0, 0.0
    err = np.abs(Yg - Zo)
    row_rms = np.sqrt((Zo ** 2).mean(axis=1))
    glob_rms = float(np.sqrt((Zo ** 2).mean()))
    tiny = np.finfo(np.float64).tiny
    row_ratio = err.max(axis=1) / np.maximum(row_rms, tiny)
    worst_row = int(np.argmax(row_ratio))
    assert row_ratio[worst_row] <= tol, (
        f"{what}: row {worst_row} max|err|/rms(row) = {row_ratio[worst_row]:.3e} > {tol}")
    g_ratio = float(err.max() / max(glob_rms, tiny))
    assert g_ratio <= tol, f"{what}: max|err|/rms(Y) = {g_ratio:.3e} > {tol}"
    return g_ratio, glob_rms


def compare_gated(Y_gpu: np.ndarray, Z_oracle: np.ndarray, dtype: str, what: str = ""):
    """Bar for the gated block Y = SiLU(G) * U with [G | U] = Z, the plain block's fp64 output.

    The plain block is allowed |dG|, |dU| <= tol * rms(Z).  Propagated through the gate
    (|SiLU'| <= 1.1) and followed by one rounding to the storage type (2^-8 |Y| covers bf16's
    2^-9 with margin; fp32: 1e-6):
        |err| <= tol * rms(Z) * (1.1 |U| + |SiLU(G)|) + r |Y|
    checked elementwise; NaN positions must agree.  Returns the largest err / bound.
    """
    tol = TOL[dtype]
    r = 1e-6 if dtype == "f32" else 2.0 ** -8
    H = Z_oracle.shape[1] // 2
    assert Y_gpu.shape == (Z_oracle.shape[0], H), (what, Y_gpu.shape, Z_oracle.shape)
    import oracle
    G, U = Z_oracle[:, :H], Z_oracle[:, H:]
    with np.errstate(all="ignore"):
        Y = oracle.silu_mul_f64(Z_oracle)                                   # SiLU(G) * U
        S = oracle.silu_mul_f64(np.concatenate([G, np.ones_like(G)], 1))    # SiLU(G)
    nan_o, nan_g = np.isnan(Y), np.isnan(Y_gpu)
    assert np.array_equal(nan_o, nan_g), f"{what}: NaN positions differ"
    ok = ~nan_o
    if not ok.any():
        return 0.0
    rmsZ = float(np.sqrt(np.nanmean(np.where(np.isnan(Z_oracle), np.nan, Z_oracle) ** 2)))
    bound = tol * rmsZ * (1.1 * np.abs(U) + np.abs(S)) + r * np.abs(Y) + np.finfo(np.float64).tiny
    ratio = np.abs(Y_gpu - Y)[ok] / bound[ok]
    worst = float(ratio.max())
    assert worst <= 1.0, f"{what}: |err| / bound = {worst:.3f} > 1 (tol {tol})"
    return worst
