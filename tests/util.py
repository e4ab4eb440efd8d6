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
