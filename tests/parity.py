"""Shared helpers for the GPU parity tests: error metrics and oracle sub-sampling."""
from __future__ import annotations

import numpy as np

from paper_2505_22179_amd import inputs as I

MAX_ABS = 1e-2      # stated bound on |y_gpu - y_oracle|
REL_FRO = 1e-3      # stated bound on ||y_gpu - y_oracle||_F / ||y_oracle||_F


def fp16_ulp(y: np.ndarray) -> np.ndarray:
    """spacing of fp16 at |y| (normal range)"""
    a = np.maximum(np.abs(y.astype(np.float64)), 2.0 ** -14)
    return 2.0 ** (np.floor(np.log2(a)) - 10)


def check_gemm(y_gpu16: np.ndarray, y32: np.ndarray, what: str = "") -> dict:
    """y_gpu16: fp16 from the GPU; y32: the oracle's fp32 result (before its own fp16 rounding).
    An element passes if |err| <= max(1e-2, 0.5 ulp_fp16(y32) + 1e-3): a correctly rounded fp16
    result can miss 1e-2 by rounding alone once |y| >= 32, where half an ulp is 0.0156."""
    g = y_gpu16.astype(np.float64)
    ref = y32.astype(np.float64)
    err = np.abs(g - ref)
    bound = np.maximum(MAX_ABS, 0.5 * fp16_ulp(y32) + 1e-3)
    rel = float(np.linalg.norm(g - ref) / max(np.linalg.norm(ref), 1e-30))
    stats = {"max_abs": float(err.max()), "rel_fro": rel,
             "max_err_in_ulps": float((err / fp16_ulp(y32)).max()), "n_over_1e-2": int((err > MAX_ABS).sum())}
    assert (err <= bound).all(), f"{what}: max abs error {err.max():.4g} (stats {stats})"
    assert rel <= REL_FRO, f"{what}: relative Frobenius error {rel:.3g}"
    return stats


def column_subproblem(inp: I.LinearInputs, cols: np.ndarray):
    """Canonical tensors of the same layer restricted to the given columns (count a multiple of 8)."""
    assert len(cols) % 8 == 0
    return (I.pack_rows(np.ascontiguousarray(inp.codes[:, cols])),
            np.ascontiguousarray(inp.scales[:, cols]),
            I.pack_cols(np.ascontiguousarray(inp.zeros[:, cols])))
