"""Helpers shared by the GPU parity tests: tolerances and oracle-side references."""
from __future__ import annotations

import numpy as np

import oracle

TOL = {"f32": 1e-4, "bf16": 2e-2}


def assert_close(gpu: np.ndarray, ref: np.ndarray, scale: np.ndarray, tol: float, what: str):
    """Both must hold: (i) ||gpu - ref||_2 <= tol ||ref||_2;
    (ii) |gpu - ref| <= tol * max(|ref|, scale) element-wise, scale = the sum of |term| magnitudes of
    that element (the forward-error scale of a dot product)."""
    gpu = np.asarray(gpu, np.float64)
    err = np.abs(gpu - ref)
    nref = float(np.linalg.norm(ref))
    rel = float(np.linalg.norm(gpu - ref)) / nref if nref > 0 else float(np.linalg.norm(gpu))
    bound = tol * np.maximum(np.abs(ref), scale)
    worst = float((err - bound).max()) if err.size else -1.0
    assert rel <= tol, f"{what}: relative L2 error {rel:.3e} > {tol}"
    assert worst <= 0.0, (f"{what}: element-wise error exceeds tol*max(|ref|, scale) by {worst:.3e} "
                          f"(max err {float(err.max()):.3e})")
    return rel


def oracle_fwd(x, w, o, i, k, n_out):
    ref = oracle.mvmr_fwd(x, w, o, i, k, n_out)
    scale = oracle.mvmr_fwd(np.abs(x), np.abs(w), o, i, k, n_out)
    return ref, scale


def oracle_bwd_input(dy, w, o, i, k, n_in):
    ref = oracle.mvmr_bwd_input(dy, w, o, i, k, n_in)
    scale = oracle.mvmr_bwd_input(np.abs(dy), np.abs(w), o, i, k, n_in)
    return ref, scale


def oracle_bwd_weight(x, dy, o, i, k, K):
    ref = oracle.mvmr_bwd_weight(x, dy, o, i, k, K)
    scale = oracle.mvmr_bwd_weight(np.abs(x), np.abs(dy), o, i, k, K)
    return ref, scale
