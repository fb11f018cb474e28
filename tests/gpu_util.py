"""Helpers for the GPU parity tests: the device plumbing of the package plus the tolerances and the
assertions the parity bar is stated in."""
from __future__ import annotations

import numpy as np

from paper_2603_22276_amd.device import (DEV, Module, desc_of, dtype_code, empty, empty_f32, rel_fro, rel_max,  # noqa: F401
                                          to_dev, to_f64, workspace)

# Tolerances (relative): norm <= 1e-3 and tensors <= 2e-2 for bf16 storage with fp32 accumulation,
# 1e-5 for the fp32 configuration.
TOL = {"bf16": {"norm": 1e-3, "tensor": 2e-2}, "f32": {"norm": 1e-5, "tensor": 1e-5}}


def assert_close(name: str, a: np.ndarray, ref: np.ndarray, tol: float) -> None:
    assert a.shape == ref.shape, (name, a.shape, ref.shape)
    assert np.all(np.isfinite(a)), f"{name}: non-finite values in the GPU result"
    em, ef = rel_max(a, ref), rel_fro(a, ref)
    assert em <= tol and ef <= tol, f"{name}: rel_max={em:.3e} rel_fro={ef:.3e} tol={tol:.1e}"


def assert_norm_close(c: np.ndarray, ref: np.ndarray, tol: float) -> None:
    assert np.all(np.isfinite(c))
    e = float(np.max(np.abs(c - ref) / ref))
    assert e <= tol, f"norm: max rel err {e:.3e} > {tol:.1e}"
