"""Helpers for the GPU parity tests: the device plumbing of the package plus the tolerances and the
assertions the parity bar is stated in."""
from __future__ import annotations

import atexit
import json
import os

import numpy as np

from paper_2603_22276_amd.device import (DEV, Module, desc_of, dtype_code, empty, empty_f32, rel_fro, rel_max,  # noqa: F401
                                          to_dev, to_f64, workspace)

# Tolerances (relative): norm <= 1e-3 and tensors <= 2e-2 for bf16 storage with fp32 accumulation,
# 1e-5 for the fp32 configuration.  fp16 storage rounds to 11 significant bits against bf16's 8, so its
# tensors are held to a quarter of the bf16 bound.
TOL = {"bf16": {"norm": 1e-3, "tensor": 2e-2}, "f16": {"norm": 1e-3, "tensor": 5e-3}, "f32": {"norm": 1e-5, "tensor": 1e-5}}


# Achieved errors of the run, keyed by "<context>/<tensor>": written to $DORA_PARITY_LOG at exit when that
# variable is set (the achieved-error table of the design notes comes from such a run).
ACHIEVED = {}
CONTEXT = [""]


def _record(name, em, ef):
    key = f"{CONTEXT[0]}/{name}" if CONTEXT[0] else name
    ACHIEVED[key] = {"rel_max": em, "rel_fro": ef}


def _dump():
    path = os.environ.get("DORA_PARITY_LOG")
    if path and ACHIEVED:
        with open(path, "w") as f:
            json.dump(ACHIEVED, f, indent=1, sort_keys=True)


atexit.register(_dump)


def assert_close(name: str, a: np.ndarray, ref: np.ndarray, tol: float) -> None:
    assert a.shape == ref.shape, (name, a.shape, ref.shape)
    assert np.all(np.isfinite(a)), f"{name}: non-finite values in the GPU result"
    em, ef = rel_max(a, ref), rel_fro(a, ref)
    _record(name, em, ef)
    assert em <= tol and ef <= tol, f"{name}: rel_max={em:.3e} rel_fro={ef:.3e} tol={tol:.1e}"


def assert_norm_close(c: np.ndarray, ref: np.ndarray, tol: float) -> None:
    assert np.all(np.isfinite(c))
    e = float(np.max(np.abs(c - ref) / ref))
    _record("norm", e, e)
    assert e <= tol, f"norm: max rel err {e:.3e} > {tol:.1e}"
