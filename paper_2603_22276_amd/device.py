"""Device-side plumbing shared by the benchmark, the smoke entry and the GPU tests: move stored host
arrays into HBM, allocate outputs and workspaces, and call the C ABI for one resident module.

Nothing of the method is computed here: torch tensors only own device memory, and every step of the
path runs inside libdora through `binding`.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as D
from . import inputs as I

DEV = "cuda:0"


def dtype_code(dtype: str) -> int:
    return {"f32": D.DORA_F32, "bf16": D.DORA_BF16, "f16": D.DORA_F16}[dtype]


def torch_dtype(dtype: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]


def to_dev(a: np.ndarray) -> torch.Tensor:
    """Stored array (float32, or uint16 bf16 bits) -> device tensor of the matching torch dtype."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def empty(shape, dtype: str) -> torch.Tensor:
    # filled with NaN so that an element the kernels forget to write fails any comparison
    return torch.full(tuple(shape), float("nan"), dtype=torch_dtype(dtype), device=DEV)


def empty_f32(*shape) -> torch.Tensor:
    return torch.full(tuple(shape), float("nan"), dtype=torch.float32, device=DEV)


def workspace(desc, phase) -> torch.Tensor:
    n = D.dora_workspace_bytes(desc, phase)
    assert n > 0
    return torch.empty(n, dtype=torch.uint8, device=DEV)


def desc_of(cfg: I.DoraConfig, tokens=None):
    return D.make_desc(cfg.d_out, cfg.d_in, cfg.r, cfg.tokens if tokens is None else tokens, dtype_code(cfg.dtype),
                       float(cfg.s), 0.0)


def rel_max(a: np.ndarray, ref: np.ndarray) -> float:
    """max |a - ref| / max |ref|"""
    d = float(np.max(np.abs(ref))) if ref.size else 0.0
    if a.size == 0:
        return 0.0
    e = float(np.max(np.abs(a - ref)))
    if not np.isfinite(e):
        return float("inf")
    return e / d if d > 0 else e


def rel_fro(a: np.ndarray, ref: np.ndarray) -> float:
    """||a - ref||_F / ||ref||_F"""
    if a.size == 0:
        return 0.0
    d = float(np.linalg.norm(ref.ravel()))
    e = float(np.linalg.norm((a - ref).ravel()))
    if not np.isfinite(e):
        return float("inf")
    return e / d if d > 0 else e


class Module:
    """One DoRA module resident on the device (inputs of make_inputs uploaded once)."""

    def __init__(self, cfg: I.DoraConfig, inp=None):
        self.cfg = cfg
        self.inp = I.make_inputs(cfg) if inp is None else inp
        self.desc = desc_of(cfg)
        for k in ("W", "A", "B", "m", "x", "dy"):
            if k in self.inp:
                setattr(self, k, to_dev(self.inp[k]))

    def f64(self, key):
        return I.to_f64(self.inp[key])

    def norm(self):
        c = empty_f32(self.cfg.d_out)
        D.dora_norm(self.desc, self.W, self.A, self.B, c, workspace(self.desc, D.PHASE_NORM))
        return c

    def forward(self, w_norm=None, save=True, fused=False, bias=None):
        cfg = self.cfg
        y = empty((cfg.tokens, cfg.d_out), cfg.dtype)
        h = empty((cfg.tokens, cfg.r), cfg.dtype) if save else None
        inner = empty((cfg.tokens, cfg.d_out), cfg.dtype) if save else None
        c = empty_f32(cfg.d_out)
        fn = D.dora_forward_fused if fused else D.dora_forward
        fn(self.desc, self.x, self.W, self.A, self.B, self.m, w_norm, bias, y, h, inner, c,
           workspace(self.desc, D.PHASE_FORWARD))
        return {"y": y, "h": h, "inner": inner, "c": c}

    def backward(self, w_norm=None, h=None, inner=None, want_dm=True):
        cfg = self.cfg
        dx = empty((cfg.tokens, cfg.d_in), cfg.dtype)
        dA = empty_f32(cfg.r, cfg.d_in)
        dB = empty_f32(cfg.d_out, cfg.r)
        dm = empty_f32(cfg.d_out) if want_dm else None
        D.dora_backward(self.desc, self.dy, self.x, self.W, self.A, self.B, self.m, w_norm, h, inner, dx, dA, dB, dm,
                        workspace(self.desc, D.PHASE_BACKWARD_RECOMPUTE))
        return {"dx": dx, "dA": dA, "dB": dB, "dm": dm}
