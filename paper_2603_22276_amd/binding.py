"""Thin ctypes binding of libdora.so: argument marshalling only.

Every function here has the name and argument order of the C entry point it calls
(include/dora.h).  Tensor arguments are torch CUDA tensors (used purely as owners of
device memory) or None; nothing is computed on the Python side.  If the shared library
has not been built the import of the library fails loudly - there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdora.so")

DORA_F32, DORA_BF16, DORA_F16 = 0, 1, 2
PHASE_NORM, PHASE_FORWARD, PHASE_BACKWARD, PHASE_BACKWARD_RECOMPUTE, PHASE_COMPOSE_BACKWARD, PHASE_FORWARD_DROPOUT, PHASE_BACKWARD_DROPOUT = range(7)
K_COUNT = 20

EXPORTS = (
    "dora_workspace_bytes", "dora_norm", "dora_norm_static", "dora_norm_static_max_bytes", "dora_base_sq", "dora_norm_cached", "dora_norm_terms", "dora_norm_assemble", "dora_mag_scale", "dora_compose", "dora_compose_backward",
    "dora_project", "dora_forward", "dora_forward_fused", "dora_backward", "dora_forward_dropout", "dora_backward_dropout", "dora_status_str",
    "dora_probe_copy", "dora_probe_mfma",
    "dora_trace_enable", "dora_trace_select", "dora_trace_reset", "dora_trace_collect", "dora_trace_get", "dora_trace_name",
)


class DoraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_str(status)})")


class dora_desc(ctypes.Structure):
    _fields_ = [
        ("d_out", ctypes.c_int64), ("d_in", ctypes.c_int64), ("r", ctypes.c_int64), ("tokens", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("s", ctypes.c_float), ("eps", ctypes.c_float),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2603_22276_amd.build). "
                "There is no CPU or PyTorch fallback for the DoRA hot path.")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, dp, fp = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(dora_desc), ctypes.c_void_p
        L.dora_workspace_bytes.argtypes = [dp, ctypes.c_int]
        L.dora_workspace_bytes.restype = sz
        L.dora_norm.argtypes = [dp, vp, vp, vp, fp, vp, sz, vp]
        L.dora_norm_static.argtypes = [dp, vp, vp, vp, fp, vp]
        L.dora_norm_static_max_bytes.argtypes = []
        L.dora_norm_static_max_bytes.restype = sz
        L.dora_base_sq.argtypes = [dp, vp, fp, vp]
        L.dora_norm_cached.argtypes = [dp, fp, vp, vp, vp, fp, vp, sz, vp]
        L.dora_norm_terms.argtypes = [dp, vp, vp, vp, fp, fp, vp, sz, vp]
        L.dora_norm_assemble.argtypes = [dp, fp, fp, vp]
        L.dora_mag_scale.argtypes = [dp, fp, fp, fp, fp, vp]
        L.dora_compose.argtypes = [dp, vp, vp, fp, fp, vp, ctypes.c_int, vp, vp]
        L.dora_compose_backward.argtypes = [dp, vp, vp, fp, fp, vp, fp, vp, sz, vp]
        L.dora_project.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.dora_forward.argtypes = [dp, vp, vp, vp, vp, fp, fp, vp, vp, vp, vp, fp, vp, sz, vp]
        L.dora_forward_fused.argtypes = L.dora_forward.argtypes
        L.dora_backward.argtypes = [dp, vp, vp, vp, vp, vp, fp, fp, vp, vp, vp, fp, fp, fp, vp, sz, vp]
        L.dora_forward_dropout.argtypes = [dp, vp, vp, vp, vp, vp, fp, fp, vp, vp, vp, vp, fp, vp, sz, vp]
        L.dora_backward_dropout.argtypes = [dp, vp, vp, vp, vp, vp, fp, fp, vp, vp, vp, vp, fp, fp, fp, vp, sz, vp]
        L.dora_probe_copy.argtypes = [vp, vp, sz, vp]
        L.dora_probe_mfma.argtypes = [vp, fp, ctypes.c_int, ctypes.c_int, vp]
        for f in (L.dora_probe_copy, L.dora_probe_mfma, L.dora_norm, L.dora_norm_static, L.dora_base_sq, L.dora_norm_cached, L.dora_norm_terms, L.dora_norm_assemble, L.dora_mag_scale, L.dora_compose, L.dora_compose_backward, L.dora_project, L.dora_forward, L.dora_forward_fused,
                  L.dora_backward, L.dora_forward_dropout, L.dora_backward_dropout, L.dora_trace_collect, L.dora_trace_get):
            f.restype = ctypes.c_int
        L.dora_status_str.argtypes = [ctypes.c_int]
        L.dora_status_str.restype = ctypes.c_char_p
        L.dora_trace_enable.argtypes = [ctypes.c_int]
        L.dora_trace_enable.restype = None
        L.dora_trace_select.argtypes = [ctypes.c_uint64]
        L.dora_trace_select.restype = None
        L.dora_trace_reset.argtypes = []
        L.dora_trace_reset.restype = None
        L.dora_trace_collect.argtypes = []
        L.dora_trace_get.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
        L.dora_trace_name.argtypes = [ctypes.c_int]
        L.dora_trace_name.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().dora_status_str(int(status)).decode()


def make_desc(d_out: int, d_in: int, r: int, tokens: int, dtype: int, s: float, eps: float = 0.0) -> dora_desc:
    return dora_desc(int(d_out), int(d_in), int(r), int(tokens), int(dtype), float(s), float(eps))


def _p(t) -> Optional[int]:
    """Device pointer of a torch tensor (or a raw integer address, or None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("libdora takes device pointers: pass CUDA tensors")
    if not t.is_contiguous():
        raise ValueError("libdora takes contiguous row-major tensors")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _nbytes(ws) -> int:
    return 0 if ws is None else ws.numel() * ws.element_size()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise DoraError(status, where)


def dora_workspace_bytes(desc: dora_desc, phase: int) -> int:
    return int(lib().dora_workspace_bytes(ctypes.byref(desc), int(phase)))


def dora_norm(desc, W, A, B, w_norm, ws, stream=None) -> None:
    _check(lib().dora_norm(ctypes.byref(desc), _p(W), _p(A), _p(B), _p(w_norm), _p(ws), _nbytes(ws), _stream(stream)),
           "dora_norm")


def dora_norm_static(desc, W, A, B, w_norm, stream=None) -> None:
    _check(lib().dora_norm_static(ctypes.byref(desc), _p(W), _p(A), _p(B), _p(w_norm), _stream(stream)), "dora_norm_static")


def dora_norm_static_max_bytes() -> int:
    return int(lib().dora_norm_static_max_bytes())


def dora_base_sq(desc, W, base_sq, stream=None) -> None:
    _check(lib().dora_base_sq(ctypes.byref(desc), _p(W), _p(base_sq), _stream(stream)), "dora_base_sq")


def dora_norm_cached(desc, base_sq, W, A, B, w_norm, ws, stream=None) -> None:
    _check(lib().dora_norm_cached(ctypes.byref(desc), _p(base_sq), _p(W), _p(A), _p(B), _p(w_norm), _p(ws), _nbytes(ws),
                                  _stream(stream)), "dora_norm_cached")


def dora_norm_terms(desc, W, A, B, terms, G, ws, stream=None) -> None:
    _check(lib().dora_norm_terms(ctypes.byref(desc), _p(W), _p(A), _p(B), _p(terms), _p(G), _p(ws), _nbytes(ws),
                                 _stream(stream)), "dora_norm_terms")


def dora_norm_assemble(desc, terms, w_norm, stream=None) -> None:
    _check(lib().dora_norm_assemble(ctypes.byref(desc), _p(terms), _p(w_norm), _stream(stream)), "dora_norm_assemble")


def dora_mag_scale(desc, m, w_norm, g, gm1, stream=None) -> None:
    _check(lib().dora_mag_scale(ctypes.byref(desc), _p(m), _p(w_norm), _p(g), _p(gm1), _stream(stream)), "dora_mag_scale")


def dora_compose(desc, base, lora, g, gm1, out, write_delta, inner, stream=None) -> None:
    _check(lib().dora_compose(ctypes.byref(desc), _p(base), _p(lora), _p(g), _p(gm1), _p(out), int(write_delta),
                              _p(inner), _stream(stream)), "dora_compose")


def dora_compose_backward(desc, dy, inner, g, w_norm, dz, dm, ws, stream=None) -> None:
    _check(lib().dora_compose_backward(ctypes.byref(desc), _p(dy), _p(inner), _p(g), _p(w_norm), _p(dz), _p(dm),
                                       _p(ws), _nbytes(ws), _stream(stream)), "dora_compose_backward")


def dora_project(desc, x, W, A, B, base, h, lora, stream=None) -> None:
    _check(lib().dora_project(ctypes.byref(desc), _p(x), _p(W), _p(A), _p(B), _p(base), _p(h), _p(lora),
                              _stream(stream)), "dora_project")


def dora_forward(desc, x, W, A, B, m, w_norm, bias, y, saved_h, saved_inner, w_norm_out, ws, stream=None) -> None:
    _check(lib().dora_forward(ctypes.byref(desc), _p(x), _p(W), _p(A), _p(B), _p(m), _p(w_norm), _p(bias), _p(y), _p(saved_h),
                              _p(saved_inner), _p(w_norm_out), _p(ws), _nbytes(ws), _stream(stream)), "dora_forward")


def dora_forward_fused(desc, x, W, A, B, m, w_norm, bias, y, saved_h, saved_inner, w_norm_out, ws, stream=None) -> None:
    _check(lib().dora_forward_fused(ctypes.byref(desc), _p(x), _p(W), _p(A), _p(B), _p(m), _p(w_norm), _p(bias), _p(y),
                                    _p(saved_h), _p(saved_inner), _p(w_norm_out), _p(ws), _nbytes(ws),
                                    _stream(stream)), "dora_forward_fused")


def dora_backward(desc, dy, x, W, A, B, m, w_norm, saved_h, saved_inner, dx, dA, dB, dm, ws, stream=None) -> None:
    _check(lib().dora_backward(ctypes.byref(desc), _p(dy), _p(x), _p(W), _p(A), _p(B), _p(m), _p(w_norm), _p(saved_h),
                               _p(saved_inner), _p(dx), _p(dA), _p(dB), _p(dm), _p(ws), _nbytes(ws), _stream(stream)),
           "dora_backward")


def dora_forward_dropout(desc, x, x_lora, W, A, B, m, w_norm, bias, y, saved_h, saved_inner, w_norm_out, ws, stream=None) -> None:
    _check(lib().dora_forward_dropout(ctypes.byref(desc), _p(x), _p(x_lora), _p(W), _p(A), _p(B), _p(m), _p(w_norm), _p(bias),
                                      _p(y), _p(saved_h), _p(saved_inner), _p(w_norm_out), _p(ws), _nbytes(ws),
                                      _stream(stream)), "dora_forward_dropout")


def dora_backward_dropout(desc, dy, x_lora, W, A, B, m, w_norm, saved_h, saved_inner, dx, dx_lora, dA, dB, dm, ws,
                          stream=None) -> None:
    _check(lib().dora_backward_dropout(ctypes.byref(desc), _p(dy), _p(x_lora), _p(W), _p(A), _p(B), _p(m), _p(w_norm),
                                       _p(saved_h), _p(saved_inner), _p(dx), _p(dx_lora), _p(dA), _p(dB), _p(dm), _p(ws),
                                       _nbytes(ws), _stream(stream)), "dora_backward_dropout")


def dora_probe_copy(src, dst, nbytes: int, stream=None) -> None:
    _check(lib().dora_probe_copy(_p(src), _p(dst), int(nbytes), _stream(stream)), "dora_probe_copy")


def dora_probe_mfma(operands, sink, iters: int, workgroups: int, stream=None) -> None:
    _check(lib().dora_probe_mfma(_p(operands), _p(sink), int(iters), int(workgroups), _stream(stream)), "dora_probe_mfma")


def dora_trace_enable(on: bool) -> None:
    lib().dora_trace_enable(1 if on else 0)


def dora_trace_select(kernel_mask: int) -> None:
    lib().dora_trace_select(int(kernel_mask) & 0xFFFFFFFFFFFFFFFF)


def dora_trace_reset() -> None:
    lib().dora_trace_reset()


def dora_trace_collect() -> None:
    _check(lib().dora_trace_collect(), "dora_trace_collect")


def dora_trace_get(kernel_id: int):
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(lib().dora_trace_get(int(kernel_id), ctypes.byref(ms), ctypes.byref(n)), "dora_trace_get")
    return ms.value, n.value


def dora_trace_name(kernel_id: int) -> str:
    return lib().dora_trace_name(int(kernel_id)).decode()
