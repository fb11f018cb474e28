"""Compile oracle/literal.c into oracle/liboracle_literal.so with gcc (test infrastructure only)."""
from __future__ import annotations

import ctypes
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "literal.c")
LIB = os.path.join(HERE, "liboracle_literal.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-o", LIB, SRC, "-lm"])
    return LIB


def load() -> ctypes.CDLL:
    lib = ctypes.CDLL(build())
    dp = ctypes.POINTER(ctypes.c_double)
    L, D = ctypes.c_long, ctypes.c_double
    lib.lit_row_norm.argtypes = [dp, dp, dp, D, L, L, L, dp]
    lib.lit_forward_via_adapted_weight.argtypes = [dp, dp, dp, dp, dp, D, D, L, L, L, L, dp]
    lib.lit_forward_compose.argtypes = [dp, dp, dp, dp, dp, D, D, L, L, L, L, dp, dp]
    lib.lit_backward.argtypes = [dp] * 6 + [D, D, L, L, L, L] + [dp] * 4
    for f in (lib.lit_row_norm, lib.lit_forward_via_adapted_weight, lib.lit_forward_compose, lib.lit_backward):
        f.restype = None
    return lib


if __name__ == "__main__":
    print(build(force=True))
