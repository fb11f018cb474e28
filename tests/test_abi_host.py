"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, sizes workspaces sensibly and rejects bad arguments before anything is enqueued."""
import ctypes
import os
import re

import pytest

from paper_2603_22276_amd import binding as D

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # a 256-byte aligned, never dereferenced "device pointer"


def header_functions():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dora_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(D.LIB_PATH)
    names = header_functions()
    assert "dora_norm" in names and "dora_forward" in names and "dora_backward" in names
    for n in names:
        assert hasattr(lib, n), n
    assert set(D.EXPORTS) == set(names)


def test_status_strings():
    assert D.status_str(0) == "ok"
    assert len({D.status_str(i) for i in range(7)}) == 7


def desc(**kw):
    base = dict(d_out=256, d_in=512, r=16, tokens=64, dtype=D.DORA_BF16, s=4.0)
    base.update(kw)
    return D.make_desc(**base)


def test_workspace_sizes():
    d = desc(d_out=8192, d_in=8192, r=384, tokens=8192, s=1.633)
    norm = D.dora_workspace_bytes(d, D.PHASE_NORM)
    # the norm needs O(d_out + r^2) scratch: far below one dense [d_out, d_in] bf16 temporary (128 MiB)
    assert 0 < norm < 16 * 2 ** 20
    fwd = D.dora_workspace_bytes(d, D.PHASE_FORWARD)
    bwd = D.dora_workspace_bytes(d, D.PHASE_BACKWARD)
    rec = D.dora_workspace_bytes(d, D.PHASE_BACKWARD_RECOMPUTE)
    act = 8192 * 8192 * 2
    assert norm + act <= fwd < norm + act + 32 * 2 ** 20
    assert act <= bwd < act + 32 * 2 ** 20
    assert bwd + act <= rec < 2 * act + 64 * 2 ** 20
    assert all(v % 256 == 0 for v in (norm, fwd, bwd, rec))
    assert D.dora_workspace_bytes(desc(d_out=250), D.PHASE_NORM) == 0       # not a multiple of 8
    assert D.dora_workspace_bytes(desc(dtype=7), D.PHASE_NORM) == 0
    assert D.dora_workspace_bytes(d, 99) == 0
    # a valid desc never sizes to 0 (0 means "invalid desc"), not even with no tokens
    assert D.dora_workspace_bytes(desc(tokens=0), D.PHASE_COMPOSE_BACKWARD) == 256
    assert D.dora_workspace_bytes(desc(tokens=0), D.PHASE_BACKWARD) >= 256
    # millions of tokens on a narrow module: row slabs no longer ride on a 65535-limited grid axis
    assert D.dora_workspace_bytes(desc(d_out=64, tokens=4_000_000, d_in=8, r=8), D.PHASE_BACKWARD) > 0


def call(fn, *args):
    with pytest.raises(D.DoraError) as e:
        fn(*args)
    return e.value.status


def test_argument_errors_are_reported_before_any_launch():
    d = desc()
    big = 1 << 30
    L = D.lib()
    ws_n = D.dora_workspace_bytes(d, D.PHASE_NORM)
    st = lambda: None
    # NULL pointers
    assert L.dora_norm(ctypes.byref(d), None, FAKE, FAKE, FAKE, FAKE, big, None) == 1
    assert L.dora_norm(None, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == 1
    # misaligned tensor / workspace
    assert L.dora_norm(ctypes.byref(d), FAKE + 2, FAKE, FAKE, FAKE, FAKE, big, None) == 3
    assert L.dora_norm(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE + 16, big, None) == 3
    # workspace too small / missing
    assert L.dora_norm(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, ws_n - 1, None) == 5
    assert L.dora_norm(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, None, 0, None) == 1
    # shapes and dtype
    for bad in (desc(d_out=0), desc(d_out=12), desc(d_in=100), desc(r=4), desc(tokens=-1),
                desc(d_out=1 << 20, d_in=1 << 20), desc(s=float("nan"))):
        assert L.dora_norm(ctypes.byref(bad), FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == 2
    assert L.dora_norm(ctypes.byref(desc(dtype=3)), FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == 4
    # forward / backward / compose reject the same way
    assert L.dora_forward(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, None, None, None, FAKE, None, None, None, FAKE, big, None) == 1
    assert L.dora_forward(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, None, None, None, FAKE, 1024, None) == 5
    assert L.dora_forward(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE + 2, FAKE, None, None, None, FAKE, big, None) == 3
    assert L.dora_backward(ctypes.byref(d), None, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None, FAKE, FAKE, FAKE,
                           FAKE, FAKE, big, None) == 1
    assert L.dora_compose(ctypes.byref(d), FAKE, FAKE, None, None, FAKE, 0, None, None) == 1
    assert L.dora_compose_backward(ctypes.byref(d), FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == 1
    assert L.dora_mag_scale(ctypes.byref(d), FAKE, FAKE, None, None, None) == 1
    assert L.dora_project(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, None) == 1
    # cached base term
    assert L.dora_base_sq(ctypes.byref(d), None, FAKE, None) == 1
    assert L.dora_base_sq(ctypes.byref(d), FAKE, FAKE + 2, None) == 3
    assert L.dora_base_sq(ctypes.byref(desc(d_in=100)), FAKE, FAKE, None) == 2
    assert L.dora_norm_cached(ctypes.byref(d), None, FAKE, FAKE, FAKE, FAKE, FAKE, big, None) == 1
    assert L.dora_norm_cached(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ws_n - 1, None) == 5


def test_binding_refuses_host_tensors():
    import torch
    t = torch.zeros(8)
    with pytest.raises(ValueError):
        D.dora_mag_scale(desc(), t, t, t, t, stream=0)
