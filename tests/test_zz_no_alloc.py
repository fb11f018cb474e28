"""The entry point that allocates nothing (dora_norm_static) against dora_norm: same kernels, scratch in
the library's fixed device array instead of a caller workspace.  Two calls in a row, the second on a
smaller shape, so that what the first left in the array is seen not to matter."""
import numpy as np
import pytest
import torch

import gpu_util as G
from oracle import dora_oracle as O
from paper_2603_22276_amd import binding as D
from paper_2603_22276_amd import inputs as I

pytestmark = pytest.mark.gpu

BIG = I.DoraConfig("static_big", 1160, 1096, 136, 0, "bf16", 32.0, 0.02, seed_offset=9100)
SMALL = I.DoraConfig("static_small", 264, 200, 24, 0, "bf16", 32.0, 0.05, seed_offset=9200)


def test_static_scratch_norm_matches_workspace_norm_twice_in_a_row():
    assert D.dora_norm_static_max_bytes() == 16 * 2 ** 20
    mods = [G.Module(c, I.make_inputs(c, with_dy=False)) for c in (BIG, SMALL)]
    got = [G.empty_f32(m.cfg.d_out) for m in mods]
    for mod, c in zip(mods, got):  # back to back on one stream: big shape first, then the smaller one
        D.dora_norm_static(mod.desc, mod.W, mod.A, mod.B, c)
    torch.cuda.synchronize()
    # no device memory is taken by further calls (the code object and the array are resident by now)
    free_before = torch.cuda.mem_get_info()[0]
    again = [G.empty_f32(m.cfg.d_out) for m in mods]
    reserved = torch.cuda.memory_reserved()
    for mod, c in zip(mods, again):
        D.dora_norm_static(mod.desc, mod.W, mod.A, mod.B, c)
    torch.cuda.synchronize()
    assert torch.cuda.memory_reserved() == reserved
    assert torch.cuda.mem_get_info()[0] >= free_before - (2 << 20)
    for a, b in zip(got, again):
        assert torch.equal(a, b)
    for mod, c in zip(mods, got):
        ref = mod.norm()  # dora_norm with a caller workspace
        torch.cuda.synchronize()
        assert torch.equal(c, ref), mod.cfg.name  # same launches, same order of sums: bit for bit
        dense = O.dense_row_norm(mod.f64("W"), mod.f64("A"), mod.f64("B"), float(mod.inp["s"]))
        G.assert_norm_close(G.to_f64(c), dense, G.TOL["bf16"]["norm"])


def test_static_scratch_rejects_shapes_beyond_its_size():
    d = D.make_desc(8192, 8192, 2048, 0, D.DORA_BF16, 1.0)
    assert D.dora_workspace_bytes(d, D.PHASE_NORM) > D.dora_norm_static_max_bytes()
    fake = 0x10000
    with pytest.raises(D.DoraError) as e:
        D.dora_norm_static(d, fake, fake, fake, fake)
    assert e.value.status == 5
