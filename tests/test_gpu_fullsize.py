"""GPU parity at the full sizes of the stated workloads, in the launch configuration bench.py times.

The oracle cannot afford every output of a [8192, 8192] x [8192, 8192] module in fp64 inside a test, so:
  * the norm is checked on every row (the dense W + sBA is formed once);
  * y, inner, h and dx are checked on sampled token rows (tokens are independent of one another);
  * dm and dB are checked on sampled output rows (a DoRA module restricted to a subset of its output rows
    is itself a DoRA module, so the oracle is simply run on that sub-module over all tokens);
  * dA, which sums over every token and every output row, is checked in full (it needs only skinny products).
Sampled indices always include the first and last index and both sides of a tile boundary.
"""
import numpy as np
import pytest
import torch

from oracle import dora_oracle as O
from paper_2603_22276_amd import inputs as I

import gpu_util as G

pytestmark = pytest.mark.gpu


def sample(n, count, seed):
    rng = np.random.default_rng(seed)
    fixed = [i for i in (0, 1, 127, 128, 255, 256, 257, n - 2, n - 1) if 0 <= i < n]
    extra = rng.choice(n, size=min(count, n), replace=False).tolist()
    return np.array(sorted(set(fixed + extra)), dtype=np.int64)


def pick(t, idx):
    return G.to_f64(t[torch.from_numpy(idx).to(t.device)])


# Regression bounds on top of the 2e-2 ceiling: about three times the error this path achieves on these
# workloads (fp32 outputs of fp32-accumulated bf16 products, and the delta of the compose), so that a tenfold
# loss of accuracy fails even though it would still sit below the ceiling.
TIGHT = {"dA": 7e-3, "dB": 7e-3, "dm": 1e-2, "delta": 1.5e-2}


def check_delta_sampled(mod, f, rows, c_dev):
    """Delta Y = (g-1) base + g s lora at full size: the three contractions as dora_forward launches them
    (dora_project), Eq. 6 and the compose pass in delta mode on the library's own base / lora / g / g-1,
    in the slab configuration of the full-size launch; sampled token rows against the oracle."""
    from paper_2603_22276_amd import binding as D
    cfg = mod.cfg
    base = G.empty((cfg.tokens, cfg.d_out), cfg.dtype)
    lora = G.empty((cfg.tokens, cfg.d_out), cfg.dtype)
    h = G.empty((cfg.tokens, cfg.r), cfg.dtype)
    D.dora_project(mod.desc, mod.x, mod.W, mod.A, mod.B, base, h, lora)
    g, gm1 = G.empty_f32(cfg.d_out), G.empty_f32(cfg.d_out)
    D.dora_mag_scale(mod.desc, mod.m, c_dev, g, gm1)
    delta = G.empty((cfg.tokens, cfg.d_out), cfg.dtype)
    D.dora_compose(mod.desc, base, lora, g, gm1, delta, 1, None)
    torch.cuda.synchronize()
    G.assert_close("base[rows]", pick(base, rows), f["base"], G.TOL[cfg.dtype]["tensor"])
    G.assert_close("lora[rows]", pick(lora, rows), f["lora"], G.TOL[cfg.dtype]["tensor"])
    G.assert_close("delta[rows]", pick(delta, rows), f["delta"], TIGHT["delta"])


def check_module_sampled(cfg, recompute, n_tok=40, n_out=40, full_dA=True, delta=False):
    G.CONTEXT[0] = cfg.name + ("/recompute" if recompute else "/saved")
    mod = G.Module(cfg)
    tol = G.TOL[cfg.dtype]
    W, A, B = mod.f64("W"), mod.f64("A"), mod.f64("B")
    m, s, eps = mod.inp["m"].astype(np.float64), float(mod.inp["s"]), cfg.eps

    c_ref = O.dense_row_norm(W, A, B, s)
    out = mod.forward(save=not recompute)
    G.assert_norm_close(G.to_f64(out["c"]), c_ref, tol["norm"])

    rows = sample(cfg.tokens, n_tok, 1)
    x_rows = I.to_f64(mod.inp["x"][rows])
    f = O.forward(x_rows, W, A, B, m, s, eps, c=c_ref)
    G.assert_close("y[rows]", pick(out["y"], rows), f["y"], tol["tensor"])
    if not recompute:
        G.assert_close("inner[rows]", pick(out["inner"], rows), f["inner"], tol["tensor"])
        G.assert_close("h[rows]", pick(out["h"], rows), f["h"], tol["tensor"])
    if delta:
        check_delta_sampled(mod, f, rows, out["c"])

    if recompute:
        grads = mod.backward()  # norm, h and inner recomputed inside (gradient-checkpointing pattern)
    else:
        grads = mod.backward(w_norm=out["c"], h=out["h"], inner=out["inner"])

    dy_rows = I.to_f64(mod.inp["dy"][rows])
    dx_ref = O.grad_x(dy_rows, x_rows, W, A, B, m, s, eps, c=c_ref)
    G.assert_close("dx[rows]", pick(grads["dx"], rows), dx_ref, tol["tensor"])

    cols = sample(cfg.d_out, n_out, 2)
    x_all = mod.f64("x")
    dy_cols = I.to_f64(np.ascontiguousarray(mod.inp["dy"][:, cols]))
    sub = dict(x=x_all, W=W[cols], A=A, B=B[cols], m=m[cols], s=s, eps=eps, c=c_ref[cols])
    G.assert_close("dm[cols]", pick(grads["dm"], cols), O.grad_m(dy_cols, **sub), TIGHT["dm"])
    G.assert_close("dB[cols]", pick(grads["dB"], cols), O.grad_B(dy_cols, **sub), TIGHT["dB"])
    del dy_cols, sub

    if full_dA:
        dA_ref = O.grad_A(mod.f64("dy"), x_all, W, A, B, m, s, eps, c=c_ref)
        G.assert_close("dA", G.to_f64(grads["dA"]), dA_ref, TIGHT["dA"])
    G.CONTEXT[0] = ""


def test_c2_forward_every_element():
    # d_out = d_in = 4096, r = 384, tokens = 4096: norm + forward, every element
    for cfg in (I.C2, I.stress(I.C2)):
        G.CONTEXT[0] = cfg.name
        mod = G.Module(cfg)
        oi = dict(x=mod.f64("x"), W=mod.f64("W"), A=mod.f64("A"), B=mod.f64("B"),
                  m=mod.inp["m"].astype(np.float64), s=float(mod.inp["s"]), eps=cfg.eps)
        f = O.forward(**oi)
        out = mod.forward()
        G.assert_norm_close(G.to_f64(out["c"]), f["c"], G.TOL["bf16"]["norm"])
        G.assert_close("y", G.to_f64(out["y"]), f["y"], G.TOL["bf16"]["tensor"])
        G.assert_close("inner", G.to_f64(out["inner"]), f["inner"], G.TOL["bf16"]["tensor"])
        # Delta Y through the compose pass in delta mode, every element
        y_minus = G.empty((cfg.tokens, cfg.d_out), cfg.dtype)
        from paper_2603_22276_amd import binding as D
        base, lora, h = (G.empty((cfg.tokens, n), cfg.dtype) for n in (cfg.d_out, cfg.d_out, cfg.r))
        D.dora_project(mod.desc, mod.x, mod.W, mod.A, mod.B, base, h, lora)
        g, gm1 = G.empty_f32(cfg.d_out), G.empty_f32(cfg.d_out)
        D.dora_mag_scale(mod.desc, mod.m, out["c"], g, gm1)
        D.dora_compose(mod.desc, base, lora, g, gm1, y_minus, 1, None)
        G.assert_close("delta", G.to_f64(y_minus), f["delta"], TIGHT["delta"])
        del f, out, mod, base, lora, h, y_minus
    G.CONTEXT[0] = ""


def test_c3_headline_forward_backward_sampled():
    # the configuration bench.py times: forward saving h / inner / w_norm, backward from the saved tensors
    check_module_sampled(I.C3, recompute=False, delta=True)


def test_c3_stress_norm_and_recompute_sampled():
    check_module_sampled(I.stress(I.C3), recompute=True, full_dA=False)


@pytest.mark.parametrize("cfg", [I.C4_UP, I.C4_DOWN], ids=["up", "down"])
def test_c4_mlp_pair_recompute_sampled(cfg):
    # 32B-class MLP shapes, 8192 tokens, norm recomputed in backward
    check_module_sampled(cfg, recompute=True, n_tok=24, n_out=24, delta=(cfg is I.C4_UP))


@pytest.mark.parametrize("module_index,r", [(1, 64), (1, 768), (4, 384), (6, 768), (0, 64), (4, 64), (4, 768), (6, 64)],
                         ids=["k_r64", "k_r768", "gate_r384", "down_r768", "q_r64", "gate_r64", "gate_r768", "down_r64"])
def test_c5_decoder_modules_recompute_sampled(module_index, r):
    cfg = I.c5_module(module_index, r)
    check_module_sampled(cfg, recompute=True, n_tok=24, n_out=24)


@pytest.mark.parametrize("d_out,d_in,r", [(8192, 28672, 384), (4096, 11008, 384), (8192, 8192, 768), (4096, 4096, 16)],
                         ids=["moe_8192x28672_r384", "4096x11008_r384", "8192x8192_r768", "4096x4096_r16"])
def test_norm_at_the_rank_sweep_shapes_sampled_rows(d_out, d_in, r):
    # shapes of Table 5; rows of the norm are independent, so the dense definition is evaluated on sampled rows
    for cfg in (I.DoraConfig("sweep", d_out, d_in, r, 8, "bf16", 32.0, 1e-3, seed_offset=9100 + r),
                I.stress(I.DoraConfig("sweep_stress", d_out, d_in, r, 8, "bf16", 32.0, 1e-3, seed_offset=9200 + r))):
        mod = G.Module(cfg)
        rows = sample(d_out, 96, 3)
        A = mod.f64("A")
        Wr = I.to_f64(mod.inp["W"][rows])
        Br = I.to_f64(mod.inp["B"][rows])
        ref = O.dense_row_norm(Wr, A, Br, float(mod.inp["s"]))
        G.assert_norm_close(pick(mod.norm(), rows), ref, G.TOL["bf16"]["norm"])
        base_sq = G.empty_f32(d_out)
        c = G.empty_f32(d_out)
        from paper_2603_22276_amd import binding as D
        D.dora_base_sq(mod.desc, mod.W, base_sq)
        D.dora_norm_cached(mod.desc, base_sq, mod.W, mod.A, mod.B, c, G.workspace(mod.desc, D.PHASE_NORM))
        G.assert_norm_close(pick(c, rows), ref, G.TOL["bf16"]["norm"])
        del mod
