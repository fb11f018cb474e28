"""GPU parity: every entry point of the C ABI against the fp64 CPU oracle, element by element,
on the same seeded inputs.  Sizes are chosen so the oracle finishes in seconds while the kernels still
cross several tiles and end in ragged tails."""
import numpy as np
import pytest
import torch

from oracle import dora_oracle as O
from paper_2603_22276_amd import binding as D
from paper_2603_22276_amd import inputs as I

import gpu_util as G

pytestmark = pytest.mark.gpu


def cfg_bf16(name, d_out, d_in, r, tokens, sigma_B=1e-3, seed=0):
    return I.DoraConfig(name, d_out, d_in, r, tokens, "bf16", 32.0, sigma_B, seed_offset=7000 + seed)


def cfg_f16(name, d_out, d_in, r, tokens, sigma_B=1e-3, seed=0):
    return I.DoraConfig(name, d_out, d_in, r, tokens, "f16", 32.0, sigma_B, seed_offset=7500 + seed)


def cfg_f32(name, d_out, d_in, r, tokens, sigma_B=1e-2, seed=0):
    return I.DoraConfig(name, d_out, d_in, r, tokens, "f32", 16.0, sigma_B, seed_offset=8000 + seed)


def mk_of(dtype):
    return {"bf16": cfg_bf16, "f16": cfg_f16, "f32": cfg_f32}[dtype]


SMALL = [
    I.C1,
    cfg_f32("f32_ragged", 100, 52, 12, 33, seed=1),
    cfg_bf16("bf16_ragged_tiny", 200, 328, 24, 77, seed=2),
    cfg_bf16("bf16_ragged", 520, 392, 40, 300, seed=3),
    I.stress(cfg_bf16("bf16_mid", 1024, 1536, 384, 640, seed=4)),
    cfg_bf16("bf16_mid", 1024, 1536, 384, 640, seed=4),
    cfg_bf16("bf16_bigtile_ragged", 4104, 264, 16, 4104, sigma_B=2e-2, seed=5),
    # dx = dz W + dh A on the 256 x 256 tile (K-strided N side) with ragged K in both segments and an odd number of K steps
    cfg_bf16("bf16_bigtile_dx_ragged", 264, 4104, 16, 4104, sigma_B=2e-2, seed=6),
    # few tiles and a long K: h = x A^T (first) and dh = s dz B (second) run split along K with a fixed-order reduce
    cfg_bf16("bf16_splitk_h", 264, 2312, 40, 300, seed=8),
    cfg_bf16("bf16_splitk_dh", 3080, 264, 24, 200, sigma_B=2e-2, seed=9),
    # fp16 storage (App. B): the same kernels with the fp16 MFMA and conversions
    cfg_f16("f16_ragged_tiny", 200, 328, 24, 77, seed=2),
    I.stress(cfg_f16("f16_mid", 1024, 1536, 384, 640, seed=4)),
    cfg_f16("f16_bigtile_ragged", 4104, 264, 16, 4104, sigma_B=2e-2, seed=5),
    cfg_f16("f16_splitk_h", 264, 2312, 40, 300, seed=8),
]
IDS = [c.name for c in SMALL]


def oracle_inputs(mod):
    return dict(x=mod.f64("x"), W=mod.f64("W"), A=mod.f64("A"), B=mod.f64("B"),
                m=mod.inp["m"].astype(np.float64), s=float(mod.inp["s"]), eps=mod.cfg.eps)


# ----------------------------------------------------------------------------- norm (a1-a6)

@pytest.mark.parametrize("cfg", SMALL, ids=IDS)
def test_norm_matches_dense_oracle(cfg):
    mod = G.Module(cfg)
    c = G.to_f64(mod.norm())
    ref = O.dense_row_norm(mod.f64("W"), mod.f64("A"), mod.f64("B"), float(mod.inp["s"]))
    G.assert_norm_close(c, ref, G.TOL[cfg.dtype]["norm"])


@pytest.mark.parametrize("cfg", SMALL, ids=IDS)
def test_cached_base_term_and_norm_from_it(cfg):
    # Sec. 2.3: the base term is rank independent and W is frozen, so it may be computed once and reused.
    # base_sq is a sum of exactly representable products in fp32: checked tightly against the fp64 sum;
    # the norm assembled from the cached term is held to the same bar as dora_norm, against the dense definition.
    mod = G.Module(cfg)
    W = mod.f64("W")
    base_sq = G.empty_f32(cfg.d_out)
    D.dora_base_sq(mod.desc, mod.W, base_sq)
    ref_sq = np.sum(W * W, axis=1)
    got_sq = G.to_f64(base_sq)
    assert np.all(np.isfinite(got_sq))
    assert np.max(np.abs(got_sq - ref_sq) / ref_sq) <= 1e-5
    c = G.empty_f32(cfg.d_out)
    D.dora_norm_cached(mod.desc, base_sq, mod.W, mod.A, mod.B, c, G.workspace(mod.desc, D.PHASE_NORM))
    ref = O.dense_row_norm(W, mod.f64("A"), mod.f64("B"), float(mod.inp["s"]))
    G.assert_norm_close(G.to_f64(c), ref, G.TOL[cfg.dtype]["norm"])
    # the cache is really what is used: a doubled base term must show up in the result
    base_sq2 = base_sq * 4.0
    D.dora_norm_cached(mod.desc, base_sq2, mod.W, mod.A, mod.B, c, G.workspace(mod.desc, D.PHASE_NORM))
    terms = O.factored_norm_terms(W, mod.f64("A"), mod.f64("B"))
    s = float(mod.inp["s"])
    ref2 = np.sqrt(np.maximum(4.0 * terms["base_sq"] + 2.0 * s * terms["cross"] + s * s * terms["ba_sq"], 0.0))
    G.assert_norm_close(G.to_f64(c), ref2, G.TOL[cfg.dtype]["norm"])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_cached_norm_with_zero_scale(dtype):
    mk = cfg_bf16 if dtype == "bf16" else cfg_f32
    cfg = mk("s0", 264, 328, 24, 8, seed=21)
    mod = G.Module(cfg)
    desc = D.make_desc(cfg.d_out, cfg.d_in, cfg.r, cfg.tokens, G.dtype_code(dtype), 0.0, 0.0)
    base_sq = G.empty_f32(cfg.d_out)
    D.dora_base_sq(desc, mod.W, base_sq)
    c = G.empty_f32(cfg.d_out)
    D.dora_norm_cached(desc, base_sq, mod.W, mod.A, mod.B, c, G.workspace(desc, D.PHASE_NORM))
    G.assert_norm_close(G.to_f64(c), np.linalg.norm(mod.f64("W"), axis=1), G.TOL[dtype]["norm"])


@pytest.mark.parametrize("cfg", SMALL, ids=IDS)
def test_norm_terms_and_their_assembly(cfg):
    # the factored terms one by one (Eq. 2-4) against their fp64 definitions, the Gram matrix, and
    # dora_norm == dora_norm_terms followed by dora_norm_assemble, bit for bit
    mod = G.Module(cfg)
    t64 = O.factored_norm_terms(mod.f64("W"), mod.f64("A"), mod.f64("B"))
    terms = G.empty_f32(3, cfg.d_out)
    Gm = G.empty_f32(cfg.r, cfg.r)
    D.dora_norm_terms(mod.desc, mod.W, mod.A, mod.B, terms, Gm, G.workspace(mod.desc, D.PHASE_NORM))
    got = G.to_f64(terms)
    np.testing.assert_allclose(got[0], t64["base_sq"], rtol=1e-5)
    # cross and ba_sq are sums with cancellation: bounded against the scale Cauchy-Schwarz gives them
    fine = 1e-5 if cfg.dtype == "f32" else 2e-4   # bf16: G carried as two bf16 terms (2^-16), fp32 sums
    scale = np.sqrt(t64["base_sq"] * t64["ba_sq"]) + 1e-30
    assert np.max(np.abs(got[1] - t64["cross"]) / scale) <= fine
    np.testing.assert_allclose(got[2], t64["ba_sq"], rtol=fine, atol=1e-30)
    assert G.rel_max(G.to_f64(Gm), t64["G"]) <= 1e-5
    c = G.empty_f32(cfg.d_out)
    D.dora_norm_assemble(mod.desc, terms, c)
    assert torch.equal(c, mod.norm())
    G.assert_norm_close(G.to_f64(c), O.dense_row_norm(mod.f64("W"), mod.f64("A"), mod.f64("B"), float(mod.inp["s"])),
                        G.TOL[cfg.dtype]["norm"])


def test_norm_terms_reuse_in_a_recomputed_backward_and_a_stale_cache_shows():
    # gradient-checkpointing pattern with the norm's terms carried from the forward: the recomputed
    # backward re-assembles Eq. 5 from them (one small launch) instead of re-running the contractions
    cfg = I.stress(cfg_bf16("terms_reuse", 520, 392, 40, 300, seed=31))
    mod = G.Module(cfg)
    ws = G.workspace(mod.desc, D.PHASE_BACKWARD_RECOMPUTE)
    terms = G.empty_f32(3, cfg.d_out)
    D.dora_norm_terms(mod.desc, mod.W, mod.A, mod.B, terms, None, ws)
    c = G.empty_f32(cfg.d_out)
    D.dora_norm_assemble(mod.desc, terms, c)
    ref = mod.backward()                     # norm, h, inner all recomputed inside
    got = mod.backward(w_norm=c)             # norm from the carried terms, h and inner recomputed
    for k in ("dx", "dA", "dB", "dm"):
        assert torch.equal(ref[k], got[k]), k
    b = O.backward(mod.f64("dy"), **oracle_inputs(mod))
    for k in ("dx", "dA", "dB", "dm"):
        G.assert_close(k, G.to_f64(got[k]), b[k], G.TOL["bf16"]["tensor"])
    # the caller owns staleness: after B changes, terms computed before the change give the OLD norm
    B_new = (mod.B.float() * 1.5).to(mod.B.dtype)
    fresh = G.empty_f32(cfg.d_out)
    D.dora_norm(mod.desc, mod.W, mod.A, B_new, fresh, ws)
    stale = G.empty_f32(cfg.d_out)
    D.dora_norm_assemble(mod.desc, terms, stale)
    assert torch.equal(stale, c)
    assert float((stale - fresh).abs().max() / fresh.abs().max()) > 1e-2


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_norm_terms_with_zero_scale(dtype):
    mk = cfg_bf16 if dtype == "bf16" else cfg_f32
    cfg = mk("s0_terms", 264, 328, 24, 8, seed=22)
    mod = G.Module(cfg)
    desc = D.make_desc(cfg.d_out, cfg.d_in, cfg.r, cfg.tokens, G.dtype_code(dtype), 0.0, 0.0)
    terms, Gm, c = G.empty_f32(3, cfg.d_out), G.empty_f32(cfg.r, cfg.r), G.empty_f32(cfg.d_out)
    D.dora_norm_terms(desc, mod.W, mod.A, mod.B, terms, Gm, G.workspace(desc, D.PHASE_NORM))
    D.dora_norm_assemble(desc, terms, c)
    W = mod.f64("W")
    np.testing.assert_allclose(G.to_f64(terms[0]), np.sum(W * W, axis=1), rtol=1e-5)
    assert float(terms[1:].abs().max()) == 0.0 and float(Gm.abs().max()) == 0.0
    G.assert_norm_close(G.to_f64(c), np.linalg.norm(W, axis=1), G.TOL[dtype]["norm"])


def test_norm_low_rank_terms_matter_in_stress_variant():
    # guards the guard: in the stress variant dropping BA would be far outside tolerance
    cfg = I.stress(cfg_bf16("bf16_mid", 1024, 1536, 384, 640, seed=4))
    mod = G.Module(cfg)
    ref = O.dense_row_norm(mod.f64("W"), mod.f64("A"), mod.f64("B"), float(mod.inp["s"]))
    only_w = np.linalg.norm(mod.f64("W"), axis=1)
    assert np.max(np.abs(only_w - ref) / ref) > 0.1


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_norm_special_cases(dtype):
    mk = mk_of(dtype)
    cfg = mk("special", 264, 200, 16, 8, seed=6)
    inp = I.make_inputs(cfg)
    tol = G.TOL[dtype]["norm"]
    # B = 0: the row norm of W
    inp0 = dict(inp); inp0["B"] = np.zeros_like(inp["B"])
    mod = G.Module(cfg, inp0)
    G.assert_norm_close(G.to_f64(mod.norm()), np.linalg.norm(mod.f64("W"), axis=1), tol)
    # s = 0 fast path
    mod = G.Module(cfg, inp)
    mod.desc.s = 0.0
    G.assert_norm_close(G.to_f64(mod.norm()), np.linalg.norm(mod.f64("W"), axis=1), tol)
    # a zero row of W and of B gives norm 0 exactly, and g = m / eps stays finite
    inpz = dict(inp); inpz["W"] = inp["W"].copy(); inpz["B"] = inp["B"].copy()
    inpz["W"][3] = 0; inpz["B"][3] = 0
    mod = G.Module(cfg, inpz)
    c = mod.norm()
    assert float(c[3]) == 0.0
    g = G.empty_f32(cfg.d_out)
    D.dora_mag_scale(mod.desc, mod.m, c, g, None)
    ref_g = O.mag_scale(mod.inp["m"].astype(np.float64), G.to_f64(c), cfg.eps)
    assert np.isfinite(float(g[3])) and abs(float(g[3]) - ref_g[3]) <= 1e-6 * abs(ref_g[3])


def test_norm_nan_propagates():
    cfg = cfg_bf16("nan", 136, 128, 16, 8, seed=7)
    inp = I.make_inputs(cfg)
    inp["W"] = inp["W"].copy(); inp["W"][5, 7] = 0x7FC0  # a NaN weight
    c = G.to_f64(G.Module(cfg, inp).norm())
    assert np.isnan(c[5]) and np.all(np.isfinite(np.delete(c, 5)))


# ----------------------------------------------------------------------------- g (a6)

@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_mag_scale(dtype):
    rng = np.random.default_rng(1)
    n = 1000
    c = np.abs(rng.standard_normal(n)).astype(np.float32) + 0.5
    c[:3] = [0.0, 1e-9, 1e-20]
    m = (c.astype(np.float64) * (1 + 1e-3 * rng.standard_normal(n))).astype(np.float32)
    m[:3] = 1.0
    eps = 1e-12 if dtype == "f32" else 1e-6
    desc = D.make_desc(n, 8, 8, 0, G.dtype_code(dtype), 1.0)
    g, gm1 = G.empty_f32(n), G.empty_f32(n)
    D.dora_mag_scale(desc, G.to_dev(m), G.to_dev(c), g, gm1)
    ref = O.mag_scale(m.astype(np.float64), c.astype(np.float64), eps)
    np.testing.assert_allclose(G.to_f64(g), ref, rtol=2e-7)
    # the explicit correction keeps full relative accuracy although g - 1 ~ 1e-3
    np.testing.assert_allclose(G.to_f64(gm1)[3:], (ref - 1)[3:], rtol=1e-6, atol=1e-10)


# ----------------------------------------------------------------------------- compose forward (a9)

@pytest.mark.parametrize("dtype,tokens,d_out", [("f32", 64, 256), ("f32", 33, 100), ("bf16", 77, 200),
                                               ("bf16", 300, 2056), ("bf16", 1, 8), ("bf16", 1030, 4096),
                                               ("f16", 77, 200), ("f16", 1030, 4096)])
def test_compose_forward(dtype, tokens, d_out):
    rng = np.random.default_rng(tokens * 7 + d_out)
    base_s = I.quantise(rng.standard_normal((tokens, d_out)), dtype)
    lora_s = I.quantise(rng.standard_normal((tokens, d_out)) * 0.02, dtype)
    g64 = 1 + 0.0015 * rng.standard_normal(d_out)
    g32 = g64.astype(np.float32)
    gm1_32 = (g64 - 1).astype(np.float32)
    s = np.float32(1.6329931)
    desc = D.make_desc(d_out, 8, 8, tokens, G.dtype_code(dtype), float(s))
    base, lora = G.to_dev(base_s), G.to_dev(lora_s)
    ref_delta = O.compose_delta(I.to_f64(base_s), I.to_f64(lora_s), g32.astype(np.float64), float(s))
    ref_inner = float(s) * I.to_f64(lora_s) + I.to_f64(base_s)
    tol = G.TOL[dtype]["tensor"]
    # delta with explicit gm1 (reference uses the same fp32 g, and gm1 as given)
    ref_delta_gm1 = gm1_32.astype(np.float64)[None] * I.to_f64(base_s) + g32.astype(np.float64)[None] * (float(s) * I.to_f64(lora_s))
    out, inner = G.empty((tokens, d_out), dtype), G.empty((tokens, d_out), dtype)
    D.dora_compose(desc, base, lora, G.to_dev(g32), G.to_dev(gm1_32), out, 1, inner)
    G.assert_close("delta(gm1)", G.to_f64(out), ref_delta_gm1, tol)
    G.assert_close("inner", G.to_f64(inner), ref_inner, tol)
    # delta with gm1 = NULL (g - 1 formed in fp32), and the y form
    D.dora_compose(desc, base, lora, G.to_dev(g32), None, out, 1, None)
    G.assert_close("delta", G.to_f64(out), ref_delta, tol)
    D.dora_compose(desc, base, lora, G.to_dev(g32), None, out, 0, None)
    G.assert_close("y", G.to_f64(out), I.to_f64(base_s) + ref_delta, tol)
    # in place: out aliases base, inner aliases lora
    b2, l2 = base.clone(), lora.clone()
    D.dora_compose(desc, b2, l2, G.to_dev(g32), G.to_dev(gm1_32), b2, 0, l2)
    G.assert_close("y in place", G.to_f64(b2), I.to_f64(base_s) + ref_delta_gm1, tol)
    G.assert_close("inner in place", G.to_f64(l2), ref_inner, tol)
    if dtype == "bf16":
        # stricter than the tolerance: the delta is within bf16 rounding of the exact value
        err = np.abs(G.to_f64(out) - (I.to_f64(base_s) + ref_delta))
        assert np.max(err) <= 2.0 ** -8 * np.max(np.abs(I.to_f64(base_s) + ref_delta))


def test_compose_forward_stable_near_unity():
    # Sec. 3.1: with g within 1 +- 0.0015 the delta written in bf16 stays at the rounding floor of the
    # delta itself (not of base), i.e. the (g-1) correction is not lost.
    rng = np.random.default_rng(5)
    tokens, d_out = 256, 1024
    base_s = I.quantise(rng.standard_normal((tokens, d_out)), "bf16")
    lora_s = I.quantise(np.zeros((tokens, d_out)), "bf16")
    g32 = (1 + 0.0015 * rng.standard_normal(d_out)).astype(np.float32)
    desc = D.make_desc(d_out, 8, 8, tokens, D.DORA_BF16, 1.0)
    out = G.empty((tokens, d_out), "bf16")
    D.dora_compose(desc, G.to_dev(base_s), G.to_dev(lora_s), G.to_dev(g32), None, out, 1, None)
    ref = O.compose_delta(I.to_f64(base_s), I.to_f64(lora_s), g32.astype(np.float64), 1.0)
    err = np.abs(G.to_f64(out) - ref)
    assert np.all(err <= 2.0 ** -8 * np.abs(ref) + 1e-30)


def test_fp16_store_overflows_to_infinity_like_the_ieee_conversion():
    # App. B "Dtype-aware epsilon": fp16 ends at 65504.  A result beyond it becomes an infinity when it is
    # stored, exactly as the IEEE conversion of the oracle's value does; nothing is clamped, and the
    # elements around it are untouched.
    tokens, d_out = 16, 64
    base64 = np.full((tokens, d_out), 100.0)
    base64[3, 5], base64[4, 6], base64[7, 9] = 60000.0, -60000.0, 65000.0
    base_s, lora_s = I.quantise(base64, "f16"), I.quantise(np.zeros((tokens, d_out)), "f16")
    g32 = np.full(d_out, 1.2, np.float32)
    g32[9] = 1.0
    desc = D.make_desc(d_out, 8, 8, tokens, D.DORA_F16, 1.0)
    out = G.empty((tokens, d_out), "f16")
    D.dora_compose(desc, G.to_dev(base_s), G.to_dev(lora_s), G.to_dev(g32), None, out, 0, None)
    ref = I.to_f64(base_s) + O.compose_delta(I.to_f64(base_s), I.to_f64(lora_s), g32.astype(np.float64), 1.0)
    ref16 = I.to_f64(I.quantise(ref, "f16"))
    got = G.to_f64(out)
    assert got[3, 5] == np.inf and got[4, 6] == -np.inf and got[7, 9] == 65000.0 - 8.0   # 65000 rounds to 64992
    assert np.array_equal(np.isinf(got), np.isinf(ref16))
    fin = np.isfinite(ref16)
    assert np.max(np.abs(got[fin] - ref[fin]) / np.abs(ref[fin])) <= 2.0 ** -11


# ----------------------------------------------------------------------------- compose backward (a10)

@pytest.mark.parametrize("dtype,tokens,d_out", [("f32", 64, 256), ("f32", 130, 100), ("bf16", 77, 200),
                                               ("bf16", 300, 2056), ("bf16", 1030, 4096), ("f16", 77, 200),
                                               ("f16", 1030, 4096)])
def test_compose_backward(dtype, tokens, d_out):
    rng = np.random.default_rng(tokens * 3 + d_out)
    dy_s = I.quantise(rng.standard_normal((tokens, d_out)), dtype)
    inner_s = I.quantise(rng.standard_normal((tokens, d_out)), dtype)
    g32 = (1 + 0.0015 * rng.standard_normal(d_out)).astype(np.float32)
    c32 = (np.abs(rng.standard_normal(d_out)) + 0.5).astype(np.float32)
    desc = D.make_desc(d_out, 8, 8, tokens, G.dtype_code(dtype), 1.5)
    eps = 1e-12 if dtype == "f32" else 1e-6
    dz, dm = G.empty((tokens, d_out), dtype), G.empty_f32(d_out)
    ws = G.workspace(desc, D.PHASE_COMPOSE_BACKWARD)
    D.dora_compose_backward(desc, G.to_dev(dy_s), G.to_dev(inner_s), G.to_dev(g32), G.to_dev(c32), dz, dm, ws)
    d_lora, d_base, ref_dm = O.grad_compose(I.to_f64(dy_s), I.to_f64(inner_s), g32.astype(np.float64),
                                            c32.astype(np.float64), 1.5, eps)
    tol = G.TOL[dtype]["tensor"]
    G.assert_close("dz", G.to_f64(dz), d_base, tol)
    np.testing.assert_allclose(d_lora, 1.5 * d_base, rtol=1e-14)  # the gradient reaching lora is s * dz
    # dm is an fp32 sum of exact products: far tighter than the bf16 tolerance
    G.assert_close("dm", G.to_f64(dm), ref_dm, 1e-5)
    # frozen magnitude: dm skipped, inner / w_norm may be NULL
    dz2 = G.empty((tokens, d_out), dtype)
    D.dora_compose_backward(desc, G.to_dev(dy_s), None, G.to_dev(g32), None, dz2, None, None)
    assert torch.equal(dz2.view(torch.uint8), dz.view(torch.uint8))


def test_compose_passes_on_millions_of_tokens_of_a_narrow_module():
    # 9 million tokens x 8 outputs: 70313 row slabs of 128, beyond what a 65535-limited grid axis could carry
    tokens, d_out = 9_000_000, 8
    rng = np.random.default_rng(99)
    base_s = I.quantise(rng.standard_normal((tokens, d_out), dtype=np.float32), "bf16")
    lora_s = I.quantise(rng.standard_normal((tokens, d_out), dtype=np.float32) * 0.02, "bf16")
    g32 = (1 + 0.0015 * rng.standard_normal(d_out)).astype(np.float32)
    c32 = np.ones(d_out, np.float32)
    desc = D.make_desc(d_out, 8, 8, tokens, D.DORA_BF16, 1.5)
    base, lora = G.to_dev(base_s), G.to_dev(lora_s)
    y, inner = G.empty((tokens, d_out), "bf16"), G.empty((tokens, d_out), "bf16")
    D.dora_compose(desc, base, lora, G.to_dev(g32), None, y, 0, inner)
    rows = np.concatenate([np.arange(300), rng.integers(0, tokens, 5000), np.arange(tokens - 300, tokens)])
    b64, l64 = I.to_f64(base_s[rows]), I.to_f64(lora_s[rows])
    ridx = torch.from_numpy(rows).to(y.device)
    G.assert_close("y[rows]", G.to_f64(y[ridx]), b64 + O.compose_delta(b64, l64, g32.astype(np.float64), 1.5), 2e-2)
    assert bool(torch.isfinite(y.float()).all())       # every slab was written
    dz, dm = G.empty((tokens, d_out), "bf16"), G.empty_f32(d_out)
    ws = G.workspace(desc, D.PHASE_COMPOSE_BACKWARD)
    D.dora_compose_backward(desc, base, inner, G.to_dev(g32), G.to_dev(c32), dz, dm, ws)
    assert bool(torch.isfinite(dz.float()).all())
    ref_dm = np.einsum("tj,tj->j", I.to_f64(base_s), G.to_f64(inner))
    G.assert_close("dm", G.to_f64(dm), ref_dm, 1e-4)


# ----------------------------------------------------------------------------- contractions (a7, a8)

@pytest.mark.parametrize("cfg", SMALL, ids=IDS)
def test_project_and_delta(cfg):
    mod = G.Module(cfg)
    base = G.empty((cfg.tokens, cfg.d_out), cfg.dtype)
    h = G.empty((cfg.tokens, cfg.r), cfg.dtype)
    lora = G.empty((cfg.tokens, cfg.d_out), cfg.dtype)
    D.dora_project(mod.desc, mod.x, mod.W, mod.A, mod.B, base, h, lora)
    f = O.forward(**oracle_inputs(mod))
    tol = G.TOL[cfg.dtype]["tensor"]
    G.assert_close("base", G.to_f64(base), f["base"], tol)
    G.assert_close("h", G.to_f64(h), f["h"], tol)
    G.assert_close("lora", G.to_f64(lora), f["lora"], tol)
    # delta through the library's own norm, g and compose
    c = mod.norm()
    g, gm1 = G.empty_f32(cfg.d_out), G.empty_f32(cfg.d_out)
    D.dora_mag_scale(mod.desc, mod.m, c, g, gm1)
    delta = G.empty((cfg.tokens, cfg.d_out), cfg.dtype)
    D.dora_compose(mod.desc, base, lora, g, gm1, delta, 1, None)
    G.assert_close("delta", G.to_f64(delta), f["delta"], tol)


# ----------------------------------------------------------------------------- whole module

@pytest.mark.parametrize("cfg", SMALL, ids=IDS)
def test_forward_backward(cfg):
    mod = G.Module(cfg)
    oi = oracle_inputs(mod)
    f = O.forward(**oi)
    tol = G.TOL[cfg.dtype]["tensor"]
    out = mod.forward()
    G.assert_norm_close(G.to_f64(out["c"]), f["c"], G.TOL[cfg.dtype]["norm"])
    G.assert_close("y", G.to_f64(out["y"]), f["y"], tol)
    G.assert_close("inner", G.to_f64(out["inner"]), f["inner"], tol)
    G.assert_close("h", G.to_f64(out["h"]), f["h"], tol)
    # forward without saving anything gives the same y
    out2 = mod.forward(save=False)
    assert torch.equal(out2["y"].view(torch.uint8), out["y"].view(torch.uint8))
    # forward with a supplied norm gives the same y
    out3 = mod.forward(w_norm=out["c"], save=False)
    assert torch.equal(out3["y"].view(torch.uint8), out["y"].view(torch.uint8))

    b = O.backward(mod.f64("dy"), **oi)
    for label, grads in (
        ("saved", mod.backward(w_norm=out["c"], h=out["h"], inner=out["inner"])),
        ("recompute", mod.backward()),
    ):
        for k in ("dx", "dA", "dB", "dm"):
            G.assert_close(f"{k} [{label}]", G.to_f64(grads[k]), b[k], tol)
    # frozen magnitude: same dx, dA, dB without inner
    gf = mod.backward(w_norm=out["c"], h=out["h"], inner=None, want_dm=False)
    ref = mod.backward(w_norm=out["c"], h=out["h"], inner=out["inner"])
    for k in ("dx", "dA", "dB"):
        assert torch.equal(gf[k].view(torch.uint8), ref[k].view(torch.uint8)), k


MINIMAL = [
    cfg_bf16("bf16_minimum", 8, 8, 8, 1, sigma_B=2e-2, seed=31),       # the smallest shapes the ABI accepts
    cfg_f32("f32_minimum", 4, 4, 4, 1, seed=32),
    cfg_bf16("bf16_one_token_wide", 8, 1032, 8, 1, sigma_B=2e-2, seed=33),
    cfg_bf16("bf16_rank_over_dims", 72, 40, 136, 65, sigma_B=2e-2, seed=34),   # r larger than d_in and d_out
]


@pytest.mark.parametrize("cfg", MINIMAL, ids=[c.name for c in MINIMAL])
def test_forward_backward_at_degenerate_sizes(cfg):
    mod = G.Module(cfg)
    oi = oracle_inputs(mod)
    f = O.forward(**oi)
    tol = G.TOL[cfg.dtype]["tensor"]
    out = mod.forward()
    G.assert_norm_close(G.to_f64(out["c"]), f["c"], G.TOL[cfg.dtype]["norm"])
    for k in ("y", "inner", "h"):
        G.assert_close(k, G.to_f64(out[k]), f[k], tol)
    if cfg.dtype != "f32":
        fused = mod.forward(fused=True)
        G.assert_close("y [fused]", G.to_f64(fused["y"]), f["y"], tol)
    b = O.backward(mod.f64("dy"), **oi)
    grads = mod.backward()
    for k in ("dx", "dA", "dB", "dm"):
        G.assert_close(k, G.to_f64(grads[k]), b[k], tol)


def test_initial_state_is_identity():
    # B = 0 and m = ||W||_row (DoRA's initialisation): y equals the base projection
    cfg = cfg_bf16("init", 520, 392, 40, 300, seed=9)
    inp = I.make_inputs(cfg)
    inp["B"] = np.zeros_like(inp["B"])
    inp["m"] = np.linalg.norm(I.to_f64(inp["W"]), axis=1).astype(np.float32)
    mod = G.Module(cfg, inp)
    out = mod.forward()
    ref = mod.f64("x") @ mod.f64("W").T
    G.assert_close("y", G.to_f64(out["y"]), ref, 2.0 ** -8)


def test_runs_are_bitwise_reproducible():
    cfg = cfg_bf16("bf16_ragged", 520, 392, 40, 300, seed=3)
    mod = G.Module(cfg)
    a, b = mod.forward(), mod.forward()
    ga, gb = mod.backward(), mod.backward()
    for k in ("y", "inner", "h", "c"):
        assert torch.equal(a[k].view(torch.uint8), b[k].view(torch.uint8)), k
    for k in ("dx", "dA", "dB", "dm"):
        assert torch.equal(ga[k].view(torch.uint8), gb[k].view(torch.uint8)), k


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_zero_tokens(dtype):
    mk = cfg_bf16 if dtype == "bf16" else cfg_f32
    cfg = mk("empty", 136, 72, 16, 0, seed=10)
    mod = G.Module(cfg)
    out = mod.forward()
    ref = O.dense_row_norm(mod.f64("W"), mod.f64("A"), mod.f64("B"), float(mod.inp["s"]))
    G.assert_norm_close(G.to_f64(out["c"]), ref, G.TOL[dtype]["norm"])
    g = mod.backward()
    assert float(g["dA"].abs().max()) == 0.0 and float(g["dB"].abs().max()) == 0.0 and float(g["dm"].abs().max()) == 0.0


def test_probes_run_and_copy_is_exact():
    n = 3 * 2 ** 20 + 4096 + 16
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=G.DEV)
    dst = torch.zeros_like(src)
    D.dora_probe_copy(src, dst, n)
    assert torch.equal(src, dst)
    sink = torch.zeros(512, dtype=torch.float32, device=G.DEV)
    operands = torch.randn(65536 // 2, device=G.DEV).to(torch.bfloat16)
    D.dora_probe_mfma(operands, sink, 4, 8)
    torch.cuda.synchronize()
    assert float(sink.abs().max()) == 0.0


BF16_CASES = [c for c in SMALL if c.dtype != "f32"]   # the 16-bit storage types


@pytest.mark.parametrize("cfg", BF16_CASES, ids=[c.name for c in BF16_CASES])
def test_fused_forward_matches_oracle_and_contract_path(cfg):
    # K-concatenated forward with the compose folded into the MFMA epilogue
    mod = G.Module(cfg)
    f = O.forward(**oracle_inputs(mod))
    tol = G.TOL[cfg.dtype]["tensor"]
    out = mod.forward(fused=True)
    G.assert_norm_close(G.to_f64(out["c"]), f["c"], G.TOL[cfg.dtype]["norm"])
    G.assert_close("y", G.to_f64(out["y"]), f["y"], tol)
    G.assert_close("inner", G.to_f64(out["inner"]), f["inner"], tol)
    G.assert_close("h", G.to_f64(out["h"]), f["h"], tol)
    # it rounds once from the fp32 accumulator: at least as close to the oracle as the two-pass path
    ref = mod.forward()
    e_fused = G.rel_fro(G.to_f64(out["y"]), f["y"])
    e_two = G.rel_fro(G.to_f64(ref["y"]), f["y"])
    assert e_fused <= 1.05 * e_two + 1e-6
    # without saved tensors, and with a supplied norm: same y
    out2 = mod.forward(fused=True, save=False, w_norm=out["c"])
    assert torch.equal(out2["y"].view(torch.uint8), out["y"].view(torch.uint8))
    # the saved tensors drive the backward as usual
    b = O.backward(mod.f64("dy"), **oracle_inputs(mod))
    grads = mod.backward(w_norm=out["c"], h=out["h"], inner=out["inner"])
    for k in ("dx", "dA", "dB", "dm"):
        G.assert_close(k, G.to_f64(grads[k]), b[k], tol)


def test_fused_forward_rejects_fp32():
    mod = G.Module(I.C1)
    with pytest.raises(D.DoraError) as e:
        mod.forward(fused=True)
    assert e.value.status == 4


# ----------------------------------------------------------------------------- LoRA dropout (App. B)

DROPOUT_CASES = [SMALL[1], SMALL[3], SMALL[4], SMALL[7], SMALL[9]]


@pytest.mark.parametrize("cfg", DROPOUT_CASES, ids=[c.name for c in DROPOUT_CASES])
def test_dropout_forward_and_backward(cfg):
    # the adapter branch sees x_lora = dropout(x); the frozen layer's output stays that of x
    mod = G.Module(cfg)
    xl_s = I.dropped_input(cfg, mod.inp["x"], 0.25)
    x_lora = G.to_dev(xl_s)
    oi = oracle_inputs(mod)
    f = O.forward(**oi, x_lora=I.to_f64(xl_s))
    tol = G.TOL[cfg.dtype]["tensor"]
    T, do, di, r = cfg.tokens, cfg.d_out, cfg.d_in, cfg.r
    y, h, inner, c = G.empty((T, do), cfg.dtype), G.empty((T, r), cfg.dtype), G.empty((T, do), cfg.dtype), G.empty_f32(do)
    D.dora_forward_dropout(mod.desc, mod.x, x_lora, mod.W, mod.A, mod.B, mod.m, None, None, y, h, inner, c,
                           G.workspace(mod.desc, D.PHASE_FORWARD_DROPOUT))
    G.assert_norm_close(G.to_f64(c), f["c"], G.TOL[cfg.dtype]["norm"])
    for k, v in (("y", y), ("h", h), ("inner", inner)):
        G.assert_close(k, G.to_f64(v), f[k], tol)
    # the dropped input must really be used: the plain forward is far away
    assert G.rel_fro(O.forward(**oi)["inner"], f["inner"]) > 0.1
    b = O.backward_dropout(mod.f64("dy"), oi["x"], I.to_f64(xl_s), oi["W"], oi["A"], oi["B"], oi["m"], oi["s"], oi["eps"])
    ws = G.workspace(mod.desc, D.PHASE_BACKWARD_DROPOUT)
    for saved in (True, False):   # from the saved tensors, and with norm, h and inner recomputed from x_lora
        dx, dxl = G.empty((T, di), cfg.dtype), G.empty((T, di), cfg.dtype)
        dA, dB, dm = G.empty_f32(r, di), G.empty_f32(do, r), G.empty_f32(do)
        D.dora_backward_dropout(mod.desc, mod.dy, x_lora, mod.W, mod.A, mod.B, mod.m, c if saved else None,
                                h if saved else None, inner if saved else None, dx, dxl, dA, dB, dm, ws)
        for k, v in (("dx", dx), ("dx_lora", dxl), ("dA", dA), ("dB", dB), ("dm", dm)):
            G.assert_close(f"{k} [{'saved' if saved else 'recompute'}]", G.to_f64(v), b[k], tol)


def test_dropout_entry_points_without_dropout_are_the_plain_module():
    cfg = cfg_bf16("dropout_p0", 520, 392, 40, 300, seed=3)
    mod = G.Module(cfg)
    plain = mod.forward()
    T, do, di, r = cfg.tokens, cfg.d_out, cfg.d_in, cfg.r
    y, h, inner, c = G.empty((T, do), "bf16"), G.empty((T, r), "bf16"), G.empty((T, do), "bf16"), G.empty_f32(do)
    D.dora_forward_dropout(mod.desc, mod.x, mod.x, mod.W, mod.A, mod.B, mod.m, None, None, y, h, inner, c,
                           G.workspace(mod.desc, D.PHASE_FORWARD_DROPOUT))
    for a, b_ in ((y, plain["y"]), (h, plain["h"]), (inner, plain["inner"])):
        assert torch.equal(a.view(torch.int16), b_.view(torch.int16))
    grads = mod.backward(w_norm=c, h=h, inner=inner)
    dx, dxl = G.empty((T, di), "bf16"), G.empty((T, di), "bf16")
    dA, dB, dm = G.empty_f32(r, di), G.empty_f32(do, r), G.empty_f32(do)
    D.dora_backward_dropout(mod.desc, mod.dy, mod.x, mod.W, mod.A, mod.B, mod.m, c, h, inner, dx, dxl, dA, dB, dm,
                            G.workspace(mod.desc, D.PHASE_BACKWARD_DROPOUT))
    for k, v in (("dA", dA), ("dB", dB), ("dm", dm)):
        assert torch.equal(v, grads[k]), k
    G.assert_close("dx + dx_lora", G.to_f64(dx) + G.to_f64(dxl), G.to_f64(grads["dx"]), G.TOL["bf16"]["tensor"])
    # a missing adapter input is an error, not a silent fall back to x
    with pytest.raises(D.DoraError) as e:
        D.dora_forward_dropout(mod.desc, mod.x, None, mod.W, mod.A, mod.B, mod.m, None, None, y, h, inner, c,
                               G.workspace(mod.desc, D.PHASE_FORWARD_DROPOUT))
    assert e.value.status == 1


# ----------------------------------------------------------------------------- bias of the base layer

@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[2], SMALL[5], SMALL[6], SMALL[10]], ids=[IDS[0], IDS[2], IDS[5], IDS[6], IDS[10]])
@pytest.mark.parametrize("fused", [False, True], ids=["compose_pass", "fused_epilogue"])
def test_forward_with_bias(cfg, fused):
    # App. A item 2: the frozen layer's bias is not part of the compose; y = base + delta + bias
    if fused and cfg.dtype == "f32":
        pytest.skip("the K-concatenated forward is for 16-bit storage only")
    mod = G.Module(cfg)
    rng = np.random.default_rng(4242)
    bias64 = rng.normal(size=cfg.d_out)
    stored = I.quantise(bias64, cfg.dtype)
    bias_dev = G.to_dev(stored)
    ref = O.forward(**oracle_inputs(mod), bias=I.to_f64(stored))
    out = mod.forward(fused=fused, bias=bias_dev)
    tol = G.TOL[cfg.dtype]["tensor"]
    G.assert_close("y", G.to_f64(out["y"]), ref["y"], tol)
    G.assert_close("inner", G.to_f64(out["inner"]), ref["inner"], tol)
    # the bias must really be there: without it the result is off by about |bias|
    plain = O.forward(**oracle_inputs(mod))
    assert G.rel_max(G.to_f64(out["y"]), plain["y"]) > 10 * tol


# ----------------------------------------------------------------------------- streams and graph capture

def _step_outputs(mod, stream=None):
    cfg = mod.cfg
    y = G.empty((cfg.tokens, cfg.d_out), cfg.dtype)
    h = G.empty((cfg.tokens, cfg.r), cfg.dtype)
    inner = G.empty((cfg.tokens, cfg.d_out), cfg.dtype)
    c = G.empty_f32(cfg.d_out)
    dx = G.empty((cfg.tokens, cfg.d_in), cfg.dtype)
    dA, dB, dm = G.empty_f32(cfg.r, cfg.d_in), G.empty_f32(cfg.d_out, cfg.r), G.empty_f32(cfg.d_out)
    ws_f = G.workspace(mod.desc, D.PHASE_FORWARD)
    ws_b = G.workspace(mod.desc, D.PHASE_BACKWARD)

    def run():
        D.dora_forward(mod.desc, mod.x, mod.W, mod.A, mod.B, mod.m, None, None, y, h, inner, c, ws_f, stream=stream)
        D.dora_backward(mod.desc, mod.dy, mod.x, mod.W, mod.A, mod.B, mod.m, c, h, inner, dx, dA, dB, dm, ws_b,
                        stream=stream)
    return run, {"y": y, "h": h, "inner": inner, "c": c, "dx": dx, "dA": dA, "dB": dB, "dm": dm}


def _same_bits(a, b):
    return all(torch.equal(a[k].view(torch.uint8), b[k].view(torch.uint8)) for k in a)


def test_work_follows_the_given_stream():
    # Everything is enqueued on the stream handed in (default priority), nothing on the null stream: results on a side
    # stream equal those on the default stream, also while the default stream is kept busy with unrelated work.
    mod = G.Module(cfg_bf16("bf16_stream", 520, 392, 40, 300, seed=41))
    run0, out0 = _step_outputs(mod)
    run0()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    run1, out1 = _step_outputs(mod, stream=side)
    torch.cuda.synchronize()
    busy = torch.empty(64 << 20, dtype=torch.uint8, device=G.DEV)
    for _ in range(4):
        busy.fill_(1)                       # on the default stream, concurrently
    run1()
    side.synchronize()
    torch.cuda.synchronize()
    assert _same_bits(out0, out1)


def test_step_can_be_captured_in_a_graph_and_replayed():
    # The library allocates nothing and synchronises nothing, so a forward + backward is capturable; every replay,
    # with eager work and synchronisation in between, must reproduce the eager result bit for bit.
    mod = G.Module(cfg_bf16("bf16_graph", 520, 392, 40, 300, seed=42))
    run_e, out_e = _step_outputs(mod)
    run_e()
    torch.cuda.synchronize()
    run_g, out_g = _step_outputs(mod)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_g()
    for rep in range(3):
        for t in out_g.values():
            t.view(torch.uint8).fill_(0xFF)    # poison the outputs (NaN patterns) before each replay
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert _same_bits(out_e, out_g), rep
        run_e()                              # eager work between replays
        torch.cuda.synchronize()
