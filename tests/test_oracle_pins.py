"""Pins for the CPU oracle: things the paper and the mathematics fix, independent of the oracle's own code.

Each test is chosen so that a plausible slip in oracle/dora_oracle.py (a dropped term, a wrong
sign, a transposed operand, the wrong reduction axis, a non-detached norm) fails at least one.
"""
import ctypes
import os

import numpy as np
import pytest

from oracle import dora_oracle as O
from oracle import build as obuild

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(seed, *shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def small_problem(seed=0, T=5, d_out=7, d_in=6, r=3, s=1.7):
    W = rnd(seed + 1, d_out, d_in)
    A = rnd(seed + 2, r, d_in)
    B = rnd(seed + 3, d_out, r)
    m = np.abs(rnd(seed + 4, d_out)) + 0.5
    x = rnd(seed + 5, T, d_in)
    dy = rnd(seed + 6, T, d_out)
    return x, W, A, B, m, s, dy


# ----------------------------------------------------------------------------- norm

def test_hand_worked_row_norm():
    # One row, by hand: W = [3, 4], A = [[1, 0]], B = [[1]], s = 2  =>  D = [5, 4], ||D|| = sqrt(41).
    W = np.array([[3.0, 4.0]])
    A = np.array([[1.0, 0.0]])
    B = np.array([[1.0]])
    assert O.dense_row_norm(W, A, B, 2.0)[0] == pytest.approx(np.sqrt(41.0), rel=1e-15)
    # Two rows, r = 2: D = W + s B A with s = 0.5
    W = np.array([[1.0, 2.0, 2.0], [0.0, -3.0, 4.0]])
    A = np.array([[2.0, 0.0, 0.0], [0.0, 2.0, 0.0]])
    B = np.array([[1.0, 1.0], [0.0, 3.0]])
    # row0: [1+1, 2+1, 2] = [2,3,2] -> sqrt(17); row1: [0, -3+3, 4] -> 4
    c = O.dense_row_norm(W, A, B, 0.5)
    np.testing.assert_allclose(c, [np.sqrt(17.0), 4.0], rtol=1e-15)
    # factored terms by hand for row0: base 9, cross <W0,(BA)0> = [1,2,2].[2,2,0] = 6, ba 8 -> 9 + 2*.5*6 + .25*8 = 17
    t = O.factored_norm_terms(W, A, B)
    assert t["base_sq"][0] == 9.0 and t["cross"][0] == 6.0 and t["ba_sq"][0] == 8.0
    np.testing.assert_allclose(O.assemble_norm(t["base_sq"], t["cross"], t["ba_sq"], 0.5), c, rtol=1e-15)


def test_B_zero_and_s_zero_give_row_norm_of_W():
    x, W, A, B, m, s, dy = small_problem(1, d_out=9, d_in=11, r=4)
    ref = np.linalg.norm(W, axis=1)
    np.testing.assert_allclose(O.dense_row_norm(W, A, np.zeros_like(B), s), ref, rtol=1e-14)
    np.testing.assert_allclose(O.dense_row_norm(W, A, B, 0.0), ref, rtol=1e-14)
    np.testing.assert_allclose(O.factored_row_norm(W, A, B, 0.0), ref, rtol=1e-14)
    np.testing.assert_allclose(O.factored_row_norm(W, A, np.zeros_like(B), s), ref, rtol=1e-14)


def test_magnitude_at_init_reproduces_W_and_base():
    # m = ||W||_row and B = 0 (DoRA's initial state): g = 1, W' = W, delta = 0, y = base.
    x, W, A, B, m, s, dy = small_problem(2)
    B0 = np.zeros_like(B)
    m0 = np.linalg.norm(W, axis=1)
    np.testing.assert_allclose(O.adapted_weight(W, A, B0, m0, s, 1e-12), W, rtol=1e-14, atol=1e-15)
    f = O.forward(x, W, A, B0, m0, s, 1e-12)
    np.testing.assert_allclose(f["g"], 1.0, rtol=1e-14)
    assert np.max(np.abs(f["delta"])) < 1e-14
    np.testing.assert_allclose(f["y"], x @ W.T, rtol=1e-13, atol=1e-14)


def test_rank_one_closed_form():
    # ||W_j + s b_j a||^2 = ||W_j||^2 + 2 s b_j (W_j . a) + s^2 b_j^2 ||a||^2
    rng = np.random.default_rng(3)
    W = rng.standard_normal((8, 10))
    a = rng.standard_normal((1, 10))
    b = rng.standard_normal((8, 1))
    s = -0.8
    closed = np.sqrt((W ** 2).sum(1) + 2 * s * b[:, 0] * (W @ a[0]) + s * s * b[:, 0] ** 2 * (a[0] @ a[0]))
    np.testing.assert_allclose(O.dense_row_norm(W, a, b, s), closed, rtol=1e-13)
    np.testing.assert_allclose(O.factored_row_norm(W, a, b, s), closed, rtol=1e-13)


def test_orthonormal_A_and_zero_W():
    rng = np.random.default_rng(4)
    d_in, r, d_out = 12, 5, 6
    Q, _ = np.linalg.qr(rng.standard_normal((d_in, r)))
    A = Q.T  # orthonormal rows: G = I
    B = rng.standard_normal((d_out, r))
    s = 1.3
    t = O.factored_norm_terms(np.zeros((d_out, d_in)), A, B)
    np.testing.assert_allclose(t["G"], np.eye(r), atol=1e-14)
    np.testing.assert_allclose(t["ba_sq"], (B ** 2).sum(1), rtol=1e-13)
    # W = 0: the norm is |s| ||B_j|| when A has orthonormal rows
    np.testing.assert_allclose(O.dense_row_norm(np.zeros((d_out, d_in)), A, B, s),
                               abs(s) * np.linalg.norm(B, axis=1), rtol=1e-13)


def test_homogeneity_and_cauchy_schwarz():
    x, W, A, B, m, s, dy = small_problem(5, d_out=10, d_in=13, r=4)
    c = O.dense_row_norm(W, A, B, s)
    for alpha in (-2.5, 0.3):
        np.testing.assert_allclose(O.dense_row_norm(alpha * W, A, alpha * B, s), abs(alpha) * c, rtol=1e-13)
    t = O.factored_norm_terms(W, A, B)
    assert np.all(np.abs(t["cross"]) <= np.sqrt(t["base_sq"] * t["ba_sq"]) * (1 + 1e-12))
    assert np.all(t["base_sq"] + 2 * s * t["cross"] + s * s * t["ba_sq"] >= 0)


@pytest.mark.parametrize("seed", range(6))
def test_factored_equals_dense_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    d_out, d_in, r = (int(v) for v in rng.integers(1, 9, size=3))
    W = rng.standard_normal((d_out, d_in))
    A = rng.standard_normal((r, d_in))
    B = rng.standard_normal((d_out, r))
    s = float(rng.standard_normal())
    dense = O.dense_row_norm(W, A, B, s)
    np.testing.assert_allclose(O.factored_row_norm(W, A, B, s), dense, rtol=1e-12, atol=1e-14)
    # independent of the chunking of d_in
    np.testing.assert_allclose(O.factored_row_norm(W, A, B, s, chunk=3), dense, rtol=1e-12, atol=1e-14)
    # library routine on the dense matrix
    np.testing.assert_allclose(dense, np.linalg.norm(W + s * B @ A, axis=1), rtol=1e-13)


def test_factored_terms_add_over_any_partition_of_the_columns():
    # every term is a sum over d_in (ba_sq is linear in G): over the blocks of a partition they add up
    # to the whole, which is what lets Algorithm 1 walk d_in in chunks
    rng = np.random.default_rng(77)
    W, A, B = rng.standard_normal((6, 11)), rng.standard_normal((3, 11)), rng.standard_normal((6, 3))
    whole = O.factored_norm_terms(W, A, B)
    perm = rng.permutation(11)
    parts = [perm[:2], perm[2:7], perm[7:]]
    blocks = [O.factored_norm_terms(W, A, B, p) for p in parts]
    for k in ("base_sq", "cross", "G", "ba_sq"):
        np.testing.assert_allclose(sum(b[k] for b in blocks), whole[k], rtol=1e-13, atol=1e-13)
    # each term against its own brute-force definition
    BA = B @ A
    np.testing.assert_allclose(whole["base_sq"], [sum(v * v for v in row) for row in W], rtol=1e-14)
    np.testing.assert_allclose(whole["cross"], [float(W[j] @ BA[j]) for j in range(6)], rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(whole["ba_sq"], [float(BA[j] @ BA[j]) for j in range(6)], rtol=1e-13)
    np.testing.assert_allclose(whole["G"], [[float(A[l] @ A[p]) for p in range(3)] for l in range(3)], rtol=1e-14)


def test_assembly_clamp_and_nan():
    # negative radicand (rounding artefact) clamps to 0; NaN propagates (App. C item 3)
    out = O.assemble_norm(np.array([1.0, np.nan, 4.0]), np.array([-1.0, 0.0, 0.0]), np.array([0.0, 0.0, 0.0]), 1.0)
    assert out[0] == 0.0 and np.isnan(out[1]) and out[2] == 2.0


def test_zero_row_and_eps():
    W = np.zeros((2, 4)); W[1] = [1, 0, 0, 0]
    A = np.ones((1, 4)); B = np.zeros((2, 1)); m = np.array([3.0, 2.0])
    g = O.mag_scale(m, O.dense_row_norm(W, A, B, 1.0), 1e-6)
    np.testing.assert_allclose(g, [3.0e6, 2.0])
    g = O.mag_scale(m, O.dense_row_norm(W, A, B, 1.0), 1e-12)
    np.testing.assert_allclose(g, [3.0e12, 2.0])


# ----------------------------------------------------------------------------- forward

def test_forward_equals_linear_layer_with_adapted_weight():
    # Eq. (1): the module's output is x W'^T.  Pins base/lora operand orientation and the compose algebra.
    x, W, A, B, m, s, dy = small_problem(6)
    f = O.forward(x, W, A, B, m, s, 1e-12)
    Wp = O.adapted_weight(W, A, B, m, s, 1e-12)
    np.testing.assert_allclose(f["y"], x @ Wp.T, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(f["delta"], x @ Wp.T - x @ W.T, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(f["inner"], x @ (W + s * B @ A).T, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(O.compose_delta(f["base"], f["lora"], f["g"], s), f["delta"], rtol=1e-14)
    # every row of W' has norm m (direction normalised, magnitude m)
    np.testing.assert_allclose(np.linalg.norm(Wp, axis=1), m, rtol=1e-13)


def test_numpy_oracle_matches_loop_transcription():
    lib = obuild.load()
    x, W, A, B, m, s, dy = small_problem(7, T=4, d_out=6, d_in=5, r=3, s=0.9)
    T, d_in = x.shape; d_out, r = B.shape
    eps = 1e-12
    P = lambda a: np.ascontiguousarray(a).ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    c = np.zeros(d_out); lib.lit_row_norm(P(W), P(A), P(B), s, d_out, d_in, r, P(c))
    np.testing.assert_allclose(O.dense_row_norm(W, A, B, s), c, rtol=1e-13)
    f = O.forward(x, W, A, B, m, s, eps)
    y = np.zeros((T, d_out)); lib.lit_forward_via_adapted_weight(P(x), P(W), P(A), P(B), P(m), s, eps, T, d_out, d_in, r, P(y))
    np.testing.assert_allclose(f["y"], y, rtol=1e-12, atol=1e-13)
    delta = np.zeros((T, d_out)); inner = np.zeros((T, d_out))
    lib.lit_forward_compose(P(x), P(W), P(A), P(B), P(m), s, eps, T, d_out, d_in, r, P(delta), P(inner))
    np.testing.assert_allclose(f["delta"], delta, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(f["inner"], inner, rtol=1e-12, atol=1e-13)
    b = O.backward(dy, x, W, A, B, m, s, eps)
    dx = np.zeros_like(x); dA = np.zeros_like(A); dB = np.zeros_like(B); dm = np.zeros_like(m)
    lib.lit_backward(P(dy), P(x), P(W), P(A), P(B), P(m), s, eps, T, d_out, d_in, r, P(dx), P(dA), P(dB), P(dm))
    for k, v in (("dx", dx), ("dA", dA), ("dB", dB), ("dm", dm)):
        np.testing.assert_allclose(b[k], v, rtol=1e-11, atol=1e-12, err_msg=k)


# ----------------------------------------------------------------------------- backward

def _loss(x, W, A, B, m, s, dy, c_frozen):
    # L = sum dy * y, with the norm either frozen at c_frozen or re-evaluated (c_frozen=None).
    # Written through Eq. (1) directly (x W'^T) so it does not reuse the oracle's compose path.
    D = W + s * B @ A
    c = np.linalg.norm(D, axis=1) if c_frozen is None else c_frozen
    Wp = (m / np.maximum(c, 1e-12))[:, None] * D
    return float(np.sum(dy * (x @ Wp.T)))


def _fd(fun, arr, h=1e-6):
    g = np.zeros_like(arr)
    it = np.nditer(arr, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = arr[i]
        arr[i] = old + h; fp = fun()
        arr[i] = old - h; fm = fun()
        arr[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


def test_gradients_match_finite_differences_with_detached_norm():
    x, W, A, B, m, s, dy = small_problem(8, T=4, d_out=5, d_in=6, r=3, s=1.1)
    c0 = O.dense_row_norm(W, A, B, s)
    b = O.backward(dy, x, W, A, B, m, s, 1e-12)
    for name, arr in (("dx", x), ("dA", A), ("dB", B), ("dm", m)):
        fd = _fd(lambda: _loss(x, W, A, B, m, s, dy, c0), arr)
        scale = np.max(np.abs(fd))
        assert np.max(np.abs(fd - b[name])) <= 1e-7 * scale, name


def test_negative_control_norm_not_detached_differs():
    # If the norm were differentiated through, dA and dB would come out different: this guards
    # against an oracle that silently implements the non-detached gradient.
    x, W, A, B, m, s, dy = small_problem(9, T=4, d_out=5, d_in=6, r=3, s=1.1)
    b = O.backward(dy, x, W, A, B, m, s, 1e-12)
    for name, arr in (("dA", A), ("dB", B)):
        fd = _fd(lambda: _loss(x, W, A, B, m, s, dy, None), arr)
        assert np.max(np.abs(fd - b[name])) > 1e-3 * np.max(np.abs(fd)), name
    # x and m do not enter the norm: their gradients are the same either way
    for name, arr in (("dx", x), ("dm", m)):
        fd = _fd(lambda: _loss(x, W, A, B, m, s, dy, None), arr)
        assert np.max(np.abs(fd - b[name])) <= 1e-7 * np.max(np.abs(fd)), name


def test_compose_gradients_match_finite_differences_of_the_compose():
    # L(base, lora, g) = sum dy * (base + delta(base, lora, g)) with delta from the compose equation
    # (App. A item 1): grad_compose must return dL/dlora, dL/dbase and, through g = m / max(c, eps)
    # with c constant, dL/dm = (dL/dg) / max(c, eps).  A wrong factor (s missing, g-1 in place of g,
    # the wrong reduction axis) shows up here.
    rng = np.random.default_rng(11)
    T, n, s = 4, 5, 0.7
    dy = rng.standard_normal((T, n)); base = rng.standard_normal((T, n)); lora = rng.standard_normal((T, n))
    c = np.abs(rng.standard_normal(n)) + 1.0
    m = c * (1 + 1e-2 * rng.standard_normal(n))
    eps = 1e-12

    def loss():
        g = m / np.maximum(c, eps)
        return float(np.sum(dy * (base + O.compose_delta(base, lora, g, s))))

    g = m / np.maximum(c, eps)
    inner = s * lora + base
    d_lora, d_base, dm = O.grad_compose(dy, inner, g, c, s, eps)
    for name, arr, got in (("d_lora", lora, d_lora), ("d_base", base, d_base), ("dm", m, dm)):
        fd = _fd(loss, arr)
        assert np.max(np.abs(fd - got)) <= 1e-8 * np.max(np.abs(fd)), name
    # compose_delta itself against the printed equation, element by element
    j, t = 2, 1
    assert O.compose_delta(base, lora, g, s)[t, j] == pytest.approx(g[j] * (s * lora[t, j]) + (g[j] - 1) * base[t, j], rel=1e-14)


def test_compose_gradients_elementwise():
    # Sec. 3.2: d_lora = g s dy, d_base (via delta) = (g-1) dy; with y = base + delta, base gets g dy.
    rng = np.random.default_rng(10)
    dy = rng.standard_normal((3, 4)); inner = rng.standard_normal((3, 4))
    g = 1 + 1e-3 * rng.standard_normal(4); c = np.abs(rng.standard_normal(4)) + 1; s = 0.7
    d_lora, d_base, dm = O.grad_compose(dy, inner, g, c, s, 1e-12)
    np.testing.assert_allclose(d_lora, dy * g * s, rtol=1e-15)
    np.testing.assert_allclose(d_base, dy * g, rtol=1e-15)
    np.testing.assert_allclose(dm, (dy * inner).sum(0) / c, rtol=1e-15)


# ----------------------------------------------------------------------------- printed numbers

def test_table5_theory_column():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table5_theory_ratio.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 8
    for d_out, d_in, r, printed in rows:
        ratio = O.theory_memory_ratio(int(d_out), int(d_in), int(r))
        decimals = 0 if "." not in printed else 1
        assert round(ratio, decimals) == pytest.approx(float(printed), abs=0.051 if decimals else 0.5), (d_out, d_in, r, ratio)


def test_table1_concrete_numbers():
    vals = {}
    for l in open(os.path.join(GOLDEN, "table1_concrete.txt")):
        if l.strip() and l[0] != "#":
            k, v, _ = l.split()
            vals[k] = float(v)
    d, r = 8192, 512
    MiB = 2.0 ** 20
    assert 4 * d * d / MiB == vals["dense_BA"]
    assert round(4 * (d * r + r * r) / MiB, 1) == vals["U_plus_G"]
    assert round(O.theory_memory_ratio(d, d, r), 1) == vals["reduction"]
    assert O.chunk_size(256 * 2 ** 20, d, d) == vals["chunk_at_256MiB_d8192"]
    # the align-to-64 branch (App. B "Chunk alignment"), by hand: 256 MiB / (4 B x 27648 rows) = 2427.26 columns,
    # below d_in = 5120, so floor(2427 / 64) x 64 = 37 x 64 = 2368
    assert O.chunk_size(256 * 2 ** 20, 27648, 5120) == 2368
    assert O.chunk_size(256 * 2 ** 20, 27648, 2000) == 2000      # whole d_in fits: no alignment applied
    assert O.chunk_size(4 * 100 * 10, 100, 5120) == 64           # never below one aligned block
    assert 4 * r * r / MiB == vals["gram_bytes_r512"]


# ----------------------------------------------------------------------------- stability (Sec. 3.1, Fig. 1)

def _bf16(a):
    from paper_2603_22276_amd.inputs import f32_to_bf16_bits, bf16_bits_to_f32
    return bf16_bits_to_f32(f32_to_bf16_bits(np.asarray(a, np.float32))).astype(np.float64)


def test_stable_form_beats_naive_form_near_unity_g():
    # bf16 I/O, g = 1 + N(0, 0.0015): the stable form evaluated in fp32 and rounded once stays at the
    # bf16 floor of the *delta*; the naive form (g*(s*lora+base) - base with bf16 intermediates)
    # loses the correction.  The printed 3.0x is read off a figure and is not pinned; the ordering is.
    rng = np.random.default_rng(11)
    T, d_out = 64, 512
    base = _bf16(rng.standard_normal((T, d_out)))
    lora = _bf16(rng.standard_normal((T, d_out)) * 0.02)
    g = 1 + 0.0015 * rng.standard_normal(d_out)
    s = 1.633
    ref = O.compose_delta(base, lora, g, s)
    g32 = g.astype(np.float32)
    stable = _bf16(((g32 - 1)[None] * base.astype(np.float32) + g32[None] * (np.float32(s) * lora.astype(np.float32))))
    naive = _bf16(_bf16(_bf16(g)[None] * _bf16(s * lora + base)) - base)
    e_stable = np.max(np.abs(stable - ref))
    e_naive = np.max(np.abs(naive - ref))
    assert e_stable <= 2.0 ** -8 * np.max(np.abs(ref))  # within bf16 rounding of the result
    assert e_naive > 3 * e_stable


def test_bias_is_re_added_unscaled():
    # App. A item 2: the base layer's bias is subtracted before the compose and re-added after, so the module
    # output is x W'^T + bias with W' the adapted weight of Eq. (1) -- the bias is NOT multiplied by g.
    rng = np.random.default_rng(77)
    d_out, d_in, r, T = 12, 10, 3, 5
    W, A, B = rng.normal(size=(d_out, d_in)), rng.normal(size=(r, d_in)), rng.normal(size=(d_out, r))
    x, bias = rng.normal(size=(T, d_in)), rng.normal(size=d_out)
    m = np.abs(rng.normal(size=d_out)) + 0.5
    s, eps = 0.7, 1e-12
    f = O.forward(x, W, A, B, m, s, eps, bias=bias)
    Wp = O.adapted_weight(W, A, B, m, s, eps)
    np.testing.assert_allclose(f["y"], x @ Wp.T + bias[None, :], rtol=1e-12, atol=1e-12)
    g = f["g"]
    assert np.max(np.abs(g - 1.0)) > 0.05  # scaling the bias by g would be visible
    wrong = x @ Wp.T + (g * bias)[None, :]
    assert np.max(np.abs(f["y"] - wrong)) > 1e-3
    # inner is the bias-free pre-scale activation
    np.testing.assert_allclose(f["inner"], x @ (W + s * B @ A).T, rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------- LoRA dropout (App. B)

def test_dropout_forward_is_the_weight_delta_applied_to_the_dropped_input():
    # y = x W^T + x_d (W' - W)^T with W' from Eq. 1: the adapter sees the dropped input, the frozen
    # layer's output is that of x; with x_d = x this is the plain forward
    x, W, A, B, m, s, dy = small_problem(20, T=6, d_out=7, d_in=8, r=3, s=0.9)
    rng = np.random.default_rng(21)
    x_d = x * (rng.random(x.shape) >= 0.25) / 0.75
    f = O.forward(x, W, A, B, m, s, 1e-12, x_lora=x_d)
    Wp = O.adapted_weight(W, A, B, m, s, 1e-12)
    np.testing.assert_allclose(f["y"], x @ W.T + x_d @ (Wp - W).T, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(f["delta"], x_d @ (Wp - W).T, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(f["inner"], x_d @ (W + s * B @ A).T, rtol=1e-12, atol=1e-13)
    plain = O.forward(x, W, A, B, m, s, 1e-12)
    same = O.forward(x, W, A, B, m, s, 1e-12, x_lora=x.copy())
    for k in ("y", "delta", "inner", "h"):
        np.testing.assert_allclose(same[k], plain[k], rtol=1e-13, atol=1e-14)


def test_dropout_gradients_match_finite_differences():
    x, W, A, B, m, s, dy = small_problem(22, T=4, d_out=5, d_in=6, r=3, s=1.1)
    rng = np.random.default_rng(23)
    x_d = x * (rng.random(x.shape) >= 0.3) / 0.7
    c0 = O.dense_row_norm(W, A, B, s)

    def loss():
        return float(np.sum(dy * O.forward(x, W, A, B, m, s, 1e-12, c=c0, x_lora=x_d)["y"]))

    b = O.backward_dropout(dy, x, x_d, W, A, B, m, s, 1e-12)
    for name, arr in (("dx", x), ("dx_lora", x_d), ("dA", A), ("dB", B), ("dm", m)):
        fd = _fd(loss, arr)
        assert np.max(np.abs(fd - b[name])) <= 1e-7 * np.max(np.abs(fd)), name
    # without dropout the two input gradients add up to the plain module's dx
    b0 = O.backward_dropout(dy, x, x, W, A, B, m, s, 1e-12)
    plain = O.backward(dy, x, W, A, B, m, s, 1e-12)
    np.testing.assert_allclose(b0["dx"] + b0["dx_lora"], plain["dx"], rtol=1e-12, atol=1e-13)
    for k in ("dA", "dB", "dm"):
        np.testing.assert_allclose(b0[k], plain[k], rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- fp16 storage (App. B "Dtype-aware epsilon")

def test_fp16_storage_rounding_epsilon_and_saturation():
    from paper_2603_22276_amd import inputs as I
    q = lambda v: float(I.quantise(np.array([v], np.float64), "f16")[0])
    # IEEE binary16, ties to even: 1 + 2^-11 is halfway between 1 and 1 + 2^-10
    assert q(1 + 2.0 ** -11) == 1.0 and q(1 + 3 * 2.0 ** -11) == 1 + 2.0 ** -9
    assert q(65504.0) == 65504.0 and q(65519.0) == 65504.0 and np.isinf(q(65520.0))   # largest finite value
    assert q(2.0 ** -24) == 2.0 ** -24 and q(2.0 ** -26) == 0.0                        # subnormals kept, then zero
    cfg = I.DoraConfig("h", 8, 16, 8, 4, "f16", 32.0, 1e-3)
    assert cfg.eps == 1e-6                                                             # same guard as bf16
    a = I.make_inputs(cfg)
    assert a["W"].dtype == np.float16 and a["x"].dtype == np.float16 and a["m"].dtype == np.float32
    assert np.array_equal(I.to_f64(a["W"]), a["W"].astype(np.float64))
    # with eps = 1e-6 a vanishing row gives g = m / eps ~ 1e6 m: beyond fp16's range, which is why g (and the
    # norm) are carried in fp32; in fp16 the quotient would already be infinite for m = 1
    g = O.mag_scale(np.array([1.0, 0.05]), np.array([0.0, 0.0]), cfg.eps)
    np.testing.assert_allclose(g, [1e6, 5e4], rtol=1e-12)
    with np.errstate(over="ignore"):
        assert np.isinf(np.float16(g[0])) and np.isfinite(np.float16(g[1]))
    assert np.isfinite(np.float32(g[0]))


def test_fp16_compose_needs_fp32_arithmetic_near_unity_g():
    # Sec. 3.1: evaluated in fp16, (g - 1) (.) base vanishes whenever |g - 1| < 2^-11 (g rounds to 1);
    # fp32 arithmetic with one rounding at the store keeps the correction
    rng = np.random.default_rng(12)
    f16 = lambda a: np.asarray(a, np.float32).astype(np.float16).astype(np.float64)
    base = f16(rng.standard_normal((32, 256)))
    lora = f16(rng.standard_normal((32, 256)) * 0.02)
    g = 1 + 0.0015 * rng.standard_normal(256)
    s = 1.633
    exact = O.compose_delta(base, lora, g, s)
    collapse = (g - 1 < 2.0 ** -11) & (g - 1 > -(2.0 ** -12))   # fp16 spacing is 2^-10 above 1 and 2^-11 below
    assert 0.1 < collapse.mean() < 0.4          # a sizeable share of the rows, as the paper observes for fp16
    g16 = f16(g)
    in_fp16 = f16(f16((g16 - 1.0)[None, :] * base) + f16(g16[None, :] * f16(s * lora)))
    in_fp32 = f16(np.float32(g - 1)[None, :].astype(np.float64) * base + np.float32(g)[None, :].astype(np.float64) * (s * lora))
    assert np.all((g16 - 1.0)[collapse] == 0.0)
    err16 = np.max(np.abs(in_fp16 - exact)[:, collapse])
    err32 = np.max(np.abs(in_fp32 - exact)[:, collapse])
    assert err32 < 0.2 * err16
