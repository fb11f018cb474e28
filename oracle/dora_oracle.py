"""CPU oracle for the DoRA module hot path (float64, numpy).

TEST INFRASTRUCTURE ONLY.  This file is the slow, literal statement of what the
HIP library must compute.  Only the tests, the smoke entry and the bench's
`cpu_baseline` leg may call it; the product path never does.  It shares no code,
table or helper with the HIP path and imports nothing from it.

Every function takes float64 arrays (the callers widen the stored, already
rounded bf16/fp32 inputs exactly) and returns float64.

What is defined here, and from where:

* `composed_weight`, `dense_row_norm`  - Eq. (1): the row norm of W + s B A,
  written out by forming the dense [d_out, d_in] matrix.  This is the plain
  definition that the factored form of Sec. 2 reaches up to rounding order.
* `mag_scale`                          - Eq. (6): g = m / max(w_norm, eps).
* `adapted_weight`                     - Eq. (1): W' = m * (W + sBA) / ||.||_row.
* `forward`                            - App. A item 1 (compose equation) with
  base = x W^T, lora = (x A^T) B^T, inner = s*lora + base (Sec. 4, Tier 1),
  delta = (g-1)*base + g*(s*lora), Y = base + delta.
* `backward` / `grad_*`                - Sec. 3.2 and App. C item 2: gradients of
  the compose, chained through the three linear maps, with the norm held
  constant (Sec. 2.2 last paragraph; App. A item 2 "detached").
* `forward(x_lora=...)`, `backward_dropout` - the same with a separate input for the
  adapter branch (LoRA dropout, App. B "Chunked dropout path").
* `factored_norm_terms`, `assemble_norm` - the terms of Eq. (2), each from its
  definition (Eq. 3, Eq. 4), and the assembly of Eq. (5).  Not used to judge the
  HIP norm (the dense definition is); kept so the three terms can be checked one
  by one and so the identity itself is pinned against the dense form.

Pins (tests/test_oracle_pins.py): B=0 / s=0 special cases, the r=1 closed form,
orthonormal-A and W=0 cases, homogeneity, Cauchy-Schwarz on the cross term,
Y == x W'^T through Eq. (1), hand-worked 2x2 values, central finite differences
for every gradient (and the negative control with the norm re-evaluated), and a
loop-by-loop C transcription of the same definitions (oracle/literal.c).
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

F64 = np.float64


def _f64(a) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype != F64:
        raise TypeError("oracle functions take float64 arrays; widen the stored inputs first")
    return a


# --------------------------------------------------------------------------- norm (Eq. 1)

def composed_weight(W, A, B, s) -> np.ndarray:
    """D = W + s * (B @ A), the dense [d_out, d_in] composed weight of Eq. (1)."""
    W, A, B = _f64(W), _f64(A), _f64(B)
    return W + F64(s) * (B @ A)


def dense_row_norm(W, A, B, s) -> np.ndarray:
    """c[j] = sqrt(sum_k D[j,k]^2): the denominator of Eq. (1), one value per output row."""
    D = composed_weight(W, A, B, s)
    return np.sqrt(np.sum(D * D, axis=1))


def mag_scale(m, c, eps) -> np.ndarray:
    """Eq. (6): g = m / max(c, eps)."""
    return _f64(m) / np.maximum(_f64(c), F64(eps))


def adapted_weight(W, A, B, m, s, eps) -> np.ndarray:
    """Eq. (1): W' = m (.) (W + sBA) / ||W + sBA||_row (with the eps guard of Eq. 6)."""
    D = composed_weight(W, A, B, s)
    c = np.sqrt(np.sum(D * D, axis=1))
    return mag_scale(m, c, eps)[:, None] * D


# --------------------------------------------------------------------------- forward

def forward(x, W, A, B, m, s, eps, c: Optional[np.ndarray] = None,
            bias: Optional[np.ndarray] = None, x_lora: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Whole forward of one module.

    base  = x W^T                  [T, d_out]   (what the frozen layer produces)
    xa    = x_lora if given else x              (the adapter's input)
    base_a = xa W^T, h = xa A^T [T, r], lora = h B^T [T, d_out]
    inner = s*lora + base_a        (the tensor Tier 1 saves for backward)
    delta = (g-1)*base_a + g*(s*lora)   (compose equation, App. A item 1) = xa (W' - W)^T
    y     = base + delta           (what the caller of the module ends up with)

    x_lora (App. B "Chunked dropout path"): with LoRA dropout active the adapter sees the dropped
    input while the frozen layer's output stays that of x, so the base the compose runs on is
    recomputed for the dropped input; without dropout base_a is base.

    bias (App. A item 2): the frozen layer's bias is taken off its output before the
    compose and put back afterwards, i.e. it is not scaled by g: y = base + delta + bias
    with base the bias-free x W^T.
    """
    x, W, A, B, m = _f64(x), _f64(W), _f64(A), _f64(B), _f64(m)
    s = F64(s)
    if c is None:
        c = dense_row_norm(W, A, B, s)
    g = mag_scale(m, c, eps)
    base = x @ W.T
    xa = x if x_lora is None else _f64(x_lora)
    base_a = base if x_lora is None else xa @ W.T
    h = xa @ A.T
    lora = h @ B.T
    inner = s * lora + base_a
    delta = (g - 1.0)[None, :] * base_a + g[None, :] * (s * lora)
    y = base + delta
    if bias is not None:
        y = y + _f64(bias)[None, :]
    return {"c": c, "g": g, "base": base, "base_a": base_a, "h": h, "lora": lora, "inner": inner, "delta": delta,
            "y": y}


def compose_delta(base, lora, g, s) -> np.ndarray:
    """App. C item 1: delta = (g-1) (.) base + g (.) s (.) lora, g broadcast along the last axis."""
    base, lora, g = _f64(base), _f64(lora), _f64(g)
    return (g - 1.0)[None, :] * base + g[None, :] * (F64(s) * lora)


# --------------------------------------------------------------------------- backward (norm detached)

def grad_compose(dy, inner, g, c, s, eps):
    """Sec. 3.2 / App. C item 2, for upstream gradient dy of y = base + delta.

    d_lora = g*s*dy ; d_base (through delta) = (g-1)*dy, plus the identity path
    of y = base + delta gives dy, so base receives g*dy in total;
    d_mag[j] = sum_t dy[t,j]*inner[t,j] is the gradient w.r.t. g, and since
    g = m / max(c, eps) with c constant, dm = d_mag / max(c, eps).
    """
    dy, inner, g, c = _f64(dy), _f64(inner), _f64(g), _f64(c)
    d_lora = g[None, :] * F64(s) * dy
    d_base_total = dy + (g - 1.0)[None, :] * dy
    d_mag = np.sum(dy * inner, axis=0)
    dm = d_mag / np.maximum(c, F64(eps))
    return d_lora, d_base_total, dm


def grad_m(dy, x, W, A, B, m, s, eps, c=None) -> np.ndarray:
    f = forward(x, W, A, B, m, s, eps, c)
    return grad_compose(_f64(dy), f["inner"], f["g"], f["c"], s, eps)[2]


def grad_B(dy, x, W, A, B, m, s, eps, c=None) -> np.ndarray:
    """lora = h B^T  =>  dB = d_lora^T h, with h = x A^T."""
    x, W, A, B, m, dy = _f64(x), _f64(W), _f64(A), _f64(B), _f64(m), _f64(dy)
    if c is None:
        c = dense_row_norm(W, A, B, s)
    g = mag_scale(m, c, eps)
    d_lora = g[None, :] * F64(s) * dy
    h = x @ A.T
    return d_lora.T @ h


def grad_A(dy, x, W, A, B, m, s, eps, c=None) -> np.ndarray:
    """h = x A^T, lora = h B^T  =>  dh = d_lora B, dA = dh^T x."""
    x, W, A, B, m, dy = _f64(x), _f64(W), _f64(A), _f64(B), _f64(m), _f64(dy)
    if c is None:
        c = dense_row_norm(W, A, B, s)
    g = mag_scale(m, c, eps)
    d_lora = g[None, :] * F64(s) * dy
    dh = d_lora @ B
    return dh.T @ x


def grad_x(dy, x, W, A, B, m, s, eps, c=None) -> np.ndarray:
    """base = x W^T and h = x A^T both depend on x: dx = d_base W + dh A."""
    x, W, A, B, m, dy = _f64(x), _f64(W), _f64(A), _f64(B), _f64(m), _f64(dy)
    if c is None:
        c = dense_row_norm(W, A, B, s)
    g = mag_scale(m, c, eps)
    d_lora = g[None, :] * F64(s) * dy
    d_base = dy + (g - 1.0)[None, :] * dy
    dh = d_lora @ B
    return d_base @ W + dh @ A


def backward(dy, x, W, A, B, m, s, eps, c=None) -> Dict[str, np.ndarray]:
    """All four gradients (W is frozen and gets none)."""
    if c is None:
        c = dense_row_norm(_f64(W), _f64(A), _f64(B), s)
    return {
        "dx": grad_x(dy, x, W, A, B, m, s, eps, c),
        "dA": grad_A(dy, x, W, A, B, m, s, eps, c),
        "dB": grad_B(dy, x, W, A, B, m, s, eps, c),
        "dm": grad_m(dy, x, W, A, B, m, s, eps, c),
    }


def backward_dropout(dy, x, x_lora, W, A, B, m, s, eps, c=None) -> Dict[str, np.ndarray]:
    """Gradients of y = x W^T + delta(x_lora) (the forward with a separate adapter input), norm constant.

    The frozen path gives dx = dy W.  The adapter path: base_a = x_lora W^T receives (g-1) dy and
    lora receives g s dy, so dx_lora = ((g-1) dy) W + dh A with dh = (g s dy) B; dA = dh^T x_lora;
    dB = (g s dy)^T h with h = x_lora A^T; dm = (sum_t dy * inner) / max(c, eps) with
    inner = s lora + base_a.
    """
    dy, x, xa, W, A, B, m = _f64(dy), _f64(x), _f64(x_lora), _f64(W), _f64(A), _f64(B), _f64(m)
    if c is None:
        c = dense_row_norm(W, A, B, s)
    g = mag_scale(m, c, eps)
    d_lora = g[None, :] * F64(s) * dy
    d_base_a = (g - 1.0)[None, :] * dy
    h = xa @ A.T
    dh = d_lora @ B
    inner = F64(s) * (h @ B.T) + xa @ W.T
    return {
        "dx": dy @ W,
        "dx_lora": d_base_a @ W + dh @ A,
        "dA": dh.T @ xa,
        "dB": d_lora.T @ h,
        "dm": np.sum(dy * inner, axis=0) / np.maximum(_f64(c), F64(eps)),
    }


# --------------------------------------------------------------------------- Algorithm 1 (factored form)

def factored_norm_terms(W, A, B, cols=None) -> Dict[str, np.ndarray]:
    """The terms of Eq. (2), each written from its own definition (Eq. 3, Eq. 4):

      base_sq[j] = ||W_j||^2                      = sum_k W[j,k]^2
      cross[j]   = <W_j, (B A)_j>                 = sum_l B[j,l] (W A^T)[j,l]         (Eq. 3)
      G          = A A^T                                                              (Eq. 4)
      ba_sq[j]   = ||(B A)_j||^2 = B_j G B_j^T    = sum_l sum_p B[j,l] G[l,p] B[j,p]

    `cols` restricts W and A to a subset of the d_in columns.  Every term is a sum over columns (ba_sq
    is linear in G), so the values over the blocks of any partition of d_in add up to the values over
    all columns: the property Algorithm 1's chunk loop rests on.
    """
    W, A, B = _f64(W), _f64(A), _f64(B)
    if cols is not None:
        W, A = W[:, cols], A[:, cols]
    base_sq = np.einsum("jk,jk->j", W, W)
    U = W @ A.T                                   # [d_out, r]
    cross = np.einsum("jl,jl->j", B, U)
    G = A @ A.T                                   # [r, r]
    ba_sq = np.einsum("jl,lp,jp->j", B, G, B)
    return {"base_sq": base_sq, "cross": cross, "G": G, "ba_sq": ba_sq}


def assemble_norm(base_sq, cross, ba_sq, s) -> np.ndarray:
    """Eq. (5): sqrt(max(base_sq + 2s*cross + s^2*ba_sq, 0)); a NaN radicand stays NaN."""
    s = F64(s)
    rad = _f64(base_sq) + (2.0 * s) * _f64(cross) + (s * s) * _f64(ba_sq)
    rad = np.where(rad < 0.0, 0.0, rad)  # NaN < 0 is False, so NaN passes through
    return np.sqrt(rad)


def factored_row_norm(W, A, B, s, chunk: Optional[int] = None) -> np.ndarray:
    """Eq. (5) from the factored terms; with `chunk`, the column sums are accumulated block by block
    over d_in (Algorithm 1's memory-bounded schedule) and ba_sq comes from the accumulated G."""
    if F64(s) == 0.0:  # scale-is-zero fast path of Algorithm 1's notes
        W = _f64(W)
        return np.sqrt(np.sum(W * W, axis=1))
    if chunk is None:
        t = factored_norm_terms(W, A, B)
        return assemble_norm(t["base_sq"], t["cross"], t["ba_sq"], s)
    B = _f64(B)
    d_in = _f64(W).shape[1]
    blocks = [factored_norm_terms(W, A, B, slice(c0, c0 + int(chunk))) for c0 in range(0, d_in, int(chunk))]
    base_sq = sum(b["base_sq"] for b in blocks)
    cross = sum(b["cross"] for b in blocks)
    G = sum(b["G"] for b in blocks)
    ba_sq = np.einsum("jl,lp,jp->j", B, G, B)
    return assemble_norm(base_sq, cross, ba_sq, s)


def chunk_size(budget_bytes: int, d_out: int, d_in: int) -> int:
    """Algorithm 1's chunk rule: min(d_in, floor(budget / (4 d_out))) aligned down to 64."""
    cs = min(d_in, budget_bytes // (4 * d_out))
    if cs < d_in:
        cs = max(64, (cs // 64) * 64)
    return int(cs)


def theory_memory_ratio(d_out: int, d_in: int, r: int) -> float:
    """Table 1 / Table 5 'theory' column: dense [d_out,d_in] over U[d_out,r] + G[r,r]."""
    return (d_out * d_in) / float(d_out * r + r * r)
