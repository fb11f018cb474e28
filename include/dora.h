/*
 * libdora - the DoRA adapter hot path on one MI355X (gfx950), C ABI.
 *
 * One adapted linear module:  W [d_out, d_in] frozen, A [r, d_in], B [d_out, r],
 * magnitude m [d_out], scaling s; activations x [tokens, d_in]  (Sec. 1, Eq. 1).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  Row-major,
 *     contiguous, 16-byte aligned.  Inputs are const and never modified.
 *   - `dtype` selects the storage type of W, A, B, x, y, dy, dx, saved_h,
 *     saved_inner, base, lora: DORA_BF16 (bfloat16), DORA_F16 (IEEE binary16) or
 *     DORA_F32.  Accumulation is always fp32.  w_norm, m, g, gm1, dm, dA, dB are
 *     fp32 for every dtype.  DORA_F16 (App. B "Dtype-aware epsilon"): eps defaults
 *     to 1e-6 as for bf16; a value beyond 65504 in magnitude becomes an infinity
 *     when it is stored (IEEE conversion, no clamping), which is why g and the norm
 *     are never held in fp16.
 *   - Shape limits: d_out, d_in, r multiples of 8 (bf16, fp16) or of 4 (fp32);
 *     tokens >= 0 (0 is a no-op that still
 *     computes weight-only results); every tensor below 2^31 elements.
 *   - `ws` is caller-provided scratch of at least dora_workspace_bytes(desc,
 *     phase) bytes, 256-byte aligned.  The library allocates no device memory,
 *     keeps no state between calls, enqueues everything on `stream` (a
 *     hipStream_t passed as void*; NULL is the default stream) and returns
 *     without synchronising.  Results are deterministic run to run (no
 *     floating-point atomics anywhere).  (The measurement hooks declared in
 *     dora_measure.h are the one exception: they keep process-global timing
 *     records and are not part of the method.)
 *   - Errors are returned, never thrown; on error nothing has been enqueued
 *     unless the status is DORA_ERR_HIP.
 */
#ifndef DORA_H
#define DORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DORA_F32 = 0, DORA_BF16 = 1, DORA_F16 = 2 } dora_dtype;

typedef enum {
    DORA_OK = 0,
    DORA_ERR_NULL = 1,      /* a required pointer is NULL */
    DORA_ERR_SHAPE = 2,     /* a dimension is negative, too large or violates the multiple-of rule */
    DORA_ERR_ALIGN = 3,     /* a pointer is not 16-byte aligned (ws: 256) */
    DORA_ERR_DTYPE = 4,     /* unknown dtype */
    DORA_ERR_WORKSPACE = 5, /* ws_bytes < dora_workspace_bytes */
    DORA_ERR_HIP = 6        /* a HIP runtime call failed (launch error) */
} dora_status;

typedef struct {
    int64_t d_out, d_in, r, tokens;
    int32_t dtype; /* dora_dtype */
    float s;       /* LoRA scaling, e.g. rsLoRA alpha / sqrt(r) */
    float eps;     /* guard of Eq. 6; <= 0 selects the default of App. A item 2: 1e-12 (F32), 1e-6 (BF16, F16) */
} dora_desc;

typedef enum {
    DORA_PHASE_NORM = 0,              /* dora_norm */
    DORA_PHASE_FORWARD = 1,           /* dora_forward with w_norm == NULL and saved_inner == NULL (worst case) */
    DORA_PHASE_BACKWARD = 2,          /* dora_backward with saved_h / saved_inner given */
    DORA_PHASE_BACKWARD_RECOMPUTE = 3,/* dora_backward with saved_* == NULL (recomputes h and inner) */
    DORA_PHASE_COMPOSE_BACKWARD = 4,  /* dora_compose_backward */
    DORA_PHASE_FORWARD_DROPOUT = 5,   /* dora_forward_dropout, worst case as for DORA_PHASE_FORWARD */
    DORA_PHASE_BACKWARD_DROPOUT = 6   /* dora_backward_dropout with everything recomputed (worst case) */
} dora_phase;

/* Scratch bytes an entry point needs for this shape.  Returns 0 for an invalid desc. */
size_t dora_workspace_bytes(const dora_desc* desc, int phase);

/*
 * Row-wise norm of the composed weight, w_norm[j] = || W[j,:] + s (B A)[j,:] ||_2, by the
 * factored form of Sec. 2 (Eq. 2-5, Algorithm 1): base_sq + 2s*cross + s^2*ba_sq, with
 * U = W A^T and G = A A^T accumulated in fp32 and never written as dense [d_out, d_in]
 * data.  s == 0 skips the cross and Gram terms (Algorithm 1, notes).  Negative radicands
 * clamp to 0, NaN propagates (App. C item 3).
 *   W, A, B : device, const, `dtype`.   w_norm : device, out, fp32 [d_out].
 */
dora_status dora_norm(const dora_desc* desc, const void* W, const void* A, const void* B,
                      float* w_norm, void* ws, size_t ws_bytes, void* stream);

/*
 * dora_norm for callers that cannot allocate or size a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same result as dora_norm, bit for bit, with
 * the scratch taken from a fixed array inside the library instead of `ws`.  Calls no hipMalloc,
 * hipFree or other allocating routine.
 *   - The array is dora_norm_static_max_bytes() = 16 MiB of device memory per GPU the library runs
 *     on, held until the process ends.  A shape whose dora_workspace_bytes(desc, DORA_PHASE_NORM)
 *     exceeds it is rejected with DORA_ERR_WORKSPACE before anything is enqueued (the workload
 *     shapes fit at every rank up to 768; r = 2048 at d_out = 8192 does not).
 *   - All calls on one GPU share that one array: two calls that overlap in time on the same GPU (two
 *     streams, two threads) race.  Calls ordered on one stream are safe; nothing needs clearing between
 *     them because each launch overwrites in full what the next one reads.
 *   - The first call on a device looks up the array's address there (host-side, thread-safe).
 */
size_t dora_norm_static_max_bytes(void);
dora_status dora_norm_static(const dora_desc* desc, const void* W, const void* A, const void* B,
                             float* w_norm, void* stream);

/*
 * Cached base term (Sec. 2.3: W is frozen, so the rank-independent term of Eq. 2 can be
 * computed once and kept in a [d_out] buffer).
 *   dora_base_sq     : base_sq[j] = sum_k W[j,k]^2, fp32 accumulation of the exact products.
 *                      W : device, const, `dtype` [d_out, d_in].  base_sq : device, out, fp32 [d_out].
 *                      Needs no workspace; desc->r and desc->tokens are not read.
 *   dora_norm_cached : dora_norm with that buffer as the base term: W is read once (for the cross
 *                      term) and never squared.  Same workspace, outputs and error behaviour as
 *                      dora_norm; the caller owns base_sq and must recompute it if W changes.
 */
dora_status dora_base_sq(const dora_desc* desc, const void* W, float* base_sq, void* stream);
dora_status dora_norm_cached(const dora_desc* desc, const float* base_sq, const void* W, const void* A,
                             const void* B, float* w_norm, void* ws, size_t ws_bytes, void* stream);

/*
 * The factored terms on their own, for reuse while A and B are unchanged (Sec. 2.3 leaves caching as future
 * work; within one training step the forward and the recomputed forward of a checkpointed backward see the
 * same W, A, B, so the second can reuse what the first computed).  Nothing is cached inside the library:
 * the caller owns the buffers and decides when they are stale.
 *   dora_norm_terms    : terms [3, d_out] fp32 out = base_sq | cross | ba_sq (Eq. 2-4), each row the
 *                        fixed-order sum of the split-K partials; G [r, r] fp32 out or NULL (Eq. 4).
 *                        s == 0: cross = ba_sq = 0, G = 0 (Algorithm 1, notes).  Workspace as for dora_norm.
 *   dora_norm_assemble : w_norm = sqrt(max(base_sq + 2 s cross + s^2 ba_sq, 0)) (Eq. 5) from such terms, with
 *                        desc->s: one small launch, bit-identical to what dora_norm returns for the same
 *                        inputs.  d_in, r, tokens of desc are not read.  Needs no workspace.
 * dora_norm(...) == dora_norm_terms(...) followed by dora_norm_assemble(...).  The default of every other
 * entry point is unchanged: the norm is recomputed unless the caller passes w_norm (App. A item 2).
 */
dora_status dora_norm_terms(const dora_desc* desc, const void* W, const void* A, const void* B,
                            float* terms, float* G, void* ws, size_t ws_bytes, void* stream);
dora_status dora_norm_assemble(const dora_desc* desc, const float* terms, float* w_norm, void* stream);

/*
 * Magnitude scale of Eq. 6: g = m / max(w_norm, eps), and the explicit small
 * correction gm1 = g - 1 of Sec. 3.1, formed as (m - cc)/cc with cc = max(w_norm, eps)
 * so that it does not suffer the rounding of g.  g or gm1 may be NULL (not both).
 */
dora_status dora_mag_scale(const dora_desc* desc, const float* m, const float* w_norm,
                           float* g, float* gm1, void* stream);

/*
 * Compose pass of Sec. 3.1 / App. C item 1 on existing activations:
 *   delta = gm1 (.) base + g (.) (s * lora)         (fp32 arithmetic, one rounding at the store)
 *   out   = write_delta ? delta : base + delta
 *   inner = s * lora + base                          (only if inner != NULL; Sec. 4, Tier 1)
 * base, lora : device, const, `dtype`, [tokens, d_out].  g : fp32 [d_out].  gm1 : fp32 [d_out]
 * or NULL (then g - 1 is formed in fp32).  out / inner : device, `dtype`, [tokens, d_out];
 * out may alias base and inner may alias lora (element-wise in place); other overlaps are
 * not allowed.  Needs no workspace.  d_in and r of desc are ignored.
 */
dora_status dora_compose(const dora_desc* desc, const void* base, const void* lora,
                         const float* g, const float* gm1,
                         void* out, int write_delta, void* inner, void* stream);

/*
 * Backward of the compose (Sec. 3.2, App. C item 2), for the upstream gradient dy of
 * y = base + delta:
 *   dz = g (.) dy      (gradient reaching base; the gradient reaching lora is s * dz)
 *   dm[j] = ( sum_t dy[t,j] * inner[t,j] ) / max(w_norm[j], eps)
 * The column sum is a two-stage, fixed-order reduction fused into the same pass (Sec. 7,
 * "LLM-guided optimization"), no atomics.  dm == NULL (frozen magnitude) skips it and then
 * inner and w_norm may be NULL.   dy, inner : const `dtype` [tokens, d_out];  dz : `dtype`.
 */
dora_status dora_compose_backward(const dora_desc* desc, const void* dy, const void* inner,
                                  const float* g, const float* w_norm,
                                  void* dz, float* dm, void* ws, size_t ws_bytes, void* stream);

/*
 * The three forward contractions on their own (App. A item 1): base = x W^T [tokens, d_out],
 * h = x A^T [tokens, r], lora = h B^T [tokens, d_out], each rounded once to `dtype`.
 * The launches dora_forward makes for these steps, except that without a workspace h = x A^T is never
 * split along K (dora_forward splits it when its tiles would leave most of the chip idle).  Needs no workspace.
 */
dora_status dora_project(const dora_desc* desc, const void* x, const void* W, const void* A, const void* B,
                         void* base, void* h, void* lora, void* stream);

/*
 * Whole forward of the module (App. A item 1): norm (unless w_norm is given), g,
 * base = x W^T, h = x A^T, lora = h B^T, compose;  y = base + delta = g (.) (base + s*lora).
 *   x [tokens, d_in], W, A, B : const `dtype`.   m : const fp32 [d_out].
 *   w_norm : const fp32 [d_out] or NULL (NULL: computed here into the workspace).
 *   bias : const `dtype` [d_out] or NULL: bias of the frozen base layer.  It takes no part in the
 *          compose (App. A item 2: subtracted before, re-added after), so it is added last:
 *          y = base + delta + bias; inner and the backward are unaffected.
 *   y : out `dtype` [tokens, d_out].
 *   saved_h : out `dtype` [tokens, r] or NULL.   saved_inner : out `dtype` [tokens, d_out] or NULL.
 *   w_norm_out : out fp32 [d_out] or NULL (receives the norm used, for the backward call).
 */
dora_status dora_forward(const dora_desc* desc, const void* x, const void* W, const void* A,
                         const void* B, const float* m, const float* w_norm, const void* bias,
                         void* y, void* saved_h, void* saved_inner, float* w_norm_out,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * Same result as dora_forward, computed without the base / lora round trip: one K-concatenated
 * contraction  inner = [s*h | x] [B | W]^T  (the h = x A^T product writes both h and s*h from its
 * accumulators) whose epilogue writes y = g (.) inner (+ bias) and, if asked, inner.
 * The cancellation issue of Sec. 3.1 concerns the *delta* form only; g (.) inner taken from an fp32
 * accumulator has none.  DORA_BF16 and DORA_F16 descs only (DORA_ERR_DTYPE otherwise).  Arguments, workspace
 * (DORA_PHASE_FORWARD) and saved tensors exactly as for dora_forward.
 */
dora_status dora_forward_fused(const dora_desc* desc, const void* x, const void* W, const void* A,
                               const void* B, const float* m, const float* w_norm, const void* bias,
                               void* y, void* saved_h, void* saved_inner, float* w_norm_out,
                               void* ws, size_t ws_bytes, void* stream);

/*
 * Backward of the module with the norm held constant (Sec. 2.2; App. A item 2) and W frozen:
 *   dz = g (.) dy;  dh = s * dz B;  dx = dz W + dh A;  dA = dh^T x;  dB = s * dz^T h;
 *   dm as in dora_compose_backward.
 *   dy [tokens, d_out], x, W, A, B : const `dtype`.  m : const fp32.
 *   w_norm : const fp32 [d_out] or NULL (NULL: recomputed).
 *   saved_h / saved_inner : const `dtype` as written by dora_forward, or NULL (recomputed
 *   here - the gradient-checkpointing pattern).
 *   dx : out `dtype` [tokens, d_in].  dA : out fp32 [r, d_in].  dB : out fp32 [d_out, r].
 *   dm : out fp32 [d_out] or NULL (frozen magnitude).  Any of dx, dA, dB may be NULL to skip it.
 */
dora_status dora_backward(const dora_desc* desc, const void* dy, const void* x, const void* W,
                          const void* A, const void* B, const float* m, const float* w_norm,
                          const void* saved_h, const void* saved_inner,
                          void* dx, float* dA, float* dB, float* dm,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * The module under LoRA dropout (App. B "Chunked dropout path"): the adapter branch sees its own input
 * x_lora = dropout(x), formed by the caller (device, const, `dtype` [tokens, d_in]; the library draws no
 * random numbers), while the frozen layer's output stays that of x.  The compose then runs on the adapter
 * branch's own base:
 *   y = x W^T + delta,   delta = (g-1) (.) (x_lora W^T) + g (.) (s * (x_lora A^T) B^T)  [+ bias]
 * i.e. delta = x_lora (W' - W)^T with W' the adapted weight of Eq. 1; h and inner are those of x_lora.
 * (The paper bounds the memory of the second base by walking d_out in slices; here it is one
 * [tokens, d_out] scratch tensor inside the workspace, DORA_PHASE_FORWARD_DROPOUT.)
 * Backward, norm constant:  dx = dy W (frozen path),  dx_lora = ((g-1) (.) dy) W + dh A,  dh = s (g (.) dy) B,
 * dA = dh^T x_lora,  dB = s (g (.) dy)^T h,  dm = (sum_t dy * inner) / max(w_norm, eps); the caller applies
 * its dropout mask to dx_lora and adds it to dx.  dx, dx_lora, dA, dB, dm may each be NULL.  saved_h /
 * saved_inner as written by dora_forward_dropout, or NULL (recomputed from x_lora).  With x_lora == x the
 * results are those of dora_forward / dora_backward (dx + dx_lora = dx of the plain module).
 */
dora_status dora_forward_dropout(const dora_desc* desc, const void* x, const void* x_lora, const void* W,
                                 const void* A, const void* B, const float* m, const float* w_norm,
                                 const void* bias, void* y, void* saved_h, void* saved_inner, float* w_norm_out,
                                 void* ws, size_t ws_bytes, void* stream);
dora_status dora_backward_dropout(const dora_desc* desc, const void* dy, const void* x_lora, const void* W,
                                  const void* A, const void* B, const float* m, const float* w_norm,
                                  const void* saved_h, const void* saved_inner, void* dx, void* dx_lora,
                                  float* dA, float* dB, float* dm, void* ws, size_t ws_bytes, void* stream);

const char* dora_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif /* DORA_H */
