/*
 * libdora - measurement hooks (NOT part of the method; nothing here is needed to use the library).
 *
 * Per-kernel timing and two probe kernels for benchmark harnesses.  Unlike the entry points of
 * dora.h these calls keep process-global mutable state (an event pool and per-kernel totals) and
 * are not thread-safe: use them from one thread, around calls made from that thread.
 */
#ifndef DORA_MEASURE_H
#define DORA_MEASURE_H

#include "dora.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-kernel timing for measurement harnesses (not part of the method).  While enabled, every
 * kernel launch made by the entry points of dora.h is bracketed by a pair of HIP events recorded on
 * the launch stream.  dora_trace_collect synchronises those events and adds each launch's
 * duration to its kernel's slot; dora_trace_get reads one slot.  Kernel ids are the
 * DORA_K_* values; dora_trace_name returns a short label.  Enabling tracing creates host-side
 * event objects only (no device memory).  dora_trace_select restricts the bracketing to some kernel ids, so
 * that a throughput measurement can carry the events of its dominant kernel only.  Not thread-safe.
 */
enum {
    DORA_K_NORM_CROSS = 0,   /* U = W A^T tile + base_sq + rowdot(B, U) partials      */
    DORA_K_GRAM = 1,         /* G = A A^T split-K partials                             */
    DORA_K_GRAM_REDUCE = 2,  /* fixed-order sum of Gram partials, hi/lo split          */
    DORA_K_BA_SQ = 3,        /* rowdot(B, B G) partials                                */
    DORA_K_NORM_FINAL = 4,   /* Eq. 5 assembly                                         */
    DORA_K_MAG_SCALE = 5,    /* Eq. 6                                                  */
    DORA_K_GEMM_BASE = 6,    /* base = x W^T                                           */
    DORA_K_GEMM_H = 7,       /* h = x A^T                                              */
    DORA_K_GEMM_LORA = 8,    /* lora = h B^T                                           */
    DORA_K_COMPOSE_FWD = 9,
    DORA_K_COMPOSE_BWD = 10,
    DORA_K_DM_FINAL = 11,    /* second stage of the dm column reduction                */
    DORA_K_GEMM_DH = 12,     /* dh = s dz B                                            */
    DORA_K_GEMM_DX = 13,     /* dx = dz W + dh A                                       */
    DORA_K_GEMM_DA = 14,     /* dA = dh^T x (bf16: the same launch also computes dB)   */
    DORA_K_GEMM_DB = 15,     /* dB = s dz^T h                                          */
    DORA_K_PROBE_COPY = 16,  /* dora_probe_copy                                        */
    DORA_K_PROBE_MFMA = 17,  /* dora_probe_mfma                                        */
    DORA_K_GEMM_FUSED_FWD = 18, /* y = g (.) ([s*h | x] [B | W]^T), dora_forward_fused  */
    DORA_K_SPLITK_REDUCE = 19,  /* fixed-order sum of the K slices of a skinny product    */
    DORA_K_COUNT = 20
};
void dora_trace_enable(int on);
void dora_trace_select(uint64_t kernel_mask); /* bit k set = bracket launches of kernel id k (default: all) */
void dora_trace_reset(void);
int dora_trace_collect(void); /* returns a dora_status */
int dora_trace_get(int kernel_id, double* total_ms, int64_t* launches);
const char* dora_trace_name(int kernel_id);

/*
 * Probes for measurement harnesses (not part of the method).
 *   dora_probe_copy : dst[i] = src[i] for `bytes` bytes (device pointers, 16-byte aligned, bytes a
 *                     multiple of 16): a plain streaming kernel that reads and writes exactly `bytes`
 *                     each - the reference against which HBM byte counters and the achieved
 *                     bandwidth of the compose passes can be scaled.
 *   dora_probe_mfma : `workgroups` workgroups of 4 wavefronts (one per SIMD, as in the large GEMM
 *                     tiles) each issue iters * 64 v_mfma_f32_16x16x32_bf16 (16384 flop per
 *                     instruction per wavefront) on 8 x 8 accumulator tiles from registers: the
 *                     matrix-core rate the card sustains with no memory traffic.  The rate depends
 *                     on the operand values (the card is power limited), so the caller supplies them:
 *                     operands : device, 65536 bytes (16 fragments of 16 bytes per lane for 256
 *                                lanes), any bf16 bit patterns; read once per wavefront.
 *                     sink     : device, fp32 [256], never written in practice.
 */
dora_status dora_probe_copy(const void* src, void* dst, size_t bytes, void* stream);
dora_status dora_probe_mfma(const void* operands, float* sink, int iters, int workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DORA_MEASURE_H */
