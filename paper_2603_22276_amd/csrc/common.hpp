// Shared declarations of the HIP translation units of libdora (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dora.h"
#include "../../include/dora_measure.h"

namespace dora {

typedef uint16_t bf16_t;  // storage only; arithmetic is fp32

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// ---- bf16 <-> fp32 on the device ------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even, NaN kept quiet
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    return (f != f) ? 0x7fc0u : r;
}
// two fp32 -> packed bf16 pair with the hardware converter (v_cvt_pk_bf16_f32: nearest-even)
typedef __bf16 bf16x2_hw_t __attribute__((ext_vector_type(2)));
typedef float f32x2_hw_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2_hw_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw_t));
}

// ---- the two 16-bit storage types --------------------------------------------------------------
// Kernels that serve both take a DT template parameter; everything element-specific goes through
// Elem16<DT>: widening a packed pair, packing two fp32 with one rounding (nearest-even; fp16 overflows
// to infinity), and the matching MFMA.
enum { DT_BF16 = 0, DT_F16 = 1 };
struct f16_t { uint16_t bits; };  // distinct C++ type for fp16 storage (bf16_t is a plain uint16_t)
typedef _Float16 f16x2_hw_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

template <int DT> struct Elem16;
template <> struct Elem16<DT_BF16> {
    static __device__ __forceinline__ float lo(uint32_t packed) { return bf16_lo(packed); }
    static __device__ __forceinline__ float hi(uint32_t packed) { return bf16_hi(packed); }
    static __device__ __forceinline__ uint32_t pack2(float a, float b) { return pack_bf16x2(a, b); }
    static __device__ __forceinline__ f32x16_t mfma(bf16x8_t a, bf16x8_t b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4_t mfma16(bf16x8_t a, bf16x8_t b, f32x4_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Elem16<DT_F16> {
    static __device__ __forceinline__ float lo(uint32_t packed)
    {
        return (float)__builtin_bit_cast(f16x2_hw_t, packed)[0];
    }
    static __device__ __forceinline__ float hi(uint32_t packed)
    {
        return (float)__builtin_bit_cast(f16x2_hw_t, packed)[1];
    }
    static __device__ __forceinline__ uint32_t pack2(float a, float b)
    {
        f32x2_hw_t v = {a, b};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_hw_t));
    }
    static __device__ __forceinline__ f32x16_t mfma(bf16x8_t a, bf16x8_t b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0,
                                                      0);
    }
    static __device__ __forceinline__ f32x4_t mfma16(bf16x8_t a, bf16x8_t b, f32x4_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0,
                                                      0);
    }
};

// ---- kernel timing hook (see dora_trace_* in dora_measure.h) ------------------------------------------
void trace_begin(int kernel_id, hipStream_t stream);
void trace_end(int kernel_id, hipStream_t stream);

struct TraceScope {
    int id;
    hipStream_t st;
    TraceScope(int kernel_id, hipStream_t stream) : id(kernel_id), st(stream) { trace_begin(id, st); }
    ~TraceScope() { trace_end(id, st); }
};

// ---- bf16 MFMA GEMM family ---------------------------------------------------------------------
// C[M,N] = alpha * sum over segments of  Aop[m,k] * Bop[n,k]
// An operand is either K-contiguous (row-major [rows, K], ld = row stride) or K-strided
// (row-major [K, rows], ld = stride between consecutive k).
enum GemmEpilogue {
    EPI_STORE_BF16 = 0,  // C bf16 [M, ldc]
    EPI_STORE_F32 = 1,   // C fp32 [M, ldc]; with ksplit > 1 slice z goes to C + z*M*ldc
    EPI_ROWDOT = 2,      // no C; partial[z*tiles_n + tn][m] = sum_n acc[m,n] * R[m,n]  (+ base_sq of Aop rows)
    EPI_COMPOSE = 3      // C bf16 = colscale[n] * acc; optionally C2 bf16 = acc (the compose folded into the epilogue)
};

struct GemmSeg {
    const bf16_t* a;
    const bf16_t* b;
    int64_t lda, ldb;
    int K;
};

struct GemmArgs {
    GemmSeg seg[2];
    int nseg;
    int M, N;
    int a_kcontig, b_kcontig;  // layout of the M-side / N-side operand (both segments)
    int epilogue;
    float alpha;
    void* c;
    int64_t ldc;
    int ksplit;                // split of segment 0's K range (nseg must be 1 when > 1)
    int tag;                   // 0 or 1: selects a differently named (otherwise identical) kernel instance
    int dt;                    // DT_BF16 or DT_F16: element type of both operands, of a 16-bit C and of rowdot / colbias
    const float* colscale;     // EPI_COMPOSE: [N] fp32
    const bf16_t* colbias;     // EPI_COMPOSE: [N] bf16 added to the scaled output, or nullptr
    void* c2;                  // second output [M, ldc] bf16 or nullptr: the unscaled accumulator (compose epilogue),
                               // alpha2 * accumulator (bf16 store epilogue)
    float alpha2;
    // EPI_ROWDOT only
    const bf16_t* rowdot;      // R [M, ld_rowdot] bf16
    int64_t ld_rowdot;
    float* rowdot_partial;     // [ksplit * tiles_n][M]
    float* base_sq_partial;    // [ksplit][M] or nullptr
};

struct GemmPair {
    GemmArgs g[2];
    int count0;  // workgroups of g[0]; the rest of the grid belongs to g[1]
};

// number of N tiles the ROWDOT epilogue will produce partials for (depends on the tile chosen)
int gemm_bf16_tiles_n(const GemmArgs& a);
hipError_t launch_gemm_bf16(const GemmArgs& a, int trace_id, hipStream_t stream);
// two independent problems of the same kind (layouts, epilogue) in one launch
hipError_t launch_gemm_bf16_pair(const GemmArgs& a, const GemmArgs& b, int trace_id, hipStream_t stream);

// ---- fp32 GEMM (simple LDS-tiled VALU kernel; the fp32 configuration is small) ------------------
struct SgemmSeg {
    const float* a;
    const float* b;
    int64_t sa_m, sa_k, sb_n, sb_k;  // element strides
    int K;
};
struct SgemmArgs {
    SgemmSeg seg[2];
    int nseg;
    int M, N;
    float alpha;
    float* c;
    int64_t ldc;
};
hipError_t launch_sgemm_f32(const SgemmArgs& a, int trace_id, hipStream_t stream);

// ---- element-wise / reduction kernels -----------------------------------------------------------
hipError_t launch_mag_scale(const float* m, const float* c, float eps, float* g, float* gm1, int d_out, hipStream_t st);
// write_delta: 0 out = base + delta (+ bias), 1 out = delta, 2 out += delta (+ bias)
hipError_t launch_compose_fwd(int dtype, const void* base, const void* lora, const float* g, const float* gm1,
                              const void* bias, float s, void* out, int write_delta, void* inner, int64_t tokens,
                              int d_out, hipStream_t st);
int compose_bwd_slabs(int64_t tokens, int d_out, int dtype);
// dzb != nullptr: also dzb = gm1 (.) dy (then gm1 must be given)
hipError_t launch_compose_bwd(int dtype, const void* dy, const void* inner, const float* g, const float* gm1, void* dz,
                              void* dzb, float* partial /* [slabs][d_out] or nullptr */, int64_t tokens, int d_out,
                              hipStream_t st);
hipError_t launch_dm_final(const float* partial, int slabs, const float* c, float eps, float* dm, int d_out, hipStream_t st);
// G = sum of partials; Ghi + Glo ~ G as two 16-bit terms of element type dt (both may be nullptr)
hipError_t launch_gram_reduce(const float* partials, int ksplit, int r, float* G, bf16_t* Ghi, bf16_t* Glo, int dt,
                              hipStream_t st);
// c and / or terms ([3, d_out]: the summed base_sq, cross, ba_sq) may be nullptr
// m != nullptr: Eq. 6 in the same launch (g and / or gm1 from m, the norm just formed and eps)
hipError_t launch_norm_final(const float* base_sq_p, int n_base, const float* cross_p, int n_cross, const float* ba_p,
                             int n_ba, double s, float* c, float* terms, int d_out, hipStream_t st,
                             const float* m = nullptr, float eps = 0.f, float* g = nullptr, float* gm1 = nullptr);
hipError_t launch_rownorm_s0_16(const bf16_t* W, int dt, float* c, int d_out, int d_in, bool squared, hipStream_t st);
// fp32 path: base_sq, cross, ba_sq and Eq. 5 from W, B, U = W A^T, BG = B G (all fp32)
hipError_t launch_rownorm_f32(const float* W, const float* base_in, const float* B, const float* U, const float* BG,
                              double s, float* c, float* terms, int d_out, int d_in, int r, bool squared, hipStream_t st);

// out[i] = sum over z (in order) of partials[z * n + i], written in the storage dtype; out2 (may be nullptr)
// receives alpha2 times the same sum.  n a multiple of 8.
hipError_t launch_splitk_reduce(const float* partials, int ksplit, int64_t n, int dtype, void* out, float alpha2, void* out2,
                                hipStream_t st);

hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t st);
hipError_t launch_mfma_probe(const void* operands, float* sink, int iters, int workgroups, hipStream_t st);

}  // namespace dora
