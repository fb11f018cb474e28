// fp32 GEMM used by the fp32 configuration of the module (small shapes: 256 x 512, r = 16).
// Plain LDS-tiled VALU kernel with arbitrary element strides, so one kernel serves every
// contraction of the forward and backward (x W^T, x A^T, h B^T, dz B, dz W + dh A, dh^T x, dz^T h)
// and of Algorithm 1 (W A^T, A A^T, B G).  fp32 FMA accumulation throughout.
#include "common.hpp"

namespace dora {
namespace {

// C tile TS x TS per workgroup of 256 threads, K step TK = 1024 / TS (every thread moves four elements of each
// operand per step), each thread owns a TT x TT block of C.  The shapes this path serves are small, so latency
// counts: global loads run along whichever axis of the operand is contiguous, the next K step is fetched into
// registers while the current one is multiplied, and problems with few 64 x 64 tiles use 32 x 32 ones.
template <int TS>
__global__ __launch_bounds__(256) void sgemm_f32_kernel(SgemmArgs p)
{
    constexpr int TK = 1024 / TS, TT = TS / 16;
    __shared__ float As[TK][TS + 1];
    __shared__ float Bs[TK][TS + 1];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const int tiles_n = (p.N + TS - 1) / TS;   // one-dimensional grid: no 65535 limit on the row-tile count
    const int m0 = (int)(blockIdx.x / tiles_n) * TS, n0 = (int)(blockIdx.x % tiles_n) * TS;
    float acc[TT][TT];
#pragma unroll
    for (int i = 0; i < TT; ++i)
#pragma unroll
        for (int j = 0; j < TT; ++j) acc[i][j] = 0.f;

    for (int sidx = 0; sidx < p.nseg; ++sidx) {
        const SgemmSeg sg = p.seg[sidx];
        // element e of a tile is (row, k): k runs fastest over the threads when the operand is K-contiguous
        const bool a_kfast = (sg.sa_k == 1), b_kfast = (sg.sb_k == 1);
        float ra[4], rb[4];
        auto fetch = [&](int k0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = tid + i * 256;
                const int ar = a_kfast ? e / TK : e % TS, ak = a_kfast ? e % TK : e / TS;
                const int br = b_kfast ? e / TK : e % TS, bk = b_kfast ? e % TK : e / TS;
                const int gm = m0 + ar, gn = n0 + br;
                ra[i] = (gm < p.M && k0 + ak < sg.K) ? sg.a[(int64_t)gm * sg.sa_m + (int64_t)(k0 + ak) * sg.sa_k] : 0.f;
                rb[i] = (gn < p.N && k0 + bk < sg.K) ? sg.b[(int64_t)gn * sg.sb_n + (int64_t)(k0 + bk) * sg.sb_k] : 0.f;
            }
        };
        if (sg.K > 0) fetch(0);
        for (int k0 = 0; k0 < sg.K; k0 += TK) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = tid + i * 256;
                As[a_kfast ? e % TK : e / TS][a_kfast ? e / TK : e % TS] = ra[i];
                Bs[b_kfast ? e % TK : e / TS][b_kfast ? e / TK : e % TS] = rb[i];
            }
            __syncthreads();
            if (k0 + TK < sg.K) fetch(k0 + TK);
#pragma unroll
            for (int k = 0; k < TK; ++k) {
                float a[TT], b[TT];
#pragma unroll
                for (int i = 0; i < TT; ++i) a[i] = As[k][ty * TT + i];
#pragma unroll
                for (int j = 0; j < TT; ++j) b[j] = Bs[k][tx * TT + j];
#pragma unroll
                for (int i = 0; i < TT; ++i)
#pragma unroll
                    for (int j = 0; j < TT; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
            }
            __syncthreads();
        }
    }
#pragma unroll
    for (int i = 0; i < TT; ++i) {
        int gm = m0 + ty * TT + i;
        if (gm >= p.M) continue;
#pragma unroll
        for (int j = 0; j < TT; ++j) {
            int gn = n0 + tx * TT + j;
            if (gn < p.N) p.c[(int64_t)gm * p.ldc + gn] = p.alpha * acc[i][j];
        }
    }
}

}  // namespace

hipError_t launch_sgemm_f32(const SgemmArgs& a, int trace_id, hipStream_t stream)
{
    if (a.M == 0 || a.N == 0) return hipSuccess;
    TraceScope ts(trace_id, stream);
    const int64_t tiles64 = (int64_t)((a.N + 63) / 64) * ((a.M + 63) / 64);
    if (tiles64 >= 128) {
        sgemm_f32_kernel<64><<<dim3((unsigned)tiles64), dim3(256), 0, stream>>>(a);
    } else {
        const int64_t tiles32 = (int64_t)((a.N + 31) / 32) * ((a.M + 31) / 32);
        sgemm_f32_kernel<32><<<dim3((unsigned)tiles32), dim3(256), 0, stream>>>(a);
    }
    return hipGetLastError();
}

}  // namespace dora
