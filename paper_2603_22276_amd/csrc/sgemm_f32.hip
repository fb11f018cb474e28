// fp32 GEMM used by the fp32 configuration of the module (small shapes: 256 x 512, r = 16).
// Plain LDS-tiled VALU kernel with arbitrary element strides, so one kernel serves every
// contraction of the forward and backward (x W^T, x A^T, h B^T, dz B, dz W + dh A, dh^T x, dz^T h)
// and of Algorithm 1 (W A^T, A A^T, B G).  fp32 FMA accumulation throughout.
#include "common.hpp"

namespace dora {
namespace {

constexpr int TS = 64;   // C tile is TS x TS
constexpr int TK = 16;   // K step
constexpr int TT = 4;    // each thread owns a TT x TT block of C

__global__ __launch_bounds__(256) void sgemm_f32_kernel(SgemmArgs p)
{
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
        for (int k0 = 0; k0 < sg.K; k0 += TK) {
            // 64 x 16 elements per operand tile, 4 per thread
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int e = tid + i * 256;
                int row = e % TS, k = e / TS;
                int gm = m0 + row, gn = n0 + row, gk = k0 + k;
                As[k][row] = (gm < p.M && gk < sg.K) ? sg.a[(int64_t)gm * sg.sa_m + (int64_t)gk * sg.sa_k] : 0.f;
                Bs[k][row] = (gn < p.N && gk < sg.K) ? sg.b[(int64_t)gn * sg.sb_n + (int64_t)gk * sg.sb_k] : 0.f;
            }
            __syncthreads();
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
    dim3 grid((unsigned)(((a.N + TS - 1) / TS) * (int64_t)((a.M + TS - 1) / TS)));
    sgemm_f32_kernel<<<grid, dim3(256), 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace dora
