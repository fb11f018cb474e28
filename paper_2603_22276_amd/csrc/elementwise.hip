// Element-wise and reduction kernels of the DoRA hot path: magnitude scale (Eq. 6), norm assembly
// (Eq. 5), compose forward (Sec. 3.1, App. C item 1), compose backward with the fused two-stage
// column reduction for the magnitude gradient (Sec. 3.2; Sec. 7 "LLM-guided optimization").
//
// All of these are HBM streams: every thread moves 16-byte vectors, a workgroup owns a fixed set
// of columns (so g / gm1 live in registers) and walks down a slab of token rows.
#include "common.hpp"

namespace dora {

namespace {

// Block shape of the compose passes: CW threads along the column direction (one 16-byte vector each), CH along
// the row direction, CW * CH = 256.  Measured inside the forward + backward sequence at 8192 x 8192: the forward
// pass (two tensors updated in place) is fastest with one thread row spanning 4 KB of every row it touches
// (256 x 1: 85 us against 95 us for 64 x 4); the backward pass (three separate streams) with 64 x 4 and short
// slabs (70 us against 83 / 95 us for 128 x 2 / 256 x 1).  The two passes are not independent: what the forward
// pass leaves behind in the memory system moves the backward pass by several microseconds, so they were tuned
// together, inside the sequence.
constexpr int BWD_CW = 64, BWD_CH = 4;

// 16-byte store with the non-temporal hint, for outputs nothing reads soon; on this part the hint lifts a
// 2-read/2-write stream from ~5.4 to ~6.9 TB/s in isolation.
typedef unsigned int u32x4_nt_t __attribute__((ext_vector_type(4)));
template <typename R>
__device__ __forceinline__ void store_plain(void* p, const R& v)
{
    *reinterpret_cast<R*>(p) = v;
}
template <typename R>
__device__ __forceinline__ void store_stream(void* p, const R& v)
{
    static_assert(sizeof(R) == 16, "16-byte vectors only");
    __builtin_nontemporal_store(__builtin_bit_cast(u32x4_nt_t, v), reinterpret_cast<u32x4_nt_t*>(p));
}

template <typename T> struct Vec;
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    typedef uint4 raw_t;
    static __device__ __forceinline__ void unpack(const raw_t& r, float* f)
    {
        f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
        f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
    }
    static __device__ __forceinline__ raw_t pack(const float* f)
    {
        raw_t r;
        r.x = pack_bf16x2(f[0], f[1]); r.y = pack_bf16x2(f[2], f[3]);
        r.z = pack_bf16x2(f[4], f[5]); r.w = pack_bf16x2(f[6], f[7]);
        return r;
    }
};
template <> struct Vec<f16_t> {
    static constexpr int N = 8;
    typedef uint4 raw_t;
    typedef Elem16<DT_F16> E;
    static __device__ __forceinline__ void unpack(const raw_t& r, float* f)
    {
        f[0] = E::lo(r.x); f[1] = E::hi(r.x); f[2] = E::lo(r.y); f[3] = E::hi(r.y);
        f[4] = E::lo(r.z); f[5] = E::hi(r.z); f[6] = E::lo(r.w); f[7] = E::hi(r.w);
    }
    static __device__ __forceinline__ raw_t pack(const float* f)
    {
        raw_t r;
        r.x = E::pack2(f[0], f[1]); r.y = E::pack2(f[2], f[3]);
        r.z = E::pack2(f[4], f[5]); r.w = E::pack2(f[6], f[7]);
        return r;
    }
};
template <> struct Vec<float> {
    static constexpr int N = 4;
    typedef float4 raw_t;
    static __device__ __forceinline__ void unpack(const raw_t& r, float* f) { f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w; }
    static __device__ __forceinline__ raw_t pack(const float* f) { return make_float4(f[0], f[1], f[2], f[3]); }
};

// ------------------------------------------------------------------------------------------------
// Eq. 6 and the explicit small correction of Sec. 3.1.
__global__ void mag_scale_kernel(const float* __restrict__ m, const float* __restrict__ c, float eps,
                                 float* __restrict__ g, float* __restrict__ gm1, int d_out)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= d_out) return;
    float cj = c[j];
    float cc = (cj < eps) ? eps : cj;  // NaN stays NaN
    float mj = m[j];
    if (g) g[j] = mj / cc;
    if (gm1) gm1[j] = (mj - cc) / cc;  // the subtraction is exact when m/cc is within [1/2, 2]
}

// Eq. 5 from the partial sums the norm kernels left behind; partials are added in index order.
// terms != nullptr: the three summed terms are also written, as rows of a [3, d_out] array (base_sq,
// cross, ba_sq); c == nullptr: only the terms are wanted.  m != nullptr: Eq. 6 follows in the same launch
// (g and / or gm1, exactly as mag_scale_kernel forms them).
__global__ void norm_final_kernel(const float* __restrict__ base_p, int n_base, const float* __restrict__ cross_p,
                                  int n_cross, const float* __restrict__ ba_p, int n_ba, float two_s, float s2,
                                  float* __restrict__ c, float* __restrict__ terms, int d_out,
                                  const float* __restrict__ m, float eps, float* __restrict__ g, float* __restrict__ gm1)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= d_out) return;
    float base_sq = 0.f, cross = 0.f, ba = 0.f;
    for (int i = 0; i < n_base; ++i) base_sq += base_p[(int64_t)i * d_out + j];
    for (int i = 0; i < n_cross; ++i) cross += cross_p[(int64_t)i * d_out + j];
    for (int i = 0; i < n_ba; ++i) ba += ba_p[(int64_t)i * d_out + j];
    if (terms) {
        terms[j] = base_sq;
        terms[(int64_t)d_out + j] = cross;
        terms[2 * (int64_t)d_out + j] = ba;
    }
    if (!c) return;
    float rad = base_sq + two_s * cross + s2 * ba;
    rad = (rad < 0.f) ? 0.f : rad;  // NaN is not < 0: it propagates (App. C item 3)
    const float cj = __fsqrt_rn(rad);
    c[j] = cj;
    if (m) {
        float cc = (cj < eps) ? eps : cj;
        float mj = m[j];
        if (g) g[j] = mj / cc;
        if (gm1) gm1[j] = (mj - cc) / cc;
    }
}

// G = sum of split-K partials (fixed order), and its two-term 16-bit expansion G ~ Ghi + Glo.
template <int DT>
__global__ void gram_reduce_kernel(const float* __restrict__ p, int ksplit, int rr, float* __restrict__ G,
                                   bf16_t* __restrict__ Ghi, bf16_t* __restrict__ Glo)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rr) return;
    float acc = 0.f;
    for (int z = 0; z < ksplit; ++z) acc += p[(int64_t)z * rr + i];
    if (G) G[i] = acc;
    if (!Ghi) return;
    typedef Elem16<DT> E;
    uint32_t hi = E::pack2(acc, 0.f) & 0xffffu;
    float rem = acc - E::lo(hi);     // exact: the leading bits of acc cancel
    Ghi[i] = (bf16_t)hi;
    Glo[i] = (bf16_t)(E::pack2(rem, 0.f) & 0xffffu);
}

// Sum of the K slices of a split contraction, in slice order, rounded once to the storage dtype.
template <typename T>
__global__ void splitk_reduce_kernel(const float* __restrict__ p, int ksplit, int64_t n, T* __restrict__ out,
                                     float alpha2, T* __restrict__ out2)
{
    typedef Vec<T> V;
    constexpr int N = V::N;
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * N;
    if (i >= n) return;
    float acc[N];
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] = 0.f;
    for (int z = 0; z < ksplit; ++z) {
#pragma unroll
        for (int e = 0; e < N; e += 4) {
            const float4 v = *reinterpret_cast<const float4*>(p + (int64_t)z * n + i + e);
            acc[e] += v.x; acc[e + 1] += v.y; acc[e + 2] += v.z; acc[e + 3] += v.w;
        }
    }
    *reinterpret_cast<typename V::raw_t*>(out + i) = V::pack(acc);
    if (out2) {
#pragma unroll
        for (int e = 0; e < N; ++e) acc[e] *= alpha2;
        *reinterpret_cast<typename V::raw_t*>(out2 + i) = V::pack(acc);
    }
}

// fp32 configuration: the three terms of Eq. 2 for one row per wavefront, from U = W A^T and BG = B G.
// base_in != nullptr: the base term is read from it instead of being summed from W (Sec. 2.3: W is frozen, so
// its squared row norms can be computed once).  squared: write the radicand itself, not its root.
__global__ void rownorm_f32_kernel(const float* __restrict__ W, const float* __restrict__ base_in,
                                   const float* __restrict__ B, const float* __restrict__ U,
                                   const float* __restrict__ BG, float two_s, float s2, float* __restrict__ c,
                                   float* __restrict__ terms, int d_out, int d_in, int r, bool squared)
{
    int lane = threadIdx.x & 63;
    int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= d_out) return;
    float base_sq = 0.f, cross = 0.f, ba = 0.f;
    const float* w = W + (int64_t)row * d_in;
    if (!base_in)
        for (int k = lane; k < d_in; k += 64) { float v = w[k]; base_sq = fmaf(v, v, base_sq); }
    if (U) {
        const float* b = B + (int64_t)row * r;
        const float* u = U + (int64_t)row * r;
        const float* bg = BG + (int64_t)row * r;
        for (int l = lane; l < r; l += 64) { float bv = b[l]; cross = fmaf(bv, u[l], cross); ba = fmaf(bv, bg[l], ba); }
    }
    for (int o = 32; o > 0; o >>= 1) {
        base_sq += __shfl_xor(base_sq, o);
        cross += __shfl_xor(cross, o);
        ba += __shfl_xor(ba, o);
    }
    if (lane == 0) {
        if (base_in) base_sq = base_in[row];
        if (terms) {
            terms[row] = base_sq;
            terms[(int64_t)d_out + row] = cross;
            terms[2 * (int64_t)d_out + row] = ba;
        }
        if (c) {
            float rad = base_sq + two_s * cross + s2 * ba;
            rad = (rad < 0.f) ? 0.f : rad;
            c[row] = squared ? rad : __fsqrt_rn(rad);
        }
    }
}

// s == 0 (Algorithm 1, notes): the norm is the row norm of W alone.  One wavefront per row, 16-bit storage.
template <typename T>
__global__ void rownorm_s0_16_kernel(const T* __restrict__ W, float* __restrict__ c, int d_out, int d_in,
                                     bool squared)
{
    int lane = threadIdx.x & 63;
    int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= d_out) return;
    const T* w = W + (int64_t)row * d_in;
    float acc = 0.f;
    for (int k = lane * 8; k < d_in; k += 64 * 8) {
        uint4 v = *reinterpret_cast<const uint4*>(w + k);
        float f[8];
        Vec<T>::unpack(v, f);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = fmaf(f[i], f[i], acc);
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) c[row] = squared ? acc : __fsqrt_rn(acc);
}

// ------------------------------------------------------------------------------------------------
// Compose forward.  delta = gm1*base + g*(s*lora);  out = delta or base + delta;  inner = s*lora + base.
// OUTMODE: 0 = no out tensor (inner only), 1 = out = base + delta, 2 = out = delta, 3 = out += delta (the
// frozen layer's output is already in out and base is the adapter branch's own base, App. B "Chunked
// dropout path").
template <typename T, int OUTMODE, bool INNER, int CW, int CH>
__global__ __launch_bounds__(CW* CH) void compose_fwd_kernel(const T* base_, const T* lora_,  // out may alias base, inner may alias lora
                                                             
                                                              const float* __restrict__ g, const float* __restrict__ gm1,
                                                              const T* __restrict__ bias,  // added to out = base + delta only; may be null
                                                              float s, T* out_, T* inner_, int64_t tokens, int d_out,
                                                              int rows_per_wg, int col_blocks)
{
    typedef Vec<T> V;
    typedef typename V::raw_t raw_t;
    constexpr int N = V::N;
    // one-dimensional grid (no 65535 limit on either extent): consecutive workgroups take neighbouring
    // column blocks of one row slab
    const int col_block = blockIdx.x % col_blocks;
    const int64_t slab = blockIdx.x / col_blocks;
    const int col = (col_block * CW + threadIdx.x) * N;
    if (col >= d_out) return;
    float gv[N], g1[N], bv[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        gv[i] = g[col + i];
        g1[i] = gm1 ? gm1[col + i] : gv[i] - 1.0f;
        bv[i] = 0.f;
    }
    if ((OUTMODE == 1 || OUTMODE == 3) && bias) V::unpack(*reinterpret_cast<const raw_t*>(bias + col), bv);
    const int64_t row_begin = slab * rows_per_wg;
    int64_t row_end = row_begin + rows_per_wg;
    if (row_end > tokens) row_end = tokens;
    constexpr int UNROLL = 4;
    for (int64_t row = row_begin + threadIdx.y; row < row_end; row += CH * UNROLL) {
        raw_t b[UNROLL], l[UNROLL], y0[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            int64_t rr = row + u * CH;
            if (rr < row_end) {
                b[u] = *reinterpret_cast<const raw_t*>(base_ + rr * d_out + col);
                l[u] = *reinterpret_cast<const raw_t*>(lora_ + rr * d_out + col);
                if (OUTMODE == 3) y0[u] = *reinterpret_cast<const raw_t*>(out_ + rr * d_out + col);
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            int64_t rr = row + u * CH;
            if (rr < row_end) {
                float bf[N], lf[N], of[N], inf[N], yf[N];
                V::unpack(b[u], bf);
                V::unpack(l[u], lf);
                if (OUTMODE == 3) V::unpack(y0[u], yf);
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    float sl = s * lf[i];                        // canonical order: s*lora first, then g*(.)
                    float delta = fmaf(g1[i], bf[i], gv[i] * sl);
                    of[i] = (OUTMODE == 2) ? delta : (((OUTMODE == 3) ? yf[i] : bf[i]) + delta) + bv[i];
                    inf[i] = sl + bf[i];
                }
                // y leaves with the streaming hint; inner with a plain store, so that the pass that reads it next (the
                // compose backward of the same module, right away when inner was recomputed) can find it in cache
                if (OUTMODE != 0) store_stream(out_ + rr * d_out + col, V::pack(of));
                if (INNER) store_plain(inner_ + rr * d_out + col, V::pack(inf));
            }
        }
    }
}

// Compose backward: dz = g*dy, and (DM) the first stage of the column sum of dy*inner over this slab.
// SPLIT: also dzb = (g-1)*dy, the gradient reaching the adapter branch's own base when that branch has an
// input of its own (dz then reaches lora only, scaled by s in the products that follow).
template <typename T, bool DM, bool SPLIT, int CW, int CH>
__global__ __launch_bounds__(CW* CH) void compose_bwd_kernel(const T* __restrict__ dy_, const T* __restrict__ inner_,
                                                              const float* __restrict__ g, const float* __restrict__ gm1,
                                                              T* __restrict__ dz_, T* __restrict__ dzb_,
                                                              float* __restrict__ partial, int64_t tokens, int d_out,
                                                              int rows_per_wg, int col_blocks)
{
    typedef Vec<T> V;
    typedef typename V::raw_t raw_t;
    constexpr int N = V::N;
    __shared__ float red[CH][CW * N];
    const int col_block = blockIdx.x % col_blocks;
    const int64_t slab = blockIdx.x / col_blocks;
    const int col = (col_block * CW + threadIdx.x) * N;
    const bool active = col < d_out;
    float gv[N], g1[N], acc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        gv[i] = active ? g[col + i] : 0.f;
        g1[i] = (SPLIT && active) ? gm1[col + i] : 0.f;
        acc[i] = 0.f;
    }
    const int64_t row_begin = slab * rows_per_wg;
    int64_t row_end = row_begin + rows_per_wg;
    if (row_end > tokens) row_end = tokens;
    constexpr int UNROLL = 4, STEP = CH * UNROLL;
    if (active) {
        // Two register sets used in turn (no copies between them): the loads of batch b+1 are in flight while
        // batch b is reduced and stored.  Batches that lie wholly inside the slab take loads and stores without
        // per-row conditions, so the waits the compiler places count exactly the loads still outstanding.
        raw_t da[UNROLL], ia[UNROLL], db[UNROLL], ib[UNROLL];
        auto load_full = [&](int64_t row, raw_t (&dd)[UNROLL], raw_t (&ii)[UNROLL]) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int64_t rr = row + u * CH;
                dd[u] = *reinterpret_cast<const raw_t*>(dy_ + rr * d_out + col);
                if (DM) ii[u] = *reinterpret_cast<const raw_t*>(inner_ + rr * d_out + col);
            }
        };
        auto row_work = [&](int64_t rr, const raw_t& dv, const raw_t& iv) {
            float df[N], nf[N], zf[N], zb[N];
            V::unpack(dv, df);
            if (DM) V::unpack(iv, nf);
#pragma unroll
            for (int i = 0; i < N; ++i) {
                zf[i] = gv[i] * df[i];
                if (SPLIT) zb[i] = g1[i] * df[i];
                if (DM) acc[i] = fmaf(df[i], nf[i], acc[i]);
            }
            store_stream(dz_ + rr * d_out + col, V::pack(zf));   // (a plain store here slows the dh product by 14 us)
            if (SPLIT) store_stream(dzb_ + rr * d_out + col, V::pack(zb));
        };
        auto work_full = [&](int64_t row, const raw_t (&dd)[UNROLL], const raw_t (&ii)[UNROLL]) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) row_work(row + u * CH, dd[u], ii[u]);
        };
        const int nfull = (int)((row_end - row_begin) / STEP);   // uniform over the workgroup
        int64_t row = row_begin + threadIdx.y;
        if (nfull > 0) load_full(row, da, ia);
        for (int b = 0; b < nfull; b += 2) {
            if (b + 1 < nfull) load_full(row + STEP, db, ib);
            work_full(row, da, ia);
            row += STEP;
            if (b + 1 >= nfull) break;
            if (b + 2 < nfull) load_full(row + STEP, da, ia);
            work_full(row, db, ib);
            row += STEP;
        }
        // ragged end of the slab (fewer than STEP rows)
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t rr = row + u * CH;
            if (rr < row_end) {
                raw_t dv = *reinterpret_cast<const raw_t*>(dy_ + rr * d_out + col), iv = dv;
                if (DM) iv = *reinterpret_cast<const raw_t*>(inner_ + rr * d_out + col);
                row_work(rr, dv, iv);
            }
        }
    }
    if (DM) {
#pragma unroll
        for (int i = 0; i < N; ++i) red[threadIdx.y][threadIdx.x * N + i] = acc[i];
        __syncthreads();
        if (threadIdx.y == 0 && active) {
#pragma unroll
            for (int i = 0; i < N; ++i) {
                float v = red[0][threadIdx.x * N + i];
                for (int y = 1; y < CH; ++y) v += red[y][threadIdx.x * N + i];  // fixed order
                partial[slab * d_out + col + i] = v;
            }
        }
    }
}

// Second stage: dm[j] = (sum over slabs, in slab order) / max(c[j], eps).
constexpr int DMF_W = 32, DMF_H = 32;
__global__ __launch_bounds__(DMF_W* DMF_H) void dm_final_kernel(const float* __restrict__ partial, int slabs,
                                                                 const float* __restrict__ c, float eps,
                                                                 float* __restrict__ dm, int d_out)
{
    __shared__ float red[DMF_H][DMF_W];
    int j = blockIdx.x * DMF_W + threadIdx.x;
    float acc = 0.f;
    if (j < d_out) {
        // each of the DMF_H thread rows owns a contiguous range of slabs
        int per = (slabs + DMF_H - 1) / DMF_H;
        int z0 = threadIdx.y * per;
        int z1 = z0 + per < slabs ? z0 + per : slabs;
        for (int z = z0; z < z1; ++z) acc += partial[(int64_t)z * d_out + j];
    }
    red[threadIdx.y][threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.y == 0 && j < d_out) {
        float v = red[0][threadIdx.x];
        for (int y = 1; y < DMF_H; ++y) v += red[y][threadIdx.x];
        float cj = c[j];
        float cc = (cj < eps) ? eps : cj;
        dm[j] = v / cc;
    }
}


}  // namespace

hipError_t launch_mag_scale(const float* m, const float* c, float eps, float* g, float* gm1, int d_out, hipStream_t st)
{
    if (d_out == 0) return hipSuccess;
    TraceScope ts(DORA_K_MAG_SCALE, st);
    mag_scale_kernel<<<dim3((d_out + 255) / 256), dim3(256), 0, st>>>(m, c, eps, g, gm1, d_out);
    return hipGetLastError();
}

hipError_t launch_norm_final(const float* base_p, int n_base, const float* cross_p, int n_cross, const float* ba_p,
                             int n_ba, double s, float* c, float* terms, int d_out, hipStream_t st, const float* m,
                             float eps, float* g, float* gm1)
{
    if (d_out == 0) return hipSuccess;
    TraceScope ts(DORA_K_NORM_FINAL, st);
    // 2s and s^2 are formed in double and rounded once (App. C item 3)
    norm_final_kernel<<<dim3((d_out + 255) / 256), dim3(256), 0, st>>>(base_p, n_base, cross_p, n_cross, ba_p, n_ba,
                                                                       (float)(2.0 * s), (float)(s * s), c, terms, d_out,
                                                                       m, eps, g, gm1);
    return hipGetLastError();
}

hipError_t launch_gram_reduce(const float* partials, int ksplit, int r, float* G, bf16_t* Ghi, bf16_t* Glo, int dt,
                              hipStream_t st)
{
    int rr = r * r;
    if (rr == 0) return hipSuccess;
    TraceScope ts(DORA_K_GRAM_REDUCE, st);
    if (dt == DT_F16) gram_reduce_kernel<DT_F16><<<dim3((rr + 255) / 256), dim3(256), 0, st>>>(partials, ksplit, rr, G, Ghi, Glo);
    else gram_reduce_kernel<DT_BF16><<<dim3((rr + 255) / 256), dim3(256), 0, st>>>(partials, ksplit, rr, G, Ghi, Glo);
    return hipGetLastError();
}

hipError_t launch_splitk_reduce(const float* partials, int ksplit, int64_t n, int dtype, void* out, float alpha2, void* out2,
                                hipStream_t st)
{
    if (n == 0) return hipSuccess;
    TraceScope ts(DORA_K_SPLITK_REDUCE, st);
    const int per = dtype == DORA_F32 ? 4 : 8;
    dim3 grid((unsigned)((n / per + 255) / 256)), block(256);
    if (dtype == DORA_BF16)
        splitk_reduce_kernel<bf16_t><<<grid, block, 0, st>>>(partials, ksplit, n, (bf16_t*)out, alpha2, (bf16_t*)out2);
    else if (dtype == DORA_F16)
        splitk_reduce_kernel<f16_t><<<grid, block, 0, st>>>(partials, ksplit, n, (f16_t*)out, alpha2, (f16_t*)out2);
    else
        splitk_reduce_kernel<float><<<grid, block, 0, st>>>(partials, ksplit, n, (float*)out, alpha2, (float*)out2);
    return hipGetLastError();
}

hipError_t launch_rownorm_s0_16(const bf16_t* W, int dt, float* c, int d_out, int d_in, bool squared, hipStream_t st)
{
    if (d_out == 0) return hipSuccess;
    TraceScope ts(DORA_K_NORM_FINAL, st);
    if (dt == DT_F16)
        rownorm_s0_16_kernel<f16_t><<<dim3((d_out + 3) / 4), dim3(256), 0, st>>>((const f16_t*)W, c, d_out, d_in, squared);
    else
        rownorm_s0_16_kernel<bf16_t><<<dim3((d_out + 3) / 4), dim3(256), 0, st>>>(W, c, d_out, d_in, squared);
    return hipGetLastError();
}

hipError_t launch_rownorm_f32(const float* W, const float* base_in, const float* B, const float* U, const float* BG,
                              double s, float* c, float* terms, int d_out, int d_in, int r, bool squared, hipStream_t st)
{
    if (d_out == 0) return hipSuccess;
    TraceScope ts(DORA_K_NORM_FINAL, st);
    rownorm_f32_kernel<<<dim3((d_out + 3) / 4), dim3(256), 0, st>>>(W, base_in, B, U, BG, (float)(2.0 * s),
                                                                    (float)(s * s), c, terms, d_out, d_in, r, squared);
    return hipGetLastError();
}

// Rows per workgroup: 128 forward, 32 backward (measured inside the whole forward + backward sequence);
// shorter ones are chosen only when the launch would otherwise leave CUs without work.
static int slab_rows(int preferred, int64_t tokens, int d_out, int dtype, int CW)
{
    const int n = dtype == DORA_F32 ? 4 : 8;
    const int64_t col_blocks = (d_out / n + CW - 1) / CW;
    for (int rows = preferred; rows > 16; rows >>= 1)
        if (col_blocks * ((tokens + rows - 1) / rows) >= 512) return rows;
    return 16;
}

template <typename T>
static hipError_t compose_fwd_t(const void* base, const void* lora, const float* g, const float* gm1, const void* bias,
                                float s, void* out, int write_delta, void* inner, int64_t tokens, int d_out,
                                hipStream_t st)
{
    constexpr int N = Vec<T>::N;
    int cpr = d_out / N;
    // the widest block that leaves no thread without a column
    const int CW = cpr >= 256 ? 256 : (cpr >= 128 ? 128 : 64), CH = 256 / CW;
    const int FWD_ROWS_PER_WG = slab_rows(128, tokens, d_out, sizeof(T) == 2 ? DORA_BF16 : DORA_F32, CW);
    const int col_blocks = (cpr + CW - 1) / CW;
    dim3 grid((unsigned)(col_blocks * ((tokens + FWD_ROWS_PER_WG - 1) / FWD_ROWS_PER_WG)));
    dim3 block(CW, CH);
    const T* b = (const T*)base;
    const T* l = (const T*)lora;
    T* o = (T*)out;
    T* in = (T*)inner;
#define DORA_LAUNCH_FWD_S(D, I, W_, H_) \
    compose_fwd_kernel<T, D, I, W_, H_><<<grid, block, 0, st>>>(b, l, g, gm1, (const T*)bias, s, o, in, tokens, d_out, FWD_ROWS_PER_WG, col_blocks)
#define DORA_LAUNCH_FWD(D, I)                                        \
    do {                                                             \
        if (CW == 256) DORA_LAUNCH_FWD_S(D, I, 256, 1);              \
        else if (CW == 128) DORA_LAUNCH_FWD_S(D, I, 128, 2);         \
        else DORA_LAUNCH_FWD_S(D, I, 64, 4);                         \
    } while (0)
    if (!out) { DORA_LAUNCH_FWD(0, true); }
    else if (write_delta == 2) { if (inner) DORA_LAUNCH_FWD(3, true); else DORA_LAUNCH_FWD(3, false); }
    else if (write_delta) { if (inner) DORA_LAUNCH_FWD(2, true); else DORA_LAUNCH_FWD(2, false); }
    else { if (inner) DORA_LAUNCH_FWD(1, true); else DORA_LAUNCH_FWD(1, false); }
#undef DORA_LAUNCH_FWD
#undef DORA_LAUNCH_FWD_S
    return hipGetLastError();
}

hipError_t launch_compose_fwd(int dtype, const void* base, const void* lora, const float* g, const float* gm1,
                              const void* bias, float s, void* out, int write_delta, void* inner, int64_t tokens,
                              int d_out, hipStream_t st)
{
    if (tokens == 0 || d_out == 0) return hipSuccess;
    TraceScope ts(DORA_K_COMPOSE_FWD, st);
    if (dtype == DORA_BF16)
        return compose_fwd_t<bf16_t>(base, lora, g, gm1, bias, s, out, write_delta, inner, tokens, d_out, st);
    if (dtype == DORA_F16)
        return compose_fwd_t<f16_t>(base, lora, g, gm1, bias, s, out, write_delta, inner, tokens, d_out, st);
    return compose_fwd_t<float>(base, lora, g, gm1, bias, s, out, write_delta, inner, tokens, d_out, st);
}

static int compose_bwd_rows(int64_t tokens, int d_out, int dtype) { return slab_rows(32, tokens, d_out, dtype, BWD_CW); }

int compose_bwd_slabs(int64_t tokens, int d_out, int dtype)
{
    const int rows = compose_bwd_rows(tokens, d_out, dtype);
    return (int)((tokens + rows - 1) / rows);
}

template <typename T>
static hipError_t compose_bwd_t(const void* dy, const void* inner, const float* g, const float* gm1, void* dz, void* dzb,
                                float* partial, int64_t tokens, int d_out, hipStream_t st)
{
    constexpr int N = Vec<T>::N;
    int cpr = d_out / N;
    const int dtype = sizeof(T) == 2 ? DORA_BF16 : DORA_F32;
    const int BWD_ROWS_PER_WG = compose_bwd_rows(tokens, d_out, dtype);
    const int col_blocks = (cpr + BWD_CW - 1) / BWD_CW;
    dim3 grid((unsigned)((int64_t)col_blocks * compose_bwd_slabs(tokens, d_out, dtype)));
    dim3 block(BWD_CW, BWD_CH);
#define DORA_LAUNCH_BWD(DM, SP)                                                                                   \
    compose_bwd_kernel<T, DM, SP, BWD_CW, BWD_CH><<<grid, block, 0, st>>>((const T*)dy, (const T*)inner, g, gm1, (T*)dz, (T*)dzb, partial, \
                                                           tokens, d_out, BWD_ROWS_PER_WG, col_blocks)
    if (partial) { if (dzb) DORA_LAUNCH_BWD(true, true); else DORA_LAUNCH_BWD(true, false); }
    else { if (dzb) DORA_LAUNCH_BWD(false, true); else DORA_LAUNCH_BWD(false, false); }
#undef DORA_LAUNCH_BWD
    return hipGetLastError();
}

hipError_t launch_compose_bwd(int dtype, const void* dy, const void* inner, const float* g, const float* gm1, void* dz,
                              void* dzb, float* partial, int64_t tokens, int d_out, hipStream_t st)
{
    if (tokens == 0 || d_out == 0) return hipSuccess;
    TraceScope ts(DORA_K_COMPOSE_BWD, st);
    if (dtype == DORA_BF16) return compose_bwd_t<bf16_t>(dy, inner, g, gm1, dz, dzb, partial, tokens, d_out, st);
    if (dtype == DORA_F16) return compose_bwd_t<f16_t>(dy, inner, g, gm1, dz, dzb, partial, tokens, d_out, st);
    return compose_bwd_t<float>(dy, inner, g, gm1, dz, dzb, partial, tokens, d_out, st);
}

hipError_t launch_dm_final(const float* partial, int slabs, const float* c, float eps, float* dm, int d_out, hipStream_t st)
{
    if (d_out == 0) return hipSuccess;
    TraceScope ts(DORA_K_DM_FINAL, st);
    dm_final_kernel<<<dim3((d_out + DMF_W - 1) / DMF_W), dim3(DMF_W, DMF_H), 0, st>>>(partial, slabs, c, eps, dm, d_out);
    return hipGetLastError();
}

}  // namespace dora
