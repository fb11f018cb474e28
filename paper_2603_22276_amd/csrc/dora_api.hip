// C ABI of libdora: argument validation, workspace layout and the kernel sequence of each entry
// point.  Every step of the hot path runs in the kernels of this library; there is no fallback.
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "common.hpp"

// Scratch of the entry point that allocates nothing (dora_norm_static): one file-scope device array,
// held by every GPU the library runs on until the process ends.  In host code the array's name is only
// a stand-in; the device address is looked up once per device and used from then on.
#define DORA_STATIC_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[DORA_STATIC_SCRATCH_BYTES];

namespace dora {

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES];  // per device: address of that device's copy of `scratch`

// Device address of the current device's scratch array (nullptr on failure).
void* static_scratch_ptr()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

// ------------------------------------------------------------------------------------------------
// kernel timing (dora_trace_*)
namespace {
struct TraceRec { int id; hipEvent_t e0, e1; };
bool g_trace_on = false;
uint64_t g_trace_mask = ~0ull;
std::vector<TraceRec> g_trace_recs;          // launches since the last collect
std::vector<hipEvent_t> g_event_pool;        // recycled events
double g_trace_ms[DORA_K_COUNT];
int64_t g_trace_n[DORA_K_COUNT];
hipEvent_t g_pending_start = nullptr;

hipEvent_t get_event()
{
    if (!g_event_pool.empty()) { hipEvent_t e = g_event_pool.back(); g_event_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

void trace_begin(int kernel_id, hipStream_t stream)
{
    if (!g_trace_on || !((g_trace_mask >> kernel_id) & 1ull)) return;
    g_pending_start = get_event();
    if (g_pending_start) (void)hipEventRecord(g_pending_start, stream);
}

void trace_end(int kernel_id, hipStream_t stream)
{
    if (!g_trace_on || !g_pending_start) return;
    hipEvent_t e1 = get_event();
    if (!e1) { g_event_pool.push_back(g_pending_start); g_pending_start = nullptr; return; }
    (void)hipEventRecord(e1, stream);
    g_trace_recs.push_back(TraceRec{kernel_id, g_pending_start, e1});
    g_pending_start = nullptr;
}

namespace {

// ------------------------------------------------------------------------------------------------
// validation helpers
constexpr int64_t MAX_ELEMS = (int64_t)1 << 31;

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t esize(int dtype) { return dtype == DORA_F32 ? 4 : 2; }
inline bool is16(int dtype) { return dtype != DORA_F32; }
inline int dt_of(int dtype) { return dtype == DORA_F16 ? DT_F16 : DT_BF16; }
inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

dora_status check_desc(const dora_desc* d, bool need_weights)
{
    if (!d) return DORA_ERR_NULL;
    if (d->dtype != DORA_F32 && d->dtype != DORA_BF16 && d->dtype != DORA_F16) return DORA_ERR_DTYPE;
    const int64_t mult = is16(d->dtype) ? 8 : 4;
    if (d->d_out < mult || d->d_out % mult) return DORA_ERR_SHAPE;
    if (d->tokens < 0) return DORA_ERR_SHAPE;
    if (d->tokens * d->d_out >= MAX_ELEMS) return DORA_ERR_SHAPE;
    if (need_weights) {
        if (d->d_in < mult || d->d_in % mult) return DORA_ERR_SHAPE;
        if (d->r < mult || d->r % mult) return DORA_ERR_SHAPE;
        if (d->d_out * d->d_in >= MAX_ELEMS || d->tokens * d->d_in >= MAX_ELEMS) return DORA_ERR_SHAPE;
        if (d->r * d->d_in >= MAX_ELEMS || d->d_out * d->r >= MAX_ELEMS || d->tokens * d->r >= MAX_ELEMS)
            return DORA_ERR_SHAPE;
    }
    if (!(d->s == d->s) || !(d->eps == d->eps)) return DORA_ERR_SHAPE;  // NaN scalars
    return DORA_OK;
}

inline float eff_eps(const dora_desc* d) { return d->eps > 0.f ? d->eps : (is16(d->dtype) ? 1e-6f : 1e-12f); }

#define DORA_REQ_PTR(p)                          \
    do {                                         \
        if (!(p)) return DORA_ERR_NULL;          \
        if (!aligned((p), 16)) return DORA_ERR_ALIGN; \
    } while (0)
#define DORA_OPT_PTR(p)                                \
    do {                                               \
        if ((p) && !aligned((p), 16)) return DORA_ERR_ALIGN; \
    } while (0)
#define DORA_HIP(call)                                 \
    do {                                               \
        if ((call) != hipSuccess) return DORA_ERR_HIP; \
    } while (0)

// ------------------------------------------------------------------------------------------------
// workspace layout: a bump allocator over the caller's scratch, every block 256-byte aligned
struct Bump {
    char* base;
    size_t off;
    explicit Bump(void* p) : base(static_cast<char*>(p)), off(0) {}
    template <typename T> T* take(size_t count)
    {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += up256(count * sizeof(T));
        return p;
    }
    void* take_bytes(size_t bytes)
    {
        void* p = base ? base + off : nullptr;
        off += up256(bytes);
        return p;
    }
};

// Split-K factors of the two norm contractions: as many workgroups as fit the chip in ONE round
// (256 CUs x two 128x128-tile workgroups each = 512 slots; a 513th would add a whole extra round),
// bounded so the partials stay small.
constexpr int TILE = 128;
inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

struct NormPlan {
    int tiles_n;   // N tiles of the [d_out, r] row-dot contractions
    int ks_u;      // split of d_in for U = W A^T
    int ks_g;      // split of d_in for G = A A^T
    // bf16 path
    float *base_p, *cross_p, *ba_p, *gram_p, *G;
    bf16_t *Ghi, *Glo;
    // fp32 path
    float *U, *BG;
};

void plan_norm(const dora_desc* d, Bump& b, NormPlan& n)
{
    memset(&n, 0, sizeof(n));
    const int ktiles = cdiv(d->d_in, 64);
    n.tiles_n = cdiv(d->r, TILE);
    const int tiles_u = cdiv(d->d_out, TILE) * n.tiles_n;
    n.ks_u = 512 / tiles_u;
    if (n.ks_u > 8) n.ks_u = 8;
    if (n.ks_u > ktiles) n.ks_u = ktiles;
    if (n.ks_u < 1) n.ks_u = 1;
    // the Gram workgroups ride in the cross term's launch: give them what that leaves of the round
    const int tiles_g = n.tiles_n * n.tiles_n;
    const int left = 512 - tiles_u * n.ks_u;
    n.ks_g = (left > 0 ? left : 512) / tiles_g;
    if (n.ks_g > 16) n.ks_g = 16;
    if (n.ks_g > ktiles) n.ks_g = ktiles;
    if (n.ks_g < 1) n.ks_g = 1;
    if (is16(d->dtype)) {
        n.base_p = b.take<float>((size_t)n.ks_u * d->d_out);
        n.cross_p = b.take<float>((size_t)n.ks_u * n.tiles_n * d->d_out);
        n.ba_p = b.take<float>((size_t)n.tiles_n * d->d_out);
        n.gram_p = b.take<float>((size_t)n.ks_g * d->r * d->r);
        n.Ghi = b.take<bf16_t>((size_t)d->r * d->r);
        n.Glo = b.take<bf16_t>((size_t)d->r * d->r);
    } else {
        n.U = b.take<float>((size_t)d->d_out * d->r);
        n.G = b.take<float>((size_t)d->r * d->r);
        n.BG = b.take<float>((size_t)d->d_out * d->r);
    }
}

// Split of K for the skinny products with a 16-bit output (h = x A^T, dh = s dz B): with [tokens, r] outputs of
// 128 x 128 tiles a launch at 4096 tokens has 96 workgroups for 256 CUs.  When at most half the CUs would have
// work, K is cut into slices (fp32 partials in the workspace, summed in slice order by a small reduce launch) so
// that the launch approaches one workgroup per CU, each slice keeping at least 16 K steps.
inline int skinny_ksplit(int dtype, int64_t M, int64_t N, int64_t K)
{
    if (!is16(dtype) || M <= 0) return 1;
    const int64_t tiles = ((M + TILE - 1) / TILE) * ((N + TILE - 1) / TILE);
    if (tiles * 2 > 256) return 1;
    int64_t ks = 256 / tiles;
    if (ks > 4) ks = 4;
    if (ks > K / 1024) ks = K / 1024;
    return ks < 1 ? 1 : (int)ks;
}

// ------------------------------------------------------------------------------------------------
// one contraction, either dtype
struct Seg { const void* a; int64_t lda; const void* b; int64_t ldb; int K; };

GemmArgs bf16_args(int dt, bool a_kc, bool b_kc, int M, int N, const Seg* segs, int nseg, float alpha, void* c,
                   int64_t ldc, bool c_f32, int tag)
{
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    for (int i = 0; i < nseg; ++i)
        g.seg[i] = GemmSeg{(const bf16_t*)segs[i].a, (const bf16_t*)segs[i].b, segs[i].lda, segs[i].ldb, segs[i].K};
    g.nseg = nseg; g.M = M; g.N = N; g.a_kcontig = a_kc; g.b_kcontig = b_kc;
    g.epilogue = c_f32 ? EPI_STORE_F32 : EPI_STORE_BF16;
    g.alpha = alpha; g.c = c; g.ldc = ldc; g.ksplit = 1; g.tag = tag; g.dt = dt;
    return g;
}

// skp != nullptr (16-bit outputs, one segment): scratch for the K slices of a skinny product; the product is then
// split as skinny_ksplit says.  c2 / alpha2: optional second output alpha2 * (A B^T) (16-bit storage only).
hipError_t contract(int dtype, bool a_kc, bool b_kc, int M, int N, const Seg* segs, int nseg, float alpha, void* c,
                    int64_t ldc, bool c_f32, int trace_id, hipStream_t st, float* skp = nullptr, void* c2 = nullptr,
                    float alpha2 = 0.f)
{
    if (is16(dtype)) {
        const int tag = (trace_id == DORA_K_GEMM_LORA || trace_id == DORA_K_GEMM_DB) ? 1 : 0;
        GemmArgs g = bf16_args(dt_of(dtype), a_kc, b_kc, M, N, segs, nseg, alpha, c, ldc, c_f32, tag);
        const int ks = (skp && nseg == 1 && !c_f32 && ldc == N) ? skinny_ksplit(dtype, M, N, segs[0].K) : 1;
        if (ks > 1) {
            g.epilogue = EPI_STORE_F32; g.c = skp; g.ksplit = ks;
            hipError_t e = launch_gemm_bf16(g, trace_id, st);
            if (e != hipSuccess) return e;
            return launch_splitk_reduce(skp, ks, (int64_t)M * N, dtype, c, alpha2, c2, st);
        }
        g.c2 = c2; g.alpha2 = alpha2;
        return launch_gemm_bf16(g, trace_id, st);
    }
    SgemmArgs g;
    memset(&g, 0, sizeof(g));
    for (int i = 0; i < nseg; ++i) {
        SgemmSeg& s = g.seg[i];
        s.a = (const float*)segs[i].a; s.b = (const float*)segs[i].b; s.K = segs[i].K;
        s.sa_m = a_kc ? segs[i].lda : 1; s.sa_k = a_kc ? 1 : segs[i].lda;
        s.sb_n = b_kc ? segs[i].ldb : 1; s.sb_k = b_kc ? 1 : segs[i].ldb;
    }
    g.nseg = nseg; g.M = M; g.N = N; g.alpha = alpha; g.c = (float*)c; g.ldc = ldc;
    return launch_sgemm_f32(g, trace_id, st);
}

// ------------------------------------------------------------------------------------------------
// factored norm (Sec. 2, Algorithm 1)
// base_sq != nullptr: the base term of Eq. 2 comes from the caller's cache and W is not squared again
// c == nullptr: only the terms are wanted.  terms != nullptr: [3, d_out] fp32 receives base_sq, cross, ba_sq.
// G_out != nullptr: [r, r] fp32 receives the Gram matrix of Eq. 4.
// Eq. 6 riding on the norm's last launch: set `done` when g / gm1 were written there
struct MagOut { const float* m; float eps; float* g; float* gm1; bool done; };

dora_status norm_impl(const dora_desc* d, const void* W, const void* A, const void* B, float* c, const NormPlan& n,
                      hipStream_t st, const float* base_sq = nullptr, float* terms = nullptr, float* G_out = nullptr,
                      MagOut* mag = nullptr)
{
    const int d_out = (int)d->d_out, d_in = (int)d->d_in, r = (int)d->r;
    if (d->s == 0.f) {  // scale-is-zero fast path: no U, no G
        if (terms) {  // base_sq from W (or the cache), cross = ba_sq = 0, G not formed
            if (G_out) DORA_HIP(launch_gram_reduce(nullptr, 0, r, G_out, nullptr, nullptr, DT_BF16, st));  // zero partials: G = 0
            if (!base_sq && is16(d->dtype)) {
                DORA_HIP(launch_rownorm_s0_16((const bf16_t*)W, dt_of(d->dtype), n.base_p, d_out, d_in, true, st));
                base_sq = n.base_p;
            }
            if (base_sq) DORA_HIP(launch_norm_final(base_sq, 1, nullptr, 0, nullptr, 0, 0.0, c, terms, d_out, st));
            else DORA_HIP(launch_rownorm_f32((const float*)W, nullptr, nullptr, nullptr, nullptr, 0.0, c, terms, d_out, d_in, r, false, st));
            return DORA_OK;
        }
        if (base_sq) DORA_HIP(launch_norm_final(base_sq, 1, nullptr, 0, nullptr, 0, 0.0, c, nullptr, d_out, st));
        else if (is16(d->dtype)) DORA_HIP(launch_rownorm_s0_16((const bf16_t*)W, dt_of(d->dtype), c, d_out, d_in, false, st));
        else DORA_HIP(launch_rownorm_f32((const float*)W, nullptr, nullptr, nullptr, nullptr, 0.0, c, nullptr, d_out, d_in, r, false, st));
        return DORA_OK;
    }
    if (is16(d->dtype)) {
        const int dt = dt_of(d->dtype);
        GemmArgs g;
        // cross term (Eq. 3) and base term: U = W A^T tile by tile, reduced against B in registers
        memset(&g, 0, sizeof(g));
        g.seg[0] = GemmSeg{(const bf16_t*)W, (const bf16_t*)A, d_in, d_in, d_in};
        g.nseg = 1; g.M = d_out; g.N = r; g.a_kcontig = 1; g.b_kcontig = 1; g.epilogue = EPI_ROWDOT; g.alpha = 1.f; g.dt = dt;
        g.ksplit = n.ks_u; g.rowdot = (const bf16_t*)B; g.ld_rowdot = r; g.rowdot_partial = n.cross_p;
        g.base_sq_partial = base_sq ? nullptr : n.base_p;
        // Gram matrix (Eq. 4): split-K partials, then a fixed-order sum and the hi/lo 16-bit expansion.  It is
        // independent of the cross term and far too small to fill the chip, so its workgroups ride in the same launch.
        GemmArgs gg;
        memset(&gg, 0, sizeof(gg));
        gg.seg[0] = GemmSeg{(const bf16_t*)A, (const bf16_t*)A, d_in, d_in, d_in};
        gg.nseg = 1; gg.M = r; gg.N = r; gg.a_kcontig = 1; gg.b_kcontig = 1; gg.epilogue = EPI_STORE_F32; gg.alpha = 1.f;
        gg.dt = dt; gg.c = n.gram_p; gg.ldc = r; gg.ksplit = n.ks_g;
        DORA_HIP(launch_gemm_bf16_pair(g, gg, DORA_K_NORM_CROSS, st));
        DORA_HIP(launch_gram_reduce(n.gram_p, n.ks_g, r, G_out, n.Ghi, n.Glo, dt, st));
        // BA-norm term: rowdot(B, B G) with G = Ghi + Glo kept to ~16 mantissa bits (G is symmetric,
        // so G serves as its own K-contiguous N-side operand)
        memset(&g, 0, sizeof(g));
        g.seg[0] = GemmSeg{(const bf16_t*)B, n.Ghi, r, r, r};
        g.seg[1] = GemmSeg{(const bf16_t*)B, n.Glo, r, r, r};
        g.nseg = 2; g.M = d_out; g.N = r; g.a_kcontig = 1; g.b_kcontig = 1; g.epilogue = EPI_ROWDOT; g.alpha = 1.f; g.dt = dt;
        g.ksplit = 1; g.rowdot = (const bf16_t*)B; g.ld_rowdot = r; g.rowdot_partial = n.ba_p; g.tag = 1;
        DORA_HIP(launch_gemm_bf16(g, DORA_K_BA_SQ, st));
        DORA_HIP(launch_norm_final(base_sq ? base_sq : n.base_p, base_sq ? 1 : n.ks_u, n.cross_p, n.ks_u * n.tiles_n,
                                   n.ba_p, n.tiles_n, (double)d->s, c, terms, d_out, st, mag ? mag->m : nullptr,
                                   mag ? mag->eps : 0.f, mag ? mag->g : nullptr, mag ? mag->gm1 : nullptr));
        if (mag) mag->done = true;
        return DORA_OK;
    }
    // fp32: Algorithm 1 with one chunk spanning d_in; U [d_out, r], G [r, r], BG [d_out, r] in scratch
    Seg su{W, d_in, A, d_in, d_in};
    DORA_HIP(contract(DORA_F32, true, true, d_out, r, &su, 1, 1.f, n.U, r, true, DORA_K_NORM_CROSS, st));
    Seg sg{A, d_in, A, d_in, d_in};
    DORA_HIP(contract(DORA_F32, true, true, r, r, &sg, 1, 1.f, n.G, r, true, DORA_K_GRAM, st));
    Seg sb{B, r, n.G, r, r};  // (B G)[j,l] = sum_k B[j,k] G[k,l]: N-side operand K-strided
    DORA_HIP(contract(DORA_F32, true, false, d_out, r, &sb, 1, 1.f, n.BG, r, true, DORA_K_BA_SQ, st));
    DORA_HIP(launch_rownorm_f32((const float*)W, base_sq, (const float*)B, n.U, n.BG, (double)d->s, c, terms, d_out, d_in,
                                r, false, st));
    if (G_out) DORA_HIP(hipMemcpyAsync(G_out, n.G, sizeof(float) * (size_t)r * r, hipMemcpyDeviceToDevice, st));
    return DORA_OK;
}

// ------------------------------------------------------------------------------------------------
// forward / backward plans
struct FwdPlan {
    NormPlan norm;
    float *c, *g, *gm1;
    void *h, *lora, *hs, *base_a;
    float* skp;   // K slices of the skinny product h = xa A^T (nullptr: not split)
};
void plan_fwd(const dora_desc* d, Bump& b, FwdPlan& p, bool need_norm, bool need_h, bool need_lora,
              bool need_hs = false, bool need_base_a = false)
{
    memset(&p, 0, sizeof(p));
    if (need_norm) plan_norm(d, b, p.norm);
    p.c = b.take<float>((size_t)d->d_out);
    p.g = b.take<float>((size_t)d->d_out);
    p.gm1 = b.take<float>((size_t)d->d_out);
    if (need_h) p.h = b.take_bytes((size_t)d->tokens * d->r * esize(d->dtype));
    if (need_lora) p.lora = b.take_bytes((size_t)d->tokens * d->d_out * esize(d->dtype));
    if (need_hs) p.hs = b.take_bytes((size_t)d->tokens * d->r * esize(d->dtype));
    if (need_base_a) p.base_a = b.take_bytes((size_t)d->tokens * d->d_out * esize(d->dtype));
    const int ks = skinny_ksplit(d->dtype, d->tokens, d->r, d->d_in);
    if (ks > 1) p.skp = b.take<float>((size_t)ks * d->tokens * d->r);
}

struct BwdPlan {
    NormPlan norm;
    float *c, *g, *gm1, *dm_partial;
    void *dz, *dh, *h, *inner, *dzb;
    float* skp;   // K slices of the skinny products dh = s dz B and (recomputed) h = xa A^T
};
void plan_bwd(const dora_desc* d, Bump& b, BwdPlan& p, bool need_norm, bool need_h, bool need_inner,
              bool need_dzb = false)
{
    memset(&p, 0, sizeof(p));
    if (need_norm) plan_norm(d, b, p.norm);
    p.c = b.take<float>((size_t)d->d_out);
    p.g = b.take<float>((size_t)d->d_out);
    p.gm1 = b.take<float>((size_t)d->d_out);
    p.dm_partial = b.take<float>((size_t)compose_bwd_slabs(d->tokens, (int)d->d_out, d->dtype) * d->d_out);
    p.dz = b.take_bytes((size_t)d->tokens * d->d_out * esize(d->dtype));
    p.dh = b.take_bytes((size_t)d->tokens * d->r * esize(d->dtype));
    if (need_h) p.h = b.take_bytes((size_t)d->tokens * d->r * esize(d->dtype));
    if (need_inner) p.inner = b.take_bytes((size_t)d->tokens * d->d_out * esize(d->dtype));
    if (need_dzb) p.dzb = b.take_bytes((size_t)d->tokens * d->d_out * esize(d->dtype));
    const int ks_dh = skinny_ksplit(d->dtype, d->tokens, d->r, d->d_out);
    const int ks_h = need_h ? skinny_ksplit(d->dtype, d->tokens, d->r, d->d_in) : 1;
    const int ks = ks_dh > ks_h ? ks_dh : ks_h;
    if (ks > 1) p.skp = b.take<float>((size_t)ks * d->tokens * d->r);
}

dora_status check_ws(void* ws, size_t ws_bytes, size_t need)
{
    if (need == 0) return DORA_OK;
    if (!ws) return DORA_ERR_NULL;
    if (!aligned(ws, 256)) return DORA_ERR_ALIGN;
    if (ws_bytes < need) return DORA_ERR_WORKSPACE;
    return DORA_OK;
}

// base = x W^T, h = x A^T, lora = h B^T (App. A item 1)
// xa: the adapter branch's input (x itself unless LoRA dropout gives that branch an input of its own)
dora_status forward_contractions(const dora_desc* d, const void* x, const void* W, const void* A, const void* B,
                                 void* base, void* h, void* lora, hipStream_t st, const void* xa = nullptr,
                                 float* skp = nullptr)
{
    const int T = (int)d->tokens, d_out = (int)d->d_out, d_in = (int)d->d_in, r = (int)d->r;
    Seg s0{x, d_in, W, d_in, d_in};
    Seg s1{xa ? xa : x, d_in, A, d_in, d_in};
    // (base and h are NOT paired into one launch: h's extra tiles would form a fifth, nearly empty
    // round behind the four full rounds of 256 x 256 base tiles and cost more than a launch of their own)
    // (h after base, not before: it then finds part of x still in the memory-side cache; the other order costs 10 us)
    DORA_HIP(contract(d->dtype, true, true, T, d_out, &s0, 1, 1.f, base, d_out, false, DORA_K_GEMM_BASE, st));
    DORA_HIP(contract(d->dtype, true, true, T, r, &s1, 1, 1.f, h, r, false, DORA_K_GEMM_H, st, skp));
    Seg s2{h, r, B, r, r};
    DORA_HIP(contract(d->dtype, true, true, T, d_out, &s2, 1, 1.f, lora, d_out, false, DORA_K_GEMM_LORA, st));
    return DORA_OK;
}

}  // namespace
}  // namespace dora

using namespace dora;

// ================================================================================================
extern "C" {

const char* dora_status_str(int status)
{
    switch (status) {
        case DORA_OK: return "ok";
        case DORA_ERR_NULL: return "required pointer is NULL";
        case DORA_ERR_SHAPE: return "invalid shape or scalar";
        case DORA_ERR_ALIGN: return "pointer not sufficiently aligned";
        case DORA_ERR_DTYPE: return "unknown dtype";
        case DORA_ERR_WORKSPACE: return "workspace too small";
        case DORA_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

size_t dora_workspace_bytes(const dora_desc* desc, int phase)
{
    if (phase == DORA_PHASE_COMPOSE_BACKWARD) {
        if (check_desc(desc, false) != DORA_OK) return 0;
        const size_t n = up256((size_t)compose_bwd_slabs(desc->tokens, (int)desc->d_out, desc->dtype) * desc->d_out * sizeof(float));
        return n > 0 ? n : 256;   // 0 is reserved for "invalid desc"
    }
    if (check_desc(desc, true) != DORA_OK) return 0;
    Bump b(nullptr);
    switch (phase) {
        case DORA_PHASE_NORM: { NormPlan n; plan_norm(desc, b, n); break; }
        case DORA_PHASE_FORWARD: { FwdPlan p; plan_fwd(desc, b, p, true, true, true, true); break; }
        case DORA_PHASE_BACKWARD: { BwdPlan p; plan_bwd(desc, b, p, false, false, false); break; }
        case DORA_PHASE_BACKWARD_RECOMPUTE: { BwdPlan p; plan_bwd(desc, b, p, true, true, true); break; }
        case DORA_PHASE_FORWARD_DROPOUT: { FwdPlan p; plan_fwd(desc, b, p, true, true, true, false, true); break; }
        case DORA_PHASE_BACKWARD_DROPOUT: { BwdPlan p; plan_bwd(desc, b, p, true, true, true, true); break; }
        default: return 0;
    }
    return b.off > 0 ? b.off : 256;
}

dora_status dora_norm(const dora_desc* desc, const void* W, const void* A, const void* B, float* w_norm, void* ws,
                      size_t ws_bytes, void* stream)
{
    dora_status st = check_desc(desc, true);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(W); DORA_REQ_PTR(A); DORA_REQ_PTR(B); DORA_REQ_PTR(w_norm);
    Bump sizing(nullptr);
    NormPlan n;
    plan_norm(desc, sizing, n);
    if ((st = check_ws(ws, ws_bytes, sizing.off)) != DORA_OK) return st;
    Bump b(ws);
    plan_norm(desc, b, n);
    return norm_impl(desc, W, A, B, w_norm, n, (hipStream_t)stream);
}

size_t dora_norm_static_max_bytes(void) { return DORA_STATIC_SCRATCH_BYTES; }

dora_status dora_norm_static(const dora_desc* desc, const void* W, const void* A, const void* B, float* w_norm,
                             void* stream)
{
    dora_status st = check_desc(desc, true);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(W); DORA_REQ_PTR(A); DORA_REQ_PTR(B); DORA_REQ_PTR(w_norm);
    Bump sizing(nullptr);
    NormPlan n;
    plan_norm(desc, sizing, n);
    if (sizing.off > DORA_STATIC_SCRATCH_BYTES) return DORA_ERR_WORKSPACE;  // shape beyond the static scratch
    void* ptr = static_scratch_ptr();
    if (!ptr) return DORA_ERR_HIP;
    // every partial the norm kernels read back is written in full by the launch before it, so nothing
    // left in the array by an earlier call (of any shape) needs clearing
    Bump b(ptr);
    plan_norm(desc, b, n);
    return norm_impl(desc, W, A, B, w_norm, n, (hipStream_t)stream);
}

dora_status dora_base_sq(const dora_desc* desc, const void* W, float* base_sq, void* stream)
{
    dora_status st = check_desc(desc, false);
    if (st != DORA_OK) return st;
    const int64_t mult = is16(desc->dtype) ? 8 : 4;
    if (desc->d_in < mult || desc->d_in % mult || desc->d_out * desc->d_in >= MAX_ELEMS) return DORA_ERR_SHAPE;
    DORA_REQ_PTR(W); DORA_REQ_PTR(base_sq);
    const int d_out = (int)desc->d_out, d_in = (int)desc->d_in;
    hipStream_t s = (hipStream_t)stream;
    if (is16(desc->dtype)) DORA_HIP(launch_rownorm_s0_16((const bf16_t*)W, dt_of(desc->dtype), base_sq, d_out, d_in, true, s));
    else DORA_HIP(launch_rownorm_f32((const float*)W, nullptr, nullptr, nullptr, nullptr, 0.0, base_sq, nullptr, d_out, d_in, 0, true, s));
    return DORA_OK;
}

dora_status dora_norm_cached(const dora_desc* desc, const float* base_sq, const void* W, const void* A, const void* B,
                             float* w_norm, void* ws, size_t ws_bytes, void* stream)
{
    dora_status st = check_desc(desc, true);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(base_sq); DORA_REQ_PTR(W); DORA_REQ_PTR(A); DORA_REQ_PTR(B); DORA_REQ_PTR(w_norm);
    Bump sizing(nullptr);
    NormPlan n;
    plan_norm(desc, sizing, n);
    if ((st = check_ws(ws, ws_bytes, sizing.off)) != DORA_OK) return st;
    Bump b(ws);
    plan_norm(desc, b, n);
    return norm_impl(desc, W, A, B, w_norm, n, (hipStream_t)stream, base_sq);
}

dora_status dora_norm_terms(const dora_desc* desc, const void* W, const void* A, const void* B, float* terms, float* G,
                            void* ws, size_t ws_bytes, void* stream)
{
    dora_status st = check_desc(desc, true);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(W); DORA_REQ_PTR(A); DORA_REQ_PTR(B); DORA_REQ_PTR(terms);
    DORA_OPT_PTR(G);
    Bump sizing(nullptr);
    NormPlan n;
    plan_norm(desc, sizing, n);
    if ((st = check_ws(ws, ws_bytes, sizing.off)) != DORA_OK) return st;
    Bump b(ws);
    plan_norm(desc, b, n);
    return norm_impl(desc, W, A, B, nullptr, n, (hipStream_t)stream, nullptr, terms, G);
}

dora_status dora_norm_assemble(const dora_desc* desc, const float* terms, float* w_norm, void* stream)
{
    dora_status st = check_desc(desc, false);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(terms); DORA_REQ_PTR(w_norm);
    const int d_out = (int)desc->d_out;
    // the same kernel, and so the same arithmetic in the same order, as the last step of dora_norm
    DORA_HIP(launch_norm_final(terms, 1, terms + d_out, 1, terms + 2 * (size_t)d_out, 1, (double)desc->s, w_norm, nullptr, d_out,
                               (hipStream_t)stream));
    return DORA_OK;
}

dora_status dora_mag_scale(const dora_desc* desc, const float* m, const float* w_norm, float* g, float* gm1,
                           void* stream)
{
    dora_status st = check_desc(desc, false);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(m); DORA_REQ_PTR(w_norm);
    if (!g && !gm1) return DORA_ERR_NULL;
    DORA_OPT_PTR(g); DORA_OPT_PTR(gm1);
    DORA_HIP(launch_mag_scale(m, w_norm, eff_eps(desc), g, gm1, (int)desc->d_out, (hipStream_t)stream));
    return DORA_OK;
}

dora_status dora_compose(const dora_desc* desc, const void* base, const void* lora, const float* g, const float* gm1,
                         void* out, int write_delta, void* inner, void* stream)
{
    dora_status st = check_desc(desc, false);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(base); DORA_REQ_PTR(lora); DORA_REQ_PTR(g); DORA_REQ_PTR(out);
    DORA_OPT_PTR(gm1); DORA_OPT_PTR(inner);
    DORA_HIP(launch_compose_fwd(desc->dtype, base, lora, g, gm1, nullptr, desc->s, out, write_delta ? 1 : 0, inner, desc->tokens,
                                (int)desc->d_out, (hipStream_t)stream));
    return DORA_OK;
}

dora_status dora_compose_backward(const dora_desc* desc, const void* dy, const void* inner, const float* g,
                                  const float* w_norm, void* dz, float* dm, void* ws, size_t ws_bytes, void* stream)
{
    dora_status st = check_desc(desc, false);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(dy); DORA_REQ_PTR(g); DORA_REQ_PTR(dz);
    DORA_OPT_PTR(dm);
    float* partial = nullptr;
    if (dm) {
        DORA_REQ_PTR(inner); DORA_REQ_PTR(w_norm);
        size_t need = up256((size_t)compose_bwd_slabs(desc->tokens, (int)desc->d_out, desc->dtype) * desc->d_out * sizeof(float));
        if ((st = check_ws(ws, ws_bytes, need)) != DORA_OK) return st;
        partial = (float*)ws;
    }
    hipStream_t s = (hipStream_t)stream;
    DORA_HIP(launch_compose_bwd(desc->dtype, dy, inner, g, nullptr, dz, nullptr, partial, desc->tokens, (int)desc->d_out, s));
    if (dm)
        DORA_HIP(launch_dm_final(partial, compose_bwd_slabs(desc->tokens, (int)desc->d_out, desc->dtype), w_norm, eff_eps(desc), dm, (int)desc->d_out, s));
    return DORA_OK;
}

dora_status dora_project(const dora_desc* desc, const void* x, const void* W, const void* A, const void* B,
                         void* base, void* h, void* lora, void* stream)
{
    dora_status st = check_desc(desc, true);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(x); DORA_REQ_PTR(W); DORA_REQ_PTR(A); DORA_REQ_PTR(B);
    DORA_REQ_PTR(base); DORA_REQ_PTR(h); DORA_REQ_PTR(lora);
    if (desc->tokens == 0) return DORA_OK;
    return forward_contractions(desc, x, W, A, B, base, h, lora, (hipStream_t)stream);
}

static dora_status forward_impl(const dora_desc* desc, const void* x, const void* x_lora, const void* W, const void* A,
                                const void* B, const float* m, const float* w_norm, const void* bias, void* y, void* saved_h,
                                void* saved_inner, float* w_norm_out, void* ws, size_t ws_bytes, void* stream)
{
    dora_status st = check_desc(desc, true);
    if (st != DORA_OK) return st;
    DORA_REQ_PTR(W); DORA_REQ_PTR(A); DORA_REQ_PTR(B); DORA_REQ_PTR(m);
    if (desc->tokens > 0) { DORA_REQ_PTR(x); DORA_REQ_PTR(y); }
    DORA_OPT_PTR(x_lora);
    DORA_OPT_PTR(w_norm); DORA_OPT_PTR(bias); DORA_OPT_PTR(saved_h); DORA_OPT_PTR(saved_inner); DORA_OPT_PTR(w_norm_out);
    const bool need_norm = (w_norm == nullptr);
    const bool dropout = (x_lora != nullptr);
    Bump sizing(nullptr);
    FwdPlan p;
    plan_fwd(desc, sizing, p, need_norm, saved_h == nullptr, saved_inner == nullptr, false, dropout);
    if ((st = check_ws(ws, ws_bytes, sizing.off)) != DORA_OK) return st;
    Bump b(ws);
    plan_fwd(desc, b, p, need_norm, saved_h == nullptr, saved_inner == nullptr, false, dropout);
    hipStream_t s = (hipStream_t)stream;
    const int T = (int)desc->tokens, d_out = (int)desc->d_out, d_in = (int)desc->d_in;

    MagOut mag{m, eff_eps(desc), p.g, p.gm1, false};
    const float* c = w_norm;
    if (need_norm) {
        float* cw = w_norm_out ? w_norm_out : p.c;
        if ((st = norm_impl(desc, W, A, B, cw, p.norm, s, nullptr, nullptr, nullptr, &mag)) != DORA_OK) return st;
        c = cw;
    } else if (w_norm_out && w_norm_out != w_norm) {
        DORA_HIP(hipMemcpyAsync(w_norm_out, w_norm, sizeof(float) * d_out, hipMemcpyDeviceToDevice, s));
    }
    if (T == 0) return DORA_OK;
    if (!mag.done) DORA_HIP(launch_mag_scale(m, c, eff_eps(desc), p.g, p.gm1, d_out, s));
    // base lands in y and lora in the inner buffer; the compose pass then runs in place on both
    void* h = saved_h ? saved_h : p.h;
    void* lora = saved_inner ? saved_inner : p.lora;
    if ((st = forward_contractions(desc, x, W, A, B, y, h, lora, s, x_lora, p.skp)) != DORA_OK) return st;
    if (!dropout) {
        DORA_HIP(launch_compose_fwd(desc->dtype, y, lora, p.g, p.gm1, bias, desc->s, y, 0, saved_inner, T, d_out, s));
        return DORA_OK;
    }
    // LoRA dropout: the compose runs on the adapter branch's own base x_lora W^T and its delta is added to
    // the frozen layer's output already in y
    Seg sa{x_lora, d_in, W, d_in, d_in};
    DORA_HIP(contract(desc->dtype, true, true, T, d_out, &sa, 1, 1.f, p.base_a, d_out, false, DORA_K_GEMM_BASE, s));
    DORA_HIP(launch_compose_fwd(desc->dtype, p.base_a, lora, p.g, p.gm1, bias, desc->s, y, 2, saved_inner, T, d_out, s));
    return DORA_OK;
}

dora_status dora_forward(const dora_desc* desc, const void* x, const void* W, const void* A, const void* B,
                         const float* m, const float* w_norm, const void* bias, void* y, void* saved_h, void* saved_inner,
                         float* w_norm_out, void* ws, size_t ws_bytes, void* stream)
{
    return forward_impl(desc, x, nullptr, W, A, B, m, w_norm, bias, y, saved_h, saved_inner, w_norm_out, ws, ws_bytes, stream);
}

dora_status dora_forward_dropout(const dora_desc* desc, const void* x, const void* x_lora, const void* W, const void* A,
                                 const void* B, const float* m, const float* w_norm, const void* bias, void* y,
                                 void* saved_h, void* saved_inner, float* w_norm_out, void* ws, size_t ws_bytes,
                                 void* stream)
{
    if (desc && desc->tokens > 0 && !x_lora) return DORA_ERR_NULL;
    return forward_impl(desc, x, x_lora, W, A, B, m, w_norm, bias, y, saved_h, saved_inner, w_norm_out, ws, ws_bytes, stream);
}

dora_status dora_forward_fused(const dora_desc* desc, const void* x, const void* W, const void* A, const void* B,
                               const float* m, const float* w_norm, const void* bias, void* y, void* saved_h, void* saved_inner,
                               float* w_norm_out, void* ws, size_t ws_bytes, void* stream)
{
    dora_status st = check_desc(desc, true);
    if (st != DORA_OK) return st;
    if (!is16(desc->dtype)) return DORA_ERR_DTYPE;
    DORA_REQ_PTR(W); DORA_REQ_PTR(A); DORA_REQ_PTR(B); DORA_REQ_PTR(m);
    if (desc->tokens > 0) { DORA_REQ_PTR(x); DORA_REQ_PTR(y); }
    DORA_OPT_PTR(w_norm); DORA_OPT_PTR(bias); DORA_OPT_PTR(saved_h); DORA_OPT_PTR(saved_inner); DORA_OPT_PTR(w_norm_out);
    const bool need_norm = (w_norm == nullptr);
    Bump sizing(nullptr);
    FwdPlan p;
    plan_fwd(desc, sizing, p, need_norm, saved_h == nullptr, false, true);
    if ((st = check_ws(ws, ws_bytes, sizing.off)) != DORA_OK) return st;
    Bump b(ws);
    plan_fwd(desc, b, p, need_norm, saved_h == nullptr, false, true);
    hipStream_t s = (hipStream_t)stream;
    const int T = (int)desc->tokens, d_out = (int)desc->d_out, d_in = (int)desc->d_in, r = (int)desc->r;

    MagOut mag{m, eff_eps(desc), p.g, nullptr, false};
    const float* c = w_norm;
    if (need_norm) {
        float* cw = w_norm_out ? w_norm_out : p.c;
        if ((st = norm_impl(desc, W, A, B, cw, p.norm, s, nullptr, nullptr, nullptr, &mag)) != DORA_OK) return st;
        c = cw;
    } else if (w_norm_out && w_norm_out != w_norm) {
        DORA_HIP(hipMemcpyAsync(w_norm_out, w_norm, sizeof(float) * d_out, hipMemcpyDeviceToDevice, s));
    }
    if (T == 0) return DORA_OK;
    if (!mag.done) DORA_HIP(launch_mag_scale(m, c, eff_eps(desc), p.g, nullptr, d_out, s));
    // h = x A^T, written twice from the same accumulators: as it is (the saved tensor) and scaled by s,
    // the low-rank operand of the K-concatenated product  [s h | x] [B | W]^T = s h B^T + x W^T
    void* h = saved_h ? saved_h : p.h;
    Seg s1{x, d_in, A, d_in, d_in};
    DORA_HIP(contract(desc->dtype, true, true, T, r, &s1, 1, 1.f, h, r, false, DORA_K_GEMM_H, s, p.skp, p.hs, desc->s));
    Seg segs[2] = {{p.hs, r, B, r, r}, {x, d_in, W, d_in, d_in}};
    GemmArgs g = bf16_args(dt_of(desc->dtype), true, true, T, d_out, segs, 2, 1.f, y, d_out, false, 0);
    g.epilogue = EPI_COMPOSE;
    g.colscale = p.g;
    g.colbias = (const bf16_t*)bias;
    g.c2 = saved_inner;
    DORA_HIP(launch_gemm_bf16(g, DORA_K_GEMM_FUSED_FWD, s));
    return DORA_OK;
}

// x_lora == nullptr: the plain module (dx = dz W + dh A).  Otherwise the adapter branch has its own input:
// dx = dy W (frozen path; x itself is not needed), dx_lora = ((g-1) dy) W + dh A, dA and the recomputed
// h / inner come from x_lora.
static dora_status backward_impl(const dora_desc* desc, const void* dy, const void* x, const void* x_lora, const void* W,
                                 const void* A, const void* B, const float* m, const float* w_norm, const void* saved_h,
                                 const void* saved_inner, void* dx, void* dx_lora, float* dA, float* dB, float* dm,
                                 void* ws, size_t ws_bytes, void* stream)
{
    dora_status st = check_desc(desc, true);
    if (st != DORA_OK) return st;
    const bool dropout = (x_lora != nullptr);
    const void* xa = dropout ? x_lora : x;
    DORA_REQ_PTR(W); DORA_REQ_PTR(A); DORA_REQ_PTR(B); DORA_REQ_PTR(m);
    if (desc->tokens > 0) { DORA_REQ_PTR(dy); DORA_REQ_PTR(xa); }
    DORA_OPT_PTR(w_norm); DORA_OPT_PTR(saved_h); DORA_OPT_PTR(saved_inner);
    DORA_OPT_PTR(dx); DORA_OPT_PTR(dx_lora); DORA_OPT_PTR(dA); DORA_OPT_PTR(dB); DORA_OPT_PTR(dm);
    const bool need_norm = (w_norm == nullptr);
    const bool need_inner = (dm != nullptr) && (saved_inner == nullptr);
    const bool need_h = (saved_h == nullptr) && (dB != nullptr || need_inner);
    const bool need_dzb = dropout && (dx_lora != nullptr);
    Bump sizing(nullptr);
    BwdPlan p;
    plan_bwd(desc, sizing, p, need_norm, need_h, need_inner, need_dzb);
    if ((st = check_ws(ws, ws_bytes, sizing.off)) != DORA_OK) return st;
    Bump b(ws);
    plan_bwd(desc, b, p, need_norm, need_h, need_inner, need_dzb);
    hipStream_t s = (hipStream_t)stream;
    const int T = (int)desc->tokens, d_out = (int)desc->d_out, d_in = (int)desc->d_in, r = (int)desc->r;
    const int dt = desc->dtype;

    MagOut mag{m, eff_eps(desc), p.g, p.gm1, false};
    const float* c = w_norm;
    if (need_norm) {
        if ((st = norm_impl(desc, W, A, B, p.c, p.norm, s, nullptr, nullptr, nullptr, &mag)) != DORA_OK) return st;
        c = p.c;
    }
    if (!mag.done) DORA_HIP(launch_mag_scale(m, c, eff_eps(desc), p.g, p.gm1, d_out, s));

    const void* h = saved_h;
    const void* inner = saved_inner;
    if (T > 0 && need_inner) {
        // recompute (gradient-checkpointing pattern): base -> dz buffer, lora -> inner buffer,
        // then inner = s*lora + base in place; the dz buffer is overwritten by dz afterwards
        void* hbuf = saved_h ? nullptr : p.h;
        if (saved_h) {
            Seg s0{xa, d_in, W, d_in, d_in};
            DORA_HIP(contract(dt, true, true, T, d_out, &s0, 1, 1.f, p.dz, d_out, false, DORA_K_GEMM_BASE, s));
            Seg s2{saved_h, r, B, r, r};
            DORA_HIP(contract(dt, true, true, T, d_out, &s2, 1, 1.f, p.inner, d_out, false, DORA_K_GEMM_LORA, s));
        } else {
            if ((st = forward_contractions(desc, xa, W, A, B, p.dz, hbuf, p.inner, s, nullptr, p.skp)) != DORA_OK) return st;
            h = hbuf;
        }
        DORA_HIP(launch_compose_fwd(dt, p.dz, p.inner, p.g, p.gm1, nullptr, desc->s, nullptr, 0, p.inner, T, d_out, s));
        inner = p.inner;
    } else if (T > 0 && need_h) {
        Seg s1{xa, d_in, A, d_in, d_in};
        DORA_HIP(contract(dt, true, true, T, r, &s1, 1, 1.f, p.h, r, false, DORA_K_GEMM_H, s, p.skp));
        h = p.h;
    }

    // compose backward: dz = g*dy (and (g-1)*dy for a separate adapter input) and the fused two-stage column
    // reduction for dm
    DORA_HIP(launch_compose_bwd(dt, dy, inner, p.g, p.gm1, p.dz, need_dzb ? p.dzb : nullptr, dm ? p.dm_partial : nullptr, T,
                                d_out, s));
    if (dm) DORA_HIP(launch_dm_final(p.dm_partial, compose_bwd_slabs(T, d_out, dt), c, eff_eps(desc), dm, d_out, s));

    // dh = s * dz B   (gradient reaching h)
    if ((dropout ? dx_lora : dx) || dA) {
        Seg sh{p.dz, d_out, B, r, d_out};
        DORA_HIP(contract(dt, true, false, T, r, &sh, 1, desc->s, p.dh, r, false, DORA_K_GEMM_DH, s, p.skp));
    }
    if (!dropout) {
        if (dx) {  // dx = dz W + dh A : one contraction over the concatenated K range
            Seg sx[2] = {{p.dz, d_out, W, d_in, d_out}, {p.dh, r, A, d_in, r}};
            DORA_HIP(contract(dt, true, false, T, d_in, sx, 2, 1.f, dx, d_in, false, DORA_K_GEMM_DX, s));
        }
    } else {
        if (dx) {  // frozen path: dx = dy W
            Seg sx{dy, d_out, W, d_in, d_out};
            DORA_HIP(contract(dt, true, false, T, d_in, &sx, 1, 1.f, dx, d_in, false, DORA_K_GEMM_DX, s));
        }
        if (dx_lora) {  // adapter path: dx_lora = ((g-1) dy) W + dh A
            Seg sx[2] = {{p.dzb, d_out, W, d_in, d_out}, {p.dh, r, A, d_in, r}};
            DORA_HIP(contract(dt, true, false, T, d_in, sx, 2, 1.f, dx_lora, d_in, false, DORA_K_GEMM_DX, s));
        }
    }
    Seg sa{p.dh, r, xa, d_in, T};  // dA = dh^T xa
    Seg sb{p.dz, d_out, h, r, T};  // dB = s * dz^T h
    if (dA && dB && is16(dt)) {
        // the two weight gradients are independent and individually too small to fill the chip: one launch
        GemmArgs ga = bf16_args(dt_of(dt), false, false, r, d_in, &sa, 1, 1.f, dA, d_in, true, 0);
        GemmArgs gb = bf16_args(dt_of(dt), false, false, d_out, r, &sb, 1, desc->s, dB, r, true, 0);
        DORA_HIP(launch_gemm_bf16_pair(ga, gb, DORA_K_GEMM_DA, s));
    } else {
        if (dA) DORA_HIP(contract(dt, false, false, r, d_in, &sa, 1, 1.f, dA, d_in, true, DORA_K_GEMM_DA, s));
        if (dB) DORA_HIP(contract(dt, false, false, d_out, r, &sb, 1, desc->s, dB, r, true, DORA_K_GEMM_DB, s));
    }
    return DORA_OK;
}

dora_status dora_backward(const dora_desc* desc, const void* dy, const void* x, const void* W, const void* A,
                          const void* B, const float* m, const float* w_norm, const void* saved_h,
                          const void* saved_inner, void* dx, float* dA, float* dB, float* dm, void* ws,
                          size_t ws_bytes, void* stream)
{
    return backward_impl(desc, dy, x, nullptr, W, A, B, m, w_norm, saved_h, saved_inner, dx, nullptr, dA, dB, dm, ws, ws_bytes,
                         stream);
}

dora_status dora_backward_dropout(const dora_desc* desc, const void* dy, const void* x_lora, const void* W, const void* A,
                                  const void* B, const float* m, const float* w_norm, const void* saved_h,
                                  const void* saved_inner, void* dx, void* dx_lora, float* dA, float* dB, float* dm,
                                  void* ws, size_t ws_bytes, void* stream)
{
    if (desc && desc->tokens > 0 && !x_lora) return DORA_ERR_NULL;
    if (desc && desc->tokens == 0 && !x_lora) x_lora = W;  // nothing of it is read; keeps the dropout code path
    return backward_impl(desc, dy, nullptr, x_lora, W, A, B, m, w_norm, saved_h, saved_inner, dx, dx_lora, dA, dB, dm, ws,
                         ws_bytes, stream);
}

dora_status dora_probe_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    DORA_REQ_PTR(src); DORA_REQ_PTR(dst);
    if (bytes % 16) return DORA_ERR_SHAPE;
    DORA_HIP(launch_copy_probe(src, dst, bytes, (hipStream_t)stream));
    return DORA_OK;
}

dora_status dora_probe_mfma(const void* operands, float* sink, int iters, int workgroups, void* stream)
{
    DORA_REQ_PTR(operands); DORA_REQ_PTR(sink);
    if (iters < 0 || workgroups < 0 || workgroups > 65536) return DORA_ERR_SHAPE;
    DORA_HIP(launch_mfma_probe(operands, sink, iters, workgroups, (hipStream_t)stream));
    return DORA_OK;
}

// ------------------------------------------------------------------------------------------------
void dora_trace_enable(int on) { g_trace_on = (on != 0); }

void dora_trace_select(uint64_t kernel_mask) { g_trace_mask = kernel_mask; }

void dora_trace_reset(void)
{
    for (auto& r : g_trace_recs) { g_event_pool.push_back(r.e0); g_event_pool.push_back(r.e1); }
    g_trace_recs.clear();
    for (int i = 0; i < DORA_K_COUNT; ++i) { g_trace_ms[i] = 0.0; g_trace_n[i] = 0; }
}

int dora_trace_collect(void)
{
    int rc = DORA_OK;
    for (auto& r : g_trace_recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) rc = DORA_ERR_HIP;
        else if (r.id >= 0 && r.id < DORA_K_COUNT) { g_trace_ms[r.id] += ms; g_trace_n[r.id] += 1; }
        g_event_pool.push_back(r.e0);
        g_event_pool.push_back(r.e1);
    }
    g_trace_recs.clear();
    return rc;
}

int dora_trace_get(int kernel_id, double* total_ms, int64_t* launches)
{
    if (kernel_id < 0 || kernel_id >= DORA_K_COUNT) return DORA_ERR_SHAPE;
    if (total_ms) *total_ms = g_trace_ms[kernel_id];
    if (launches) *launches = g_trace_n[kernel_id];
    return DORA_OK;
}

const char* dora_trace_name(int kernel_id)
{
    static const char* names[DORA_K_COUNT] = {
        "norm_cross_WAt", "gram_AAt", "gram_reduce", "ba_sq_BGB", "norm_final", "mag_scale", "gemm_base_xWt",
        "gemm_h_xAt", "gemm_lora_hBt", "compose_fwd", "compose_bwd", "dm_final", "gemm_dh_dzB", "gemm_dx",
        "gemm_dA", "gemm_dB", "probe_copy", "probe_mfma", "gemm_fused_fwd", "splitk_reduce"};
    return (kernel_id >= 0 && kernel_id < DORA_K_COUNT) ? names[kernel_id] : "?";
}

}  // extern "C"
