// 16-bit (bf16 or fp16 storage) MFMA GEMM family for gfx950 (CDNA4), fp32 accumulation.
//
//   C[M,N] = alpha * sum_seg sum_k Aop[m,k] * Bop[n,k]
//
// One kernel template serves every dense contraction of the DoRA module: x W^T, x A^T, h B^T
// (both operands K-contiguous), dz W + dh A and dz B (N-side operand K-strided), dh^T x and dz^T h
// (both K-strided), and the factored-norm products of Sec. 2: U = W A^T with the row-dot epilogue
// of Eq. 3 (U never leaves registers), G = A A^T (Eq. 4, split-K partials), and rowdot(B, B G).
//
// Structure (per workgroup): a BM x BN tile of C; K is walked in steps of 64 through rings of LDS
// buffers that the global loads fill directly (buffer_load ... lds, 16 bytes per lane, no register
// staging).  A K step of 64 makes every row segment a load instruction fetches a full 128-byte line;
// 64-byte segments stream at about two thirds of that rate.  Four 64-wide wavefronts per workgroup,
// each owning a (BM/2) x (BN/2) sub-tile.  The N-side fragment is fed as the MFMA's first operand so
// that every lane ends up holding four consecutive n for one m, which makes the epilogue's stores and
// row-dots vector-friendly.  Workgroup ids are remapped so that each of the 8 XCDs (own L2 each) works
// on a compact block of tiles, walked in groups of 8 tile-rows.
//
// Two tile shapes.  128 x 128 (64 x 64 per wave as 2 x 2 of v_mfma_f32_32x32x16, two workgroups per CU,
// which hide each other's stalls) for the skinny products.  256 x 256 (128 x 128 per wave as 8 x 8 of
// v_mfma_f32_16x16x32, accumulators in AGPRs, one wave per SIMD, all 160 KB of LDS) for the large ones:
// this is the wave tile with the fewest fragment reads per MFMA, the instruction shape that draws the
// least power per flop (these launches are power limited), and its memory instructions are interleaved
// with the MFMAs by hand.
#include "common.hpp"

#include <type_traits>
#include <utility>

namespace dora {
namespace {

constexpr int NUM_XCD = 8;
constexpr int GROUP_M = 8;

template <int BM_, int BN_, int WGM_, int WGN_, int BK_, int STAGES_, bool MI16_ = false>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
    static constexpr bool MI16 = MI16_;     // 16x16x32 MFMAs (8 x 8 per wave) instead of 32x32x16 (4 x 4)
    static constexpr int BK = BK_;          // K step per LDS buffer (elements)
    static constexpr int CPR = BK / 8;      // 16-byte chunks per K-contiguous LDS row
    static constexpr int STAGES = STAGES_;  // LDS ring depth (K steps)
    static constexpr int WAVES = WGM * WGN, THREADS = 64 * WAVES;
    static constexpr int WM = BM / WGM, WN = BN / WGN;
    static constexpr int MT = WM / 32, NT = WN / 32;
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int NLA = BM * CPR / THREADS;  // 16-byte loads per lane per K step, M side
    static constexpr int NLB = BN * CPR / THREADS;
    static constexpr int EPI_BYTES_PER_WAVE = 32 * (WN * 4 + 16);
    // Four waves of 128 x 128 each: the M-side operand gets a ring one deeper than STAGES and the two
    // rings lie one after the other; otherwise slot s holds the M-side tile followed by the N-side tile.
    static constexpr bool SPLIT_RING = (WAVES == 4) && (MT * NT >= 16);
    static constexpr int A_STAGES = SPLIT_RING ? STAGES + 1 : STAGES, B_STAGES = STAGES;
    static constexpr int RING_BYTES = A_STAGES * A_BYTES + B_STAGES * B_BYTES;
    static constexpr int LDS_BYTES = (RING_BYTES > WAVES * EPI_BYTES_PER_WAVE) ? RING_BYTES : WAVES * EPI_BYTES_PER_WAVE;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of a gfx950 CU");
    static constexpr int a_slot_off(int s) { return SPLIT_RING ? s * A_BYTES : s * STAGE_BYTES; }
    static constexpr int b_slot_off(int s) { return SPLIT_RING ? A_STAGES * A_BYTES + s * B_BYTES : s * STAGE_BYTES + A_BYTES; }
    static_assert(BK == 64, "the LDS layouts are written for K steps of 64");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
    static_assert(WAVES == 4, "the schedules are written for four waves");
    static_assert(!MI16 || (SPLIT_RING && WM == 128 && WN == 128), "the 16x16x32 schedule is written for 128 x 128 per wave");
    static_assert((BM * CPR) % THREADS == 0 && (BN * CPR) % THREADS == 0, "load plan must divide evenly");
};

typedef Tile<256, 256, 2, 2, 64, 2, true> TileBig; // 256 threads, (3 + 2) x 32 KB of LDS, 256 accumulator registers (AGPRs) per lane
typedef Tile<128, 128, 2, 2, 64, 2> TileMed;      // 256 threads, 2 x 32 KB of LDS, two workgroups fit a CU
typedef Tile<128, 128, 2, 2, 64, 4> TileMedDeep;  // the same with a ring of four, for launches of at most one workgroup per CU

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef uint64_t u64x1_t;
typedef uint64_t u64x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_void_ptr_t;

// The LDS serves a 16-byte-per-lane access 16 lanes at a time, and those 16 lanes must touch 16
// different 16-byte slots modulo 256 bytes.
//
// K-contiguous operand: [rows][64] bf16, 128 bytes per row, the chunk index XORed with row/2: the 16
// rows one group of lanes reads (same logical chunk) then cover all 16 slots.
template <int BK>
__device__ __forceinline__ int kc_swizzle(int row)
{
    static_assert(BK == 64, "swizzle of 128-byte rows");
    return (row >> 1) & 7;
}
template <int BK>
__device__ __forceinline__ int lds_off(int row, int k)
{
    return row * (BK * 2) + ((((k >> 3) ^ kc_swizzle<BK>(row)) & (BK / 8 - 1)) << 4) + ((k & 7) << 1);
}
// K-strided operand: kept as loaded, [BK][ROWS] bf16; chunks of 8 rows XORed with 4*(k mod 4) so the four
// k-rows one transposing read touches fall into different slots, and with 2*(bit 3 of k) so that two
// 16-lane blocks reading the same rows 8 k-rows apart do too.
__device__ __forceinline__ int ks_swizzle(int k)
{
    return ((k & 3) << 2) | (((k >> 3) & 1) << 1);
}
template <int ROWS>
__device__ __forceinline__ int lds_off_ks(int row, int k)
{
    static_assert(ROWS >= 128, "swizzle needs at least 16 chunks per k-row");
    return k * (ROWS * 2) + ((((row >> 3) ^ ks_swizzle(k))) << 4) + ((row & 7) << 1);
}

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{})
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// LDS reads are issued as inline assembly with immediate offsets: the compiler neither tracks them in
// lgkmcnt nor makes them wait for global -> LDS loads still in flight to other ring slots, so every
// consumer is preceded by an explicit wait_lgkmcnt.
template <int OFF>
__device__ __forceinline__ bf16x8_t lds_read_b128(uint32_t addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "ds_read offset field is 16 bits");
    bf16x8_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
// Two transposing reads (k and k + 4 of a K-strided tile, HI bytes apart) forming one MFMA fragment.
// ds_read_b64_tr_b16: inside each block of 16 lanes, lane i receives element (i & 3) of the 8 bytes
// addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.
template <int OFF, int HI>
__device__ __forceinline__ bf16x8_t lds_read_tr(uint32_t addr)
{
    static_assert(OFF >= 0 && OFF + HI < 65536, "ds_read offset field is 16 bits");
    u64x1_t lo, hi;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(OFF));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(OFF + HI));
    u64x2_t v = {lo, hi};
    return __builtin_bit_cast(bf16x8_t, v);
}

// Byte offset, inside an operand's LDS tile, that lane `lane` reads for the MFMA fragment of the 32
// rows starting at row0: the lane gets row row0 + (lane & 31), k = k16*16 + 8*(lane >> 5) + 0..7.
// K-contiguous tile: one 16-byte read.  K-strided tile: the lane points at k-row
// k16*16 + 8*(lane >> 5) + (lane & 15) / 4 and rows 4*(lane & 3) .. +3 of its 16-lane block; blocks 1
// and 3 sit 16 rows further; the second read takes k + 4 (same swizzle).
template <int ROWS, int BK, bool KCONTIG>
__device__ __forceinline__ uint32_t frag_off(int row0, int k16, int lane)
{
    if (KCONTIG) return (uint32_t)lds_off<BK>(row0 + (lane & 31), k16 * 16 + (lane >> 5) * 8);
    return (uint32_t)lds_off_ks<ROWS>(row0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4,
                                      k16 * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2));
}

// The same for the 16x16x32 MFMA: the lane gets row row0 + (lane & 15), k = k32*32 + 8*(lane >> 4) + 0..7.
// K-strided tile: the lane points at k-row k32*32 + 8*(lane >> 4) + (lane & 15) / 4 and rows 4*(lane & 3) .. +3.
template <int ROWS, int BK, bool KCONTIG>
__device__ __forceinline__ uint32_t frag16_off(int row0, int k32, int lane)
{
    if (KCONTIG) return (uint32_t)lds_off<BK>(row0 + (lane & 15), k32 * 32 + (lane >> 4) * 8);
    return (uint32_t)lds_off_ks<ROWS>(row0 + (lane & 3) * 4, k32 * 32 + (lane >> 4) * 8 + ((lane & 15) >> 2));
}

// Global -> LDS for one [ROWS x BK] operand tile.  Each wave-wide load instruction fills 1 KB of
// contiguous LDS (lane i lands at byte 16*i of it), so lane i fetches from global memory whatever
// belongs at that position of the swizzled tile; consecutive lanes cover one row segment of 2*BK bytes.
// Loads go through a buffer descriptor: an offset at or beyond num_records yields zeros, which
// covers rows past the end of the operand; rows or k out of range for other reasons get the offset
// 0xFFFFFFFF.  The K advance travels in the scalar offset.  The LW waves of the workgroup share the tile.
// The issue path itself has no vector arithmetic: a select feeding a load's address, with other vector
// instructions around it, stalls a wave that is otherwise issuing back-to-back 16-cycle MFMAs for several
// MFMAs' time (register-resident probe: 64 MFMAs + 8 such loads + 16 additions 1670 cycles against 1060
// with the loads taking their offsets as they are).  The k mask of a ragged last K step is therefore
// folded into the offsets once, before that step, and an exhausted cursor gets an empty descriptor.
template <int ROWS, int BK, int NL, int LW, bool KCONTIG>
struct OperandLoader {
    static constexpr int CPR = BK / 8;
    static __device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const bf16_t* base, int64_t ld, int rows, int K)
    {
        int64_t elems = KCONTIG ? ((int64_t)(rows - 1) * ld + K) : ((int64_t)(K - 1) * ld + rows);
        if (rows <= 0 || K <= 0) elems = 0;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(base), 0, (int)(uint32_t)(elems * 2), 0x00020000);
    }
    // tile-local (row, k) of the chunk that load i of this lane brings in
    static __device__ __forceinline__ void chunk_of(int i, int lw, int lane, int& row, int& k)
    {
        const int pos = (i * LW + lw) * 64 + lane;  // chunk position in the LDS tile
        if (KCONTIG) {
            row = pos / CPR;
            k = (((pos % CPR) ^ kc_swizzle<BK>(row)) & (CPR - 1)) * 8;
        } else {
            k = pos / (ROWS / 8);
            row = ((pos % (ROWS / 8)) ^ ks_swizzle(k)) * 8;
        }
    }
    // The k index (inside the K step) of load i is that of load 0 plus a compile-time increment: zero for
    // a K-contiguous tile (the swizzle repeats every 16 rows and LW loads cover a multiple of that), the
    // number of k-rows LW wave-loads span for a K-strided one.
    static_assert((LW * 64 / CPR) % 16 == 0, "K-contiguous swizzle must not depend on the load index");
    static constexpr int K_INC = KCONTIG ? 0 : LW * 64 / (ROWS / 8);
    static_assert(KCONTIG || (LW * 64) % (ROWS / 8) == 0, "K-strided loads must step whole k-rows");
    // per-lane constants: byte offset of the chunk of load i at k0 = 0 (0xFFFFFFFF if its row is out of
    // range) and the k index of load 0's chunk inside the K step
    static __device__ __forceinline__ void offsets(uint32_t (&vo)[NL], int& kl0, int64_t ld, int row0, int rows, int lw,
                                                   int lane)
    {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            int row, k;
            chunk_of(i, lw, lane, row, k);
            int grow = row0 + row;
            uint32_t off = KCONTIG ? (uint32_t)(((int64_t)grow * ld + k) * 2) : (uint32_t)(((int64_t)k * ld + grow) * 2);
            vo[i] = (grow < rows) ? off : 0xFFFFFFFFu;
            if (i == 0) kl0 = k;
        }
    }
    // Before a ragged last K step with `krem` k left: chunks whose k index is at or beyond it are pushed
    // out of range and load zeros.
    static __device__ __forceinline__ void mask_tail(uint32_t (&vo)[NL], int kl0, int krem)
    {
#pragma unroll
        for (int i = 0; i < NL; ++i)
            if (kl0 + i * K_INC >= krem) vo[i] = 0xFFFFFFFFu;
    }
    // load I of a K step; `off` is its entry of the offset table
    template <int I>
    static __device__ __forceinline__ void issue_one(char* tile, __amdgpu_buffer_rsrc_t rs, uint32_t off, uint32_t soffset,
                                                     int lw)
    {
        static_assert(I >= 0 && I < NL, "load index");
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_ptr_t)(tile + (I * LW + lw) * 1024), 16, off, soffset, 0, 0);
    }
    static __device__ __forceinline__ void issue(char* tile, __amdgpu_buffer_rsrc_t rs, const uint32_t (&vo)[NL],
                                                 uint32_t soffset, int lw)
    {
        static_for<NL>([&](auto it) { issue_one<decltype(it)::value>(tile, rs, vo[decltype(it)::value], soffset, lw); });
    }
};

// Issue cursor of one operand: descriptor, per-lane offsets and the running scalar offset of the
// segment its global -> LDS loads are walking.  It runs ahead of the MFMAs.
template <class L, int NL, int BK, bool KCONTIG>
struct Cursor {
    uint32_t vo[NL];
    int kl0;
    __amdgpu_buffer_rsrc_t rs;
    uint32_t so, so_step;   // scalar byte offset of the next K step and its increment
    __device__ __forceinline__ void open(const bf16_t* base, int64_t ld, int K, int row0, int rows, int k_first, int wave,
                                         int lane)
    {
        rs = L::make_rsrc(base, ld, rows, K);
        L::offsets(vo, kl0, ld, row0, rows, wave, lane);
        so_step = KCONTIG ? (uint32_t)(BK * 2) : (uint32_t)(BK * ld * 2);
        so = KCONTIG ? (uint32_t)(k_first * 2) : (uint32_t)((int64_t)k_first * ld * 2);
    }
    // the next K step is the ragged last one of its segment, with krem k left
    __device__ __forceinline__ void mask_tail(int krem) { L::mask_tail(vo, kl0, krem); }
    // nothing left to load: every further load brings zeros
    __device__ __forceinline__ void exhaust(const bf16_t* base) { rs = L::make_rsrc(base, 0, 0, 0); }
    template <int I>
    __device__ __forceinline__ void issue_one(char* tile, int wave) const
    {
        L::template issue_one<I>(tile, rs, vo[I], so, wave);
    }
    __device__ __forceinline__ void issue_all(char* tile, int wave) const { L::issue(tile, rs, vo, so, wave); }
    __device__ __forceinline__ void step() { so += so_step; }
};

struct TileCoord { int tm, tn, z; };

// Workgroup id -> (tile row, tile column, K slice).  Hardware hands consecutive ids to the XCDs
// round-robin; undo that so each XCD owns a contiguous range of logical ids, then walk tiles in
// groups of GROUP_M rows so that co-resident tiles share operand panels in that XCD's L2.
__device__ __forceinline__ TileCoord map_tile(int wg, int tiles_m, int tiles_n, int ksplit)
{
    int total = tiles_m * tiles_n * ksplit;
    int q = total / NUM_XCD, rem = total % NUM_XCD;
    int xcd = wg % NUM_XCD, idx = wg / NUM_XCD;
    int logical = (xcd < rem) ? xcd * (q + 1) + idx : rem * (q + 1) + (xcd - rem) * q + idx;
    int tiles = tiles_m * tiles_n;
    TileCoord t;
    t.z = logical / tiles;
    int id = logical % tiles;
    int per_group = GROUP_M * tiles_n;
    int group = id / per_group;
    int first_m = group * GROUP_M;
    int gsz = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
    int in_group = id % per_group;
    t.tm = first_m + in_group % gsz;
    t.tn = in_group / gsz;
    return t;
}

// s_waitcnt with only one counter constrained (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt
// 6:4, lgkmcnt 11:8; the others are left at their maxima)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}
template <int N>
__device__ __forceinline__ void wait_lgkmcnt()
{
    static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
    __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));
}

// TAG takes no part in the computation: it gives the two contractions that would otherwise share an
// instantiation separate kernel names, so that a profiler's per-kernel statistics line up with them.
// DT: element type of the operands (and of a 16-bit C, the row-dot operand and the column bias).
template <class T, bool A_KC, bool B_KC, int EPI, int TAG, int DT>
__global__ __launch_bounds__(T::THREADS) void gemm_bf16_kernel(GemmPair grp)
{
    typedef Elem16<DT> E;
    // one launch may carry two independent problems of the same kind (e.g. dA and dB): workgroups
    // past count0 belong to the second one
    const bool second = (int)blockIdx.x >= grp.count0;
    const GemmArgs& p = second ? grp.g[1] : grp.g[0];
    const int wg_id = (int)blockIdx.x - (second ? grp.count0 : 0);
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, MT = T::MT, NT = T::NT;
    constexpr int KSTEPS = BK / 16;  // MFMA k-steps per K step
    constexpr int FRAG_OPS = MT * (A_KC ? 1 : 2) + NT * (B_KC ? 1 : 2);  // LDS reads per k-step of 16
    constexpr int LPT = T::NLA + T::NLB;  // load instructions per K step per loader lane
    constexpr int STAGES = T::STAGES;
    __shared__ __attribute__((aligned(1024))) char smem[T::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    const int wm = wave / T::WGN, wn = wave % T::WGN;
    const int wm0 = wm * T::WM, wn0 = wn * T::WN;

    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const TileCoord tc = map_tile(wg_id, tiles_m, tiles_n, p.ksplit);
    const int m0 = tc.tm * BM, n0 = tc.tn * BN;

    // flattened K-step schedule over the segments; split-K slices segment 0 only
    const int kt0_total = (p.seg[0].K + BK - 1) / BK;
    const int kt1_total = (p.nseg > 1) ? (p.seg[1].K + BK - 1) / BK : 0;
    int t_begin = 0, t_end = kt0_total + kt1_total;
    if (p.ksplit > 1) {
        int per = (kt0_total + p.ksplit - 1) / p.ksplit;
        t_begin = tc.z * per;
        t_end = t_begin + per < kt0_total ? t_begin + per : kt0_total;
        if (t_end < t_begin) t_end = t_begin;
    }
    const int nsteps = t_end - t_begin;

    constexpr bool MI16 = T::MI16;
    constexpr int M16 = MI16 ? T::WM / 16 : 1, N16 = MI16 ? T::WN / 16 : 1;  // 16 x 16 accumulator tiles per wave
    f32x16_t acc[MI16 ? 1 : MT][MI16 ? 1 : NT];
    f32x4_t acc16[M16][N16];
    if constexpr (MI16) {
#pragma unroll
        for (int i = 0; i < M16; ++i)
#pragma unroll
            for (int j = 0; j < N16; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc16[i][j][e] = 0.f;
    } else {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    }
    float bsq[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) bsq[i] = 0.f;
    const bool want_bsq = (EPI == EPI_ROWDOT) && (p.base_sq_partial != nullptr) && (tc.tn == 0);
    typedef OperandLoader<BM, BK, T::NLA, T::WAVES, A_KC> LA;
    typedef OperandLoader<BN, BK, T::NLB, T::WAVES, B_KC> LB;
    // One cursor per operand; each walks its own schedule.  Segment 0 covers K steps
    // [t_begin, min(t_end, kt0_total)); segment 1 (never split) the rest.  Phases of a schedule: 0 = the
    // whole K steps of segment 0, 1 = its ragged last step, 2 and 3 = the same for segment 1, 4 = exhausted.
    // A counter per cursor runs down to the end of the phase; only then is anything but the scalar offset
    // touched (offsets masked for a ragged step, the next segment opened, the descriptor emptied).
    Cursor<LA, T::NLA, BK, A_KC> ca;
    Cursor<LB, T::NLB, BK, B_KC> cb;
    const bool has_seg1 = (p.nseg > 1) && (t_end > kt0_total);
    const int seg0_k0 = t_begin * BK;
    const int seg0_k1 = (t_end < kt0_total ? t_end : kt0_total) * BK;
    int len0 = (seg0_k1 < p.seg[0].K ? seg0_k1 : p.seg[0].K) - seg0_k0;   // k of segment 0 in this K slice
    if (len0 < 0) len0 = 0;
    const int len1 = has_seg1 ? p.seg[1].K : 0;
    const int whole0 = len0 / BK, rag0 = len0 % BK, whole1 = len1 / BK, rag1 = len1 % BK;
    auto open_a = [&](int sidx) {
        const GemmSeg& sg = p.seg[sidx];
        ca.open(sg.a, sg.lda, sg.K, m0, p.M, sidx ? 0 : seg0_k0, wave, lane);
    };
    auto open_b = [&](int sidx) {
        const GemmSeg& sg = p.seg[sidx];
        cb.open(sg.b, sg.ldb, sg.K, n0, p.N, sidx ? 0 : seg0_k0, wave, lane);
    };
    int a_ph = -1, b_ph = -1, a_left = 0, b_left = 0;   // phase and K steps left in it (negative: never ends)
    // move a cursor to its next non-empty phase
    auto next_phase = [&](auto& cur, int& ph, int& left, auto&& open1, const bf16_t* base0) {
        const int from = ph;
        if (from < 0 && whole0 > 0) { ph = 0; left = whole0; return; }
        if (from < 1 && rag0 > 0) { cur.mask_tail(rag0); ph = 1; left = 1; return; }
        if (from < 2 && (whole1 | rag1) != 0) open1();
        if (from < 2 && whole1 > 0) { ph = 2; left = whole1; return; }
        if (from < 3 && rag1 > 0) { cur.mask_tail(rag1); ph = 3; left = 1; return; }
        cur.exhaust(base0);
        ph = 4;
        left = -1;
    };
    auto next_phase_a = [&]() { next_phase(ca, a_ph, a_left, [&]() { open_a(1); }, p.seg[0].a); };
    auto next_phase_b = [&]() { next_phase(cb, b_ph, b_left, [&]() { open_b(1); }, p.seg[0].b); };
    open_a(0);
    open_b(0);
    next_phase_a();
    next_phase_b();
    auto advance_a = [&]() {
        ca.step();
        if (--a_left == 0) next_phase_a();
    };
    auto advance_b = [&]() {
        cb.step();
        if (--b_left == 0) next_phase_b();
    };
    auto issue = [&](int slot) {   // every load of the next K step of both operands
        ca.issue_all(smem + T::a_slot_off(slot), wave);
        cb.issue_all(smem + T::b_slot_off(slot), wave);
        advance_a();
        advance_b();
    };
    // Per-lane LDS read offsets of the MFMA fragments, relative to the start of the operand's tile.
    // K-contiguous operand: one per k-step of 16; its 32-row blocks follow 32 rows apart, which the
    // swizzle does not see, so they go into the instruction's immediate offset.  K-strided operand: one
    // per 32-row block; its k-steps follow 16 k-rows apart, again an immediate.
    typedef __attribute__((address_space(3))) const char* lds_cptr_t;
    const uint32_t smem_lds = (uint32_t)(uintptr_t)(lds_cptr_t)smem;
    uint32_t rda[4], rdb[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        rda[q] = A_KC ? frag_off<BM, BK, true>(wm0, q < KSTEPS ? q : 0, lane)
                      : frag_off<BM, BK, false>(wm0 + (q < MT ? q : 0) * 32, 0, lane);
        rdb[q] = B_KC ? frag_off<BN, BK, true>(wn0, q < KSTEPS ? q : 0, lane)
                      : frag_off<BN, BK, false>(wn0 + (q < NT ? q : 0) * 32, 0, lane);
    }
    static_assert(MT <= 4 && NT <= 4 && KSTEPS <= 4, "fragment offset tables hold four entries");
    // fragment f (M side first) of k-step KK (both compile time) of the tiles at LDS addresses sa, sb
    auto read_frag = [&](auto kk_tag, auto f_tag, bf16x8_t (&af)[MT], bf16x8_t (&bfr)[NT], uint32_t sa, uint32_t sb) {
        constexpr int KK = decltype(kk_tag)::value, f = decltype(f_tag)::value;
        static_assert(KK < KSTEPS, "k-step outside the K step");
        if constexpr (f < MT) {
            if (A_KC) af[f] = lds_read_b128<f * 32 * BK * 2>(sa + rda[KK]);
            else af[f] = lds_read_tr<KK * 16 * BM * 2, 4 * BM * 2>(sa + rda[f]);
        } else {
            constexpr int j = f - MT;
            if (B_KC) bfr[j] = lds_read_b128<j * 32 * BK * 2>(sb + rdb[KK]);
            else bfr[j] = lds_read_tr<KK * 16 * BN * 2, 4 * BN * 2>(sb + rdb[j]);
        }
    };
    // all fragments of k-step KK of ring slot `slot`
    auto frags = [&](auto kk_tag, bf16x8_t (&af)[MT], bf16x8_t (&bfr)[NT], int slot) {
        const uint32_t sa = smem_lds + T::a_slot_off(slot), sb = smem_lds + T::b_slot_off(slot);
        static_for<MT + NT>([&](auto ft) { read_frag(kk_tag, ft, af, bfr, sa, sb); });
    };
    typedef std::integral_constant<int, 0> K0;
    typedef std::integral_constant<int, 1> K1;
    typedef std::integral_constant<int, 2> K2;
    typedef std::integral_constant<int, 3> K3;
    auto base_term = [&](const bf16x8_t (&af)[MT], int kk) {
        if (EPI == EPI_ROWDOT) {
            // base term of Eq. 2: sum of squares of the M-side rows, taken from the fragments
            // already in registers; the waves along N share the K steps between them
            if (want_bsq && (kk % T::WGN) == wn) {
#pragma unroll
                for (int i = 0; i < MT; ++i) {
                    uint4 u = __builtin_bit_cast(uint4, af[i]);
                    uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float lo = E::lo(w[e]), hi = E::hi(w[e]);
                        bsq[i] = fmaf(lo, lo, bsq[i]);
                        bsq[i] = fmaf(hi, hi, bsq[i]);
                    }
                }
            }
        }
    };
    auto mma = [&](const bf16x8_t (&af)[MT], const bf16x8_t (&bfr)[NT], int kk) {
        if constexpr (!MI16) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = E::mfma(bfr[j], af[i], acc[i][j]);
            base_term(af, kk);
        }
    };

    bf16x8_t a0[MT], b0[NT], a1[MT], b1[NT];
    if constexpr (MI16) {
        // Four waves, one per SIMD, each owning 128 x 128 of the tile as 8 x 8 accumulator tiles of
        // v_mfma_f32_16x16x32 (accumulators in the AGPR half of the register file).  At the power limit the
        // chip sustains about a tenth more flops with this instruction than with 32x32x16 (register-resident
        // loops on random operands: 0.78 against 0.70 of the 2.4 GHz peak): it reads and writes the
        // accumulators half as often per flop.  The LDS traffic is the same: sixteen fragment reads (eight
        // per operand) feed the 64 MFMAs of a k-step of 32.  128 x 128 per wave needs the fewest LDS bytes
        // per MFMA, and with a single wave per SIMD nothing else hides the issue of memory instructions, so
        // they are interleaved with the MFMAs by hand; a 16-cycle MFMA leaves room for three other
        // instructions of the same wave, so whatever can be is kept out of the loop (addresses in immediates).
        //
        // A "burst" runs the 64 MFMAs of one k-step from one fragment set; behind each of the first sixteen,
        // one fragment of the next k-step is read into the other set, in the order the next burst needs
        // them; behind the others, one operand's eight global loads of a K step are issued, one every sixth
        // MFMA.  A K step is two bursts with the workgroup barrier between them.
        //
        // LDS holds three M-side tiles and two N-side tiles.  With barrier(u) = the barrier in the middle of
        // K step u, at which every wave's fragment reads of step u are done:
        //     burst before barrier(u):  M side of step u+2 -> the slot step u-1 used (free since barrier(u-1))
        //     burst after barrier(u):   N side of step u+2 -> the slot step u used; fragments of step u+1
        // At barrier(u) everything but the M side of step u+2 has landed (loads complete in order), which
        // includes all of step u+1.  Either side has about one K step to land.
        //
        // The loop takes two K steps per trip, so that the N-side slot, and with it every N-side LDS address,
        // is a compile-time offset.  An odd number of K steps is rounded up: the loads past the end of the
        // schedule bring zeros, so the extra step adds nothing.  (Separate code for the odd step, or for a
        // steady state without load masking, makes the compiler copy the 256 accumulators between paths.)
        constexpr int NM = M16 * N16, NF = M16 + N16;
        static_assert(KSTEPS == 4 && STAGES == 2 && T::NLA <= NM - NF && T::NLB <= NM - NF, "burst schedule assumptions");
        static_assert(T::B_BYTES + 7 * 16 * BK * 2 < 65536 && T::B_BYTES + 32 * BN * 2 + 4 * BN * 2 < 65536, "immediate offsets");
        // Per-lane LDS read addresses of the fragments.  K-contiguous operand: one per k-step of 32; its 16-row
        // blocks follow 16 rows apart, which the swizzle does not see (immediate offset).  K-strided: one per
        // 16-row block; the k-steps follow 32 k-rows apart (immediate offset).  The N-side ones include the
        // start of the N-side ring; the M-side ones are relative to the slot (three slots: run-time rotation).
        constexpr int NRA = A_KC ? 2 : M16, NRB = B_KC ? 2 : N16;
        uint32_t ra16[NRA], rb16[NRB];
#pragma unroll
        for (int q = 0; q < NRA; ++q)
            ra16[q] = A_KC ? frag16_off<BM, BK, true>(wm0, q, lane) : frag16_off<BM, BK, false>(wm0 + q * 16, 0, lane);
#pragma unroll
        for (int q = 0; q < NRB; ++q)
            rb16[q] = smem_lds + T::b_slot_off(0) +
                      (B_KC ? frag16_off<BN, BK, true>(wn0, q, lane) : frag16_off<BN, BK, false>(wn0 + q * 16, 0, lane));
        // fragment f (M side first) of k-step KK2 (0 or 1): M side from the tile at LDS address sa, N side from
        // N-side slot SLOT
        auto read_frag16 = [&](auto kk_tag, auto slot_tag, auto f_tag, bf16x8_t (&af)[M16], bf16x8_t (&bfr)[N16], uint32_t sa) {
            constexpr int KK2 = decltype(kk_tag)::value, SLOT = decltype(slot_tag)::value, f = decltype(f_tag)::value;
            static_assert(KK2 < 2 && SLOT < 2 && f < NF, "fragment index");
            if constexpr (f < M16) {
                // (K-contiguous: the caller passes the address of the k-step, slot and per-lane part added up
                // ahead of the burst; an addition right in front of the read it feeds holds the wave up)
                if constexpr (A_KC) af[f] = lds_read_b128<f * 16 * BK * 2>(sa);
                else af[f] = lds_read_tr<KK2 * 32 * BM * 2, 4 * BM * 2>(sa + ra16[f]);
            } else {
                constexpr int j = f - M16;
                if constexpr (B_KC) bfr[j] = lds_read_b128<SLOT * T::B_BYTES + j * 16 * BK * 2>(rb16[KK2]);
                else bfr[j] = lds_read_tr<SLOT * T::B_BYTES + KK2 * 32 * BN * 2, 4 * BN * 2>(rb16[j]);
            }
        };
        // MFMAs of the k-step held in (xa, xb); fragments of k-step KK2 of (sa, N-side slot SLOT) -> (na, nb),
        // first the ones the next burst starts with (M block 0, then every N block, then the other M blocks);
        // the loads of one K step of the M side (SIDE 0) or N side (SIDE 1) into `tile`
        auto burst16 = [&](auto kk_tag, auto slot_tag, auto side_tag, const bf16x8_t (&xa)[M16],
                           const bf16x8_t (&xb)[N16], bf16x8_t (&na)[M16], bf16x8_t (&nb)[N16], uint32_t sa, char* tile) {
            constexpr int SIDE = decltype(side_tag)::value;
            constexpr int NL = SIDE == 0 ? T::NLA : T::NLB;
            constexpr int LS = (NM - NF) / NL;
            static_for<NM>([&](auto nt) {
                constexpr int n = decltype(nt)::value;
                constexpr int i = n / N16, j = n % N16;
                acc16[i][j] = E::mfma16(xb[j], xa[i], acc16[i][j]);
                if constexpr (n < NF) {
                    constexpr int f = (n == 0) ? 0 : (n <= N16 ? M16 + n - 1 : n - N16);
                    read_frag16(kk_tag, slot_tag, std::integral_constant<int, f>{}, na, nb, sa);
                } else if constexpr ((n - NF) % LS == 0 && (n - NF) / LS < NL) {
                    constexpr int t = (n - NF) / LS;
                    if constexpr (SIDE == 0) {
                        ca.template issue_one<t>(tile, wave);
                        if constexpr (t == T::NLA - 1) advance_a();
                    } else {
                        cb.template issue_one<t>(tile, wave);
                        if constexpr (t == T::NLB - 1) advance_b();
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        typedef std::integral_constant<int, 0> SideA;
        typedef std::integral_constant<int, 1> SideB;
        bf16x8_t fa0[M16], fb0[N16], fa1[M16], fb1[N16];
        int sa_cur = 0, sa_nxt = 1, sa_fill = 2;       // M-side slots of steps u, u+1, u+2 (mod 3)
        // K step u, u mod 2 == PAR
        auto kstep = [&](auto par_tag) {
            constexpr int PAR = decltype(par_tag)::value;
            typedef std::integral_constant<int, PAR> Cur;
            typedef std::integral_constant<int, PAR ^ 1> Nxt;
            uint32_t sa = smem_lds + T::a_slot_off(sa_cur), sa1 = smem_lds + T::a_slot_off(sa_nxt);
            if constexpr (A_KC) { sa += ra16[1]; sa1 += ra16[0]; }
            wait_lgkmcnt<0>();
            __builtin_amdgcn_sched_barrier(0);
            // k-step 0; fragments of k-step 1; M side of step u+2
            burst16(K1{}, Cur{}, SideA{}, fa0, fb0, fa1, fb1, sa, smem + T::a_slot_off(sa_fill));
            // Everything but the M side of step u+2 has landed, i.e. all of step u+1 (own share); own
            // reads of step u are done.  After the barrier step u+1 is visible to all and the slots of
            // step u may be refilled.
            __builtin_amdgcn_sched_barrier(0);
            wait_vmcnt<T::NLA>();
            wait_lgkmcnt<0>();
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);          // no MFMA may move above the waits
            // k-step 1; first fragments of step u+1; N side of step u+2
            burst16(K0{}, Nxt{}, SideB{}, fa1, fb1, fa0, fb0, sa1, smem + T::b_slot_off(PAR));
            const int t = sa_cur;
            sa_cur = sa_nxt; sa_nxt = sa_fill; sa_fill = t;
        };
        // before the loop: both sides of steps 0 and 1
        ca.issue_all(smem + T::a_slot_off(0), wave);
        advance_a();
        cb.issue_all(smem + T::b_slot_off(0), wave);
        advance_b();
        ca.issue_all(smem + T::a_slot_off(1), wave);
        advance_a();
        cb.issue_all(smem + T::b_slot_off(1), wave);
        advance_b();
        wait_vmcnt<T::NLA + T::NLB>();                 // own share of step 0 landed
        __builtin_amdgcn_s_barrier();                  // all of step 0 landed
        static_for<NF>([&](auto ft) { read_frag16(K0{}, K0{}, ft, fa0, fb0, smem_lds + T::a_slot_off(0) + (A_KC ? ra16[0] : 0u)); });
        for (int u = 0; u < nsteps; u += 2) {
            kstep(K0{});
            kstep(K1{});
        }
        wait_vmcnt<0>();
        wait_lgkmcnt<0>();
    } else if constexpr (STAGES >= 3) {
        // 64 x 64 per wave, one workgroup per CU (launches of at most one workgroup per CU get this
        // tile): with a single wave per SIMD and only four MFMAs per k-step, a fragment read issued one
        // k-step ahead has not landed when its MFMAs are due.  Fragments are therefore read two k-steps
        // ahead into four register sets (one per k-step of a K step), one fragment behind each MFMA.
        // The workgroup barrier sits in the middle of a K step: before k-step 2, whose MFMAs are
        // interleaved with the first reads of the next K step.  By then every wave has consumed all
        // fragments of the previous K step, so its buffer is refilled from there on: a quarter of a K
        // step's global loads behind the MFMAs of each of the next four k-steps (k-steps 2, 3 and, past the
        // end of the loop body, 0 and 1), one load every other MFMA.  (All of them behind one k-step held
        // the wave up for half a K step's time: loads closer together than about six MFMA slots of 16
        // cycles wait for one another.)
        constexpr int NM = MT * NT, NF = MT + NT;
        static_assert(KSTEPS == 4 && NF <= NM && LPT % NM == 0, "deep-prefetch schedule assumptions");
        bf16x8_t fa[4][MT], fb[4][NT];
        // MFMAs of k-step KC (set KC); fragments of k-step KN (set KN) of ring slot `slot`; quarter Q of
        // the global loads of the cursors' K step into ring slot `fill` (M side first)
        constexpr int LQ = LPT / 4;
        static_assert(LPT % 4 == 0 && T::NLA % LQ == 0 && LQ * 2 <= NM, "a quarter of the loads behind every other MFMA");
        auto burst = [&](auto kc_tag, auto kn_tag, auto q_tag, int slot, int fill, int kk) {
            constexpr int KC = decltype(kc_tag)::value, KN = decltype(kn_tag)::value, Q = decltype(q_tag)::value;
            const uint32_t sa = smem_lds + T::a_slot_off(slot), sb = smem_lds + T::b_slot_off(slot);
            static_for<NM>([&](auto nt) {
                constexpr int n = decltype(nt)::value;
                constexpr int i = n / NT, j = n % NT;
                acc[i][j] = E::mfma(fb[KC][j], fa[KC][i], acc[i][j]);
                if constexpr (n < NF) read_frag(kn_tag, nt, fa[KN], fb[KN], sa, sb);
                if constexpr (n % 2 == 1 && n / 2 < LQ) {
                    constexpr int t = Q * LQ + n / 2;
                    if constexpr (t < T::NLA) {
                        ca.template issue_one<t>(smem + T::a_slot_off(fill), wave);
                        if constexpr (t == T::NLA - 1) advance_a();
                    } else {
                        cb.template issue_one<t - T::NLA>(smem + T::b_slot_off(fill), wave);
                        if constexpr (t == LPT - 1) advance_b();
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            base_term(fa[KC], kk);
        };
        // before the loop: steps 0 .. STAGES-3 and the first half of the loads of step STAGES-2
#pragma unroll
        for (int u = 0; u < STAGES - 2; ++u) issue(u);
        static_for<LPT / 2>([&](auto tt) {
            constexpr int t = decltype(tt)::value;
            if constexpr (t < T::NLA) {
                ca.template issue_one<t>(smem + T::a_slot_off(STAGES - 2), wave);
                if constexpr (t == T::NLA - 1) advance_a();
            } else {
                cb.template issue_one<t - T::NLA>(smem + T::b_slot_off(STAGES - 2), wave);
            }
        });
        wait_vmcnt<(STAGES - 3) * LPT + LPT / 2>();    // own share of step 0 landed
        __builtin_amdgcn_s_barrier();
        frags(K0{}, fa[0], fb[0], 0);
        frags(K1{}, fa[1], fb[1], 0);
        for (int u = 0; u < nsteps; ++u) {
            const int slot = u % STAGES, next = (u + 1) % STAGES;
            const int fill_late = (u + STAGES - 2) % STAGES, fill = (u + STAGES - 1) % STAGES;
            wait_lgkmcnt<FRAG_OPS>();                  // set 0 landed; set 1 may still be in flight
            __builtin_amdgcn_sched_barrier(0);
            burst(K0{}, K2{}, K2{}, slot, fill_late, 4 * u);        // third quarter of step u + STAGES - 2
            wait_lgkmcnt<FRAG_OPS>();
            __builtin_amdgcn_sched_barrier(0);
            burst(K1{}, K3{}, K3{}, slot, fill_late, 4 * u + 1);    // its last quarter
            // own share of step u+1 landed (STAGES-3 later steps may be in flight); after the barrier it
            // is visible to all, and the buffer of step u-1, whose last fragments every wave consumed
            // before it got here, takes step u + STAGES - 1
            wait_vmcnt<(STAGES - 3) * LPT>();
            wait_lgkmcnt<FRAG_OPS>();                  // set 2 landed
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);          // no MFMA may move above the waits
            burst(K2{}, K0{}, K0{}, next, fill, 4 * u + 2);         // first quarter of step u + STAGES - 1
            wait_lgkmcnt<FRAG_OPS>();
            __builtin_amdgcn_sched_barrier(0);
            burst(K3{}, K1{}, K1{}, next, fill, 4 * u + 3);         // second quarter
        }
        wait_vmcnt<0>();
        wait_lgkmcnt<0>();
    } else {
        // Four waves.  STAGES-1 K steps are in flight behind the one being
        // multiplied.  Per K step (two or four k-steps of 16): wait for its data, workgroup barrier (which
        // also says every wave is done reading the previous step), refill the buffer that step used,
        // then alternate fragment reads and MFMAs with the fragments double buffered in registers; the
        // last MFMAs of a step run after the next step's barrier and cover its first fragment reads.
        if (nsteps > 0) {
#pragma unroll
            for (int u = 0; u < STAGES - 1; ++u) issue(u);
        }
        for (int u = 0; u < nsteps; ++u) {
            const int slot = u % STAGES;
            __builtin_amdgcn_sched_barrier(0);
            wait_vmcnt<(STAGES - 2) * LPT>();
            wait_lgkmcnt<0>();
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);          // no MFMA may move above the waits
            frags(K0{}, a0, b0, slot);
            __builtin_amdgcn_sched_barrier(0);
            if (u > 0) {
                // the last MFMAs of the previous step (their fragments were complete before the barrier) with
                // the loads of step u + STAGES - 1 behind them, a share behind each
                const int fill = (u + STAGES - 1) % STAGES;
                static_for<MT * NT>([&](auto nt) {
                    constexpr int n = decltype(nt)::value, i = n / NT, j = n % NT;
                    acc[i][j] = E::mfma(b1[j], a1[i], acc[i][j]);
                    static_for<LPT / (MT * NT)>([&](auto dt) {
                        constexpr int t = n * (LPT / (MT * NT)) + decltype(dt)::value;
                        if constexpr (t < T::NLA) ca.template issue_one<t>(smem + T::a_slot_off(fill), wave);
                        else cb.template issue_one<t - T::NLA>(smem + T::b_slot_off(fill), wave);
                    });
                    __builtin_amdgcn_sched_barrier(0);
                });
                base_term(a1, KSTEPS * u - 1);
                advance_a();
                advance_b();
            } else {
                issue((u + STAGES - 1) % STAGES);
            }
            __builtin_amdgcn_sched_barrier(0);
            static_for<KSTEPS / 2>([&](auto qt) {
                constexpr int q = decltype(qt)::value;
                frags(std::integral_constant<int, 2 * q + 1>{}, a1, b1, slot);
                __builtin_amdgcn_sched_barrier(0);
                wait_lgkmcnt<FRAG_OPS>();                // a0/b0 landed; a1/b1 may still be in flight
                __builtin_amdgcn_sched_barrier(0);
                mma(a0, b0, KSTEPS * u + 2 * q);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (2 * q + 2 < KSTEPS) {
                    frags(std::integral_constant<int, 2 * q + 2>{}, a0, b0, slot);
                    __builtin_amdgcn_sched_barrier(0);
                    wait_lgkmcnt<FRAG_OPS>();
                    __builtin_amdgcn_sched_barrier(0);
                    mma(a1, b1, KSTEPS * u + 2 * q + 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            });
        }
        wait_vmcnt<0>();
        wait_lgkmcnt<0>();
        __builtin_amdgcn_sched_barrier(0);
        if (nsteps > 0) mma(a1, b1, KSTEPS * nsteps - 1);
    }
    __syncthreads();

    // ------------------------------------------------------------------------------ epilogues
    if constexpr (MI16) {
        // 16x16 accumulator tiles: the lane holds n = 4*(lane >> 4) .. +3 of row m = lane & 15 of tile
        // (i, j).  Two tile rows (32 rows of C) are staged through LDS at a time, then written as whole
        // 16-byte vectors along N.  16-bit outputs only (the launcher sends nothing else here).
        static_assert(EPI == EPI_STORE_BF16 || EPI == EPI_COMPOSE, "the 16x16x32 path stores 16-bit tiles");
        constexpr int ROW_BYTES = T::WN * 2 + 16;
        constexpr int CHUNKS_PER_ROW = T::WN * 2 / 16;
        constexpr int ROWS_PER_PASS = 64 / CHUNKS_PER_ROW;
        char* stg = smem + wave * T::EPI_BYTES_PER_WAVE;
        const int l16 = lane & 15, lq = lane >> 4;
        // Everything the stores need from the argument block, read once (left in place, each store would
        // fetch its share from memory again); per lane, one pointer that walks down the rows and the number
        // of rows below its first one that exist (zero when its columns do not).
        const int pM = p.M, pN = p.N;
        const int64_t row_step = (int64_t)p.ldc * 2 * ROWS_PER_PASS;
        const float alpha[2] = {p.alpha, p.alpha2};
        char* const cptr[2] = {reinterpret_cast<char*>(p.c), reinterpret_cast<char*>(p.c2)};
        const float* const colscale = p.colscale;
        const bf16_t* const colbias = p.colbias;
        const int ch = lane % CHUNKS_PER_ROW;
        const int mg0 = m0 + wm0 + lane / CHUNKS_PER_ROW, ng0 = n0 + wn0 + ch * 8;
        const int rows_left = (ng0 < pN) ? pM - mg0 : 0;
        // EPI_COMPOSE: pass 0 writes colscale[n] * acc (+ bias) to C (y = g (.) inner), pass 1 writes acc to C2
        // EPI_STORE_BF16 with a second output: pass 1 writes alpha2 * acc to C2
        const int npass = (cptr[1] != nullptr) ? 2 : 1;
        for (int pass = 0; pass < npass; ++pass) {
            char* ptr = cptr[pass] + ((int64_t)mg0 * p.ldc + ng0) * 2;
            const float al = alpha[pass];
#pragma unroll
            for (int ib = 0; ib < M16 / 2; ++ib) {
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int j = 0; j < N16; ++j) {
                        const int col = j * 16 + lq * 4;
                        const f32x4_t a = acc16[ib * 2 + half][j];
                        float v0, v1, v2, v3;
                        if (EPI == EPI_COMPOSE) {
                            float4 g4 = make_float4(1.f, 1.f, 1.f, 1.f);
                            uint2 b4 = make_uint2(0u, 0u);
                            if (pass == 0) {
                                const int ng = n0 + wn0 + col;
                                g4 = (ng < pN) ? *reinterpret_cast<const float4*>(colscale + ng) : make_float4(0.f, 0.f, 0.f, 0.f);
                                if (colbias && ng < pN) b4 = *reinterpret_cast<const uint2*>(colbias + ng);
                            }
                            v0 = fmaf(g4.x, a[0], E::lo(b4.x)); v1 = fmaf(g4.y, a[1], E::hi(b4.x));
                            v2 = fmaf(g4.z, a[2], E::lo(b4.y)); v3 = fmaf(g4.w, a[3], E::hi(b4.y));
                        } else {
                            v0 = al * a[0]; v1 = al * a[1]; v2 = al * a[2]; v3 = al * a[3];
                        }
                        uint2 o;
                        o.x = E::pack2(v0, v1);
                        o.y = E::pack2(v2, v3);
                        *reinterpret_cast<uint2*>(stg + (half * 16 + l16) * ROW_BYTES + col * 2) = o;
                    }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int ps = 0; ps < 32 / ROWS_PER_PASS; ++ps) {
                    const int row = ps * ROWS_PER_PASS + lane / CHUNKS_PER_ROW;
                    uint4 v = *reinterpret_cast<const uint4*>(stg + row * ROW_BYTES + ch * 16);
                    if (ib * 32 + ps * ROWS_PER_PASS < rows_left) *reinterpret_cast<uint4*>(ptr) = v;
                    ptr += row_step;
                }
            }
        }
        return;
    } else {
    // Everything the epilogues need from the argument block, read once: left in place, every use would fetch
    // its share from memory again (the block is selected at run time), each fetch a wait of its own.
    const int pM = p.M, pN = p.N, p_ksplit = p.ksplit, p_epilogue = p.epilogue;
    const int64_t p_ldc = p.ldc, p_ld_rowdot = p.ld_rowdot;
    const float p_alpha = p.alpha, p_alpha2 = p.alpha2;
    void* const p_c = p.c;
    void* const p_c2 = p.c2;
    const float* const p_colscale = p.colscale;
    const bf16_t* const p_colbias = p.colbias;
    const bf16_t* const p_rowdot = p.rowdot;
    float* const p_rowdot_partial = p.rowdot_partial;
    float* const p_base_sq_partial = p.base_sq_partial;
    // (a row-dot instance may carry a second problem that stores its fp32 tile instead: the Gram matrix riding
    // along with the cross term; it falls through to the store epilogue below)
    if (EPI == EPI_ROWDOT && p_epilogue == EPI_ROWDOT) {
        float* red = reinterpret_cast<float*>(smem);          // [WGN][BM] row-dot, then [WGN][BM] base_sq
        float* red2 = red + T::WGN * BM;
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            const int mg = m0 + wm0 + i * 32 + l32;
            float rs = 0.f;
            if (mg < pM) {
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int ng = n0 + wn0 + j * 32 + b * 8 + lh * 4;
                        if (ng < pN) {
                            uint2 rv = *reinterpret_cast<const uint2*>(p_rowdot + (int64_t)mg * p_ld_rowdot + ng);
                            rs = fmaf(acc[i][j][b * 4 + 0], E::lo(rv.x), rs);
                            rs = fmaf(acc[i][j][b * 4 + 1], E::hi(rv.x), rs);
                            rs = fmaf(acc[i][j][b * 4 + 2], E::lo(rv.y), rs);
                            rs = fmaf(acc[i][j][b * 4 + 3], E::hi(rv.y), rs);
                        }
                    }
            }
            rs += __shfl_xor(rs, 32);
            float bq = bsq[i] + __shfl_xor(bsq[i], 32);
            if (lh == 0) {
                red[wn * BM + wm0 + i * 32 + l32] = rs;
                red2[wn * BM + wm0 + i * 32 + l32] = bq;
            }
        }
        __syncthreads();
        if (tid < BM && m0 + tid < pM) {
            float v = red[tid], q = red2[tid];
            for (int w = 1; w < T::WGN; ++w) { v += red[w * BM + tid]; q += red2[w * BM + tid]; }
            p_rowdot_partial[(int64_t)(tc.z * tiles_n + tc.tn) * pM + m0 + tid] = v;
            if (want_bsq) p_base_sq_partial[(int64_t)tc.z * pM + m0 + tid] = q;
        }
        return;
    }

    // STORE: stage each 32-row band of the wave's sub-tile through LDS, then write whole 16-byte
    // vectors along N.
    constexpr bool OUT_BF16 = (EPI == EPI_STORE_BF16) || (EPI == EPI_COMPOSE);
    constexpr int ESZ = OUT_BF16 ? 2 : 4;
    constexpr int ROW_BYTES = T::WN * ESZ + 16;
    constexpr int CHUNKS_PER_ROW = T::WN * ESZ / 16;
    constexpr int ROWS_PER_PASS = 64 / CHUNKS_PER_ROW;
    char* stg = smem + wave * T::EPI_BYTES_PER_WAVE;
    // EPI_COMPOSE: pass 0 writes colscale[n] * acc to C (y = g (.) inner), pass 1 writes acc to C2 (inner)
    // (the per-column scale and bias are re-read for every 32-row band: sixteen float4 per lane kept
    // across the whole epilogue would not fit beside 256 accumulators)
    // EPI_STORE_BF16 with a second output: pass 1 writes alpha2 * acc to C2
    const int npass = ((EPI == EPI_COMPOSE || EPI == EPI_STORE_BF16) && p_c2 != nullptr) ? 2 : 1;
    for (int pass = 0; pass < npass; ++pass) {
    char* cbase = reinterpret_cast<char*>(pass == 0 ? p_c : p_c2) +
                  (p_ksplit > 1 ? (int64_t)tc.z * pM * p_ldc * ESZ : 0);
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int col = j * 32 + b * 8 + lh * 4;
                float v0, v1, v2, v3;
                if (EPI == EPI_COMPOSE) {
                    float4 g4 = make_float4(1.f, 1.f, 1.f, 1.f);
                    uint2 b4 = make_uint2(0u, 0u);
                    if (pass == 0) {
                        const int ng = n0 + wn0 + col;
                        g4 = (ng < pN) ? *reinterpret_cast<const float4*>(p_colscale + ng) : make_float4(0.f, 0.f, 0.f, 0.f);
                        if (p_colbias && ng < pN) b4 = *reinterpret_cast<const uint2*>(p_colbias + ng);
                    }
                    v0 = fmaf(g4.x, acc[i][j][b * 4 + 0], E::lo(b4.x)); v1 = fmaf(g4.y, acc[i][j][b * 4 + 1], E::hi(b4.x));
                    v2 = fmaf(g4.z, acc[i][j][b * 4 + 2], E::lo(b4.y)); v3 = fmaf(g4.w, acc[i][j][b * 4 + 3], E::hi(b4.y));
                } else {
                    const float al = (pass == 0) ? p_alpha : p_alpha2;
                    v0 = al * acc[i][j][b * 4 + 0]; v1 = al * acc[i][j][b * 4 + 1];
                    v2 = al * acc[i][j][b * 4 + 2]; v3 = al * acc[i][j][b * 4 + 3];
                }
                if (OUT_BF16) {
                    uint2 o;
                    o.x = E::pack2(v0, v1);
                    o.y = E::pack2(v2, v3);
                    *reinterpret_cast<uint2*>(stg + l32 * ROW_BYTES + col * 2) = o;
                } else {
                    *reinterpret_cast<float4*>(stg + l32 * ROW_BYTES + col * 4) = make_float4(v0, v1, v2, v3);
                }
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int ps = 0; ps < 32 / ROWS_PER_PASS; ++ps) {
            const int row = ps * ROWS_PER_PASS + lane / CHUNKS_PER_ROW;
            const int ch = lane % CHUNKS_PER_ROW;
            uint4 v = *reinterpret_cast<const uint4*>(stg + row * ROW_BYTES + ch * 16);
            const int mg = m0 + wm0 + i * 32 + row;
            const int ng = n0 + wn0 + ch * (16 / ESZ);
            if (mg < pM && ng < pN)
                *reinterpret_cast<uint4*>(cbase + ((int64_t)mg * p_ldc + ng) * ESZ) = v;
        }
    }
    }
    }  // !MI16
}

template <class T>
int grid_of(const GemmArgs& a)
{
    if (a.M <= 0 || a.N <= 0) return 0;
    return ((a.M + T::BM - 1) / T::BM) * ((a.N + T::BN - 1) / T::BN) * a.ksplit;
}

template <class T, bool A_KC, bool B_KC, int EPI>
hipError_t launch_one(const GemmArgs& a, const GemmArgs* b, hipStream_t stream)
{
    GemmPair grp;
    grp.g[0] = a;
    grp.g[1] = b ? *b : a;
    grp.count0 = grid_of<T>(a);
    const int grid = grp.count0 + (b ? grid_of<T>(*b) : 0);
    if (grid == 0) return hipSuccess;
    if (b && b->dt != a.dt) return hipErrorInvalidValue;
    if (a.dt == DT_F16) {
        if (a.tag) gemm_bf16_kernel<T, A_KC, B_KC, EPI, 1, DT_F16><<<dim3(grid), dim3(T::THREADS), 0, stream>>>(grp);
        else gemm_bf16_kernel<T, A_KC, B_KC, EPI, 0, DT_F16><<<dim3(grid), dim3(T::THREADS), 0, stream>>>(grp);
    } else {
        if (a.tag) gemm_bf16_kernel<T, A_KC, B_KC, EPI, 1, DT_BF16><<<dim3(grid), dim3(T::THREADS), 0, stream>>>(grp);
        else gemm_bf16_kernel<T, A_KC, B_KC, EPI, 0, DT_BF16><<<dim3(grid), dim3(T::THREADS), 0, stream>>>(grp);
    }
    return hipGetLastError();
}

bool use_big(const GemmArgs& a)
{
    // the large tile pays off once it still yields a few tiles per CU
    int64_t big_tiles = (int64_t)((a.M + 255) / 256) * ((a.N + 255) / 256);
    return (a.epilogue == EPI_STORE_BF16 || a.epilogue == EPI_COMPOSE) && a.ksplit == 1 && big_tiles >= 256;
}

hipError_t dispatch(const GemmArgs& a, const GemmArgs* b, hipStream_t stream)
{
    const bool big = use_big(a);
    // at most one 128x128-tile workgroup per CU: give it the deep ring
    const bool deep = !big && (grid_of<TileMed>(a) + (b ? grid_of<TileMed>(*b) : 0)) <= 256;
#define DORA_GEMM_MED(AKC, BKC, E) \
    (deep ? launch_one<TileMedDeep, AKC, BKC, E>(a, b, stream) : launch_one<TileMed, AKC, BKC, E>(a, b, stream))
#define DORA_GEMM_CASE(AKC, BKC, E)                                                     \
    if (a.a_kcontig == (AKC) && a.b_kcontig == (BKC) && a.epilogue == (E))              \
        return big ? launch_one<TileBig, AKC, BKC, E>(a, b, stream) : DORA_GEMM_MED(AKC, BKC, E);
    DORA_GEMM_CASE(true, true, EPI_STORE_BF16)
    DORA_GEMM_CASE(true, false, EPI_STORE_BF16)
    DORA_GEMM_CASE(true, true, EPI_COMPOSE)
#undef DORA_GEMM_CASE
#define DORA_GEMM_CASE_MED(AKC, BKC, E)                                                 \
    if (a.a_kcontig == (AKC) && a.b_kcontig == (BKC) && a.epilogue == (E))              \
        return DORA_GEMM_MED(AKC, BKC, E);
    DORA_GEMM_CASE_MED(true, true, EPI_STORE_F32)
    DORA_GEMM_CASE_MED(true, false, EPI_STORE_F32)
    DORA_GEMM_CASE_MED(true, true, EPI_ROWDOT)
    DORA_GEMM_CASE_MED(false, false, EPI_STORE_F32)
#undef DORA_GEMM_CASE_MED
#undef DORA_GEMM_MED
    return hipErrorInvalidValue;
}

}  // namespace

int gemm_bf16_tiles_n(const GemmArgs& a) { return (a.N + TileMed::BN - 1) / TileMed::BN; }

hipError_t launch_gemm_bf16(const GemmArgs& a, int trace_id, hipStream_t stream)
{
    if (a.M == 0 || a.N == 0) return hipSuccess;
    TraceScope ts(trace_id, stream);
    return dispatch(a, nullptr, stream);
}

hipError_t launch_gemm_bf16_pair(const GemmArgs& a, const GemmArgs& b, int trace_id, hipStream_t stream)
{
    // both problems run the same kernel instance: same operand layouts and element type; same epilogue without
    // split-K, or a row-dot problem (split or not) followed by an fp32-store problem (split or not)
    const bool same = a.epilogue == b.epilogue && a.ksplit == 1 && b.ksplit == 1;
    const bool rowdot_then_store = a.epilogue == EPI_ROWDOT && b.epilogue == EPI_STORE_F32 && b.nseg == 1;
    if (a.a_kcontig != b.a_kcontig || a.b_kcontig != b.b_kcontig || a.dt != b.dt || !(same || rowdot_then_store))
        return hipErrorInvalidValue;
    if ((a.M == 0 || a.N == 0) && (b.M == 0 || b.N == 0)) return hipSuccess;
    TraceScope ts(trace_id, stream);
    return dispatch(a, &b, stream);
}

}  // namespace dora
