// gfx950 kernels of libppd: paged KV append, the one-launch mixed attention kernel (narrow tiles for
// decode-like rows, MFMA row-block tiles for append-prefill / full prefill) and the log-sum-exp merge of
// split partials.
//
// Operation (paper section 4.1, "Full Prefill vs. Append Prefill"; L = cached, n = new): new row j of a
// sequence attends to keys 0 .. L + j, all read from the page pool.  Both tile kinds compute the
// transposed products  S^T = K Q^T  and  O^T = V^T P^T  so that the accumulator layout of the first
// product is already the operand layout of the second, and every per-row softmax quantity lives in the
// lane that owns the row's column.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "ppd_internal.h"

#ifndef PPD_PINGPONG
#define PPD_PINGPONG 1  // 0: all waves take the loop barrier at the end of the iteration; 1: waves 4..7 mid-iteration
#endif

namespace ppd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define NEG_INF (-__builtin_inff())

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2 f = {a, b};
    bf16x2 r = __builtin_convertvector(f, bf16x2);  // round to nearest even
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// Query row of a column of a row block (columns are row-major over the G query heads of the group): col / G
// with inv = 65536 / G + 1, exact for col < 4096 and G <= 16.
__device__ __forceinline__ int col_row(int col, int inv) { return (int)(((unsigned)col * (unsigned)inv) >> 16); }

__device__ __forceinline__ float xor_shuffle(float v, int mask) { return __shfl_xor(v, mask, 64); }

// max / sum of v over lanes l and l^32 (v_permlane32_swap: no LDS round trip).  The instruction exchanges
// the upper half of its first register with the lower half of its second.  It is written as inline asm on
// two copies of v (the builtin's second result was folded into the first by the compiler when both inputs
// hold the same value); the s_nop cover the VALU-write -> permlane-read wait states on both sides.
__device__ __forceinline__ void swap_halves(float v, float* lo, float* hi) {
    float a = v, b = v;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    *lo = a;  // {v[0..31], v[0..31]}
    *hi = b;  // {v[32..63], v[32..63]}
}
__device__ __forceinline__ float max_halves(float v) {
    float lo, hi;
    swap_halves(v, &lo, &hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_halves(float v) {
    float lo, hi;
    swap_halves(v, &lo, &hi);
    return lo + hi;
}

// The running maximum is only raised (and the accumulators rescaled) when it would grow by more than this many
// powers of two; until then probabilities may exceed 1, by at most 2^kLazyRescale.  The final o / l is unchanged.
#ifndef kLazyRescale
#define kLazyRescale 8.0f
#endif

// Raw page-table entry of logical page `pi` of a sequence; pi is clamped so that no access leaves the page
// table row.  The value is NOT inspected here: a caller that prefetches it must not wait for the load.
__device__ __forceinline__ int load_page_id(const int32_t* pt_row, int pi, int last_page) {
    pi = pi < last_page ? pi : last_page;
    return pt_row[pi];
}

// Checks a page id at the point of use: an id outside the pool raises the sticky flag and is replaced by
// page 0, so that no access leaves the pool.
__device__ __forceinline__ int64_t checked_page(const KParams& P, int page) {
    if (page < 0 || page >= P.num_pages) {
        atomicOr(&P.counters[9], 2u);
        page = 0;
    }
    return page;
}

// FP8 pages hold OCP FP8 E4M3 codes (1 sign, 4 exponent bits of bias 7, 3 mantissa bits).  Every code's value is a
// bf16 number, so the tiles turn codes into bf16 MFMA operands exactly; the tensor's scale is applied once, to the
// scores (K) and to the final output (V).
// Four codes of a dword -> four bf16, in order (the conversion instruction takes the two codes of one 16-bit half).
__device__ __forceinline__ u32x2 fp8x4_to_bf16x4(uint32_t w) {
    const bf16x2 lo = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
    const bf16x2 hi = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true);
    return u32x2{__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
}
__device__ __forceinline__ u32x4 fp8x8_to_bf16x8(u32x2 w) {
    const u32x2 a = fp8x4_to_bf16x4(w[0]), b = fp8x4_to_bf16x4(w[1]);
    return u32x4{a[0], a[1], b[0], b[1]};
}

// Code of a binary32 value: nearest, ties to the even code, magnitudes from 448 on (infinities included) saturate
// to 448, NaN gives the NaN code.  Integer arithmetic on the bits, so that the stored byte does not depend on any
// conversion instruction's treatment of ties, overflow or subnormals.
__device__ __forceinline__ uint32_t e4m3_code(float y) {
    const uint32_t u = __builtin_bit_cast(uint32_t, y);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t a = u & 0x7FFFFFFFu;
    uint32_t code;
    if (a > 0x7F800000u) {
        code = 0x7Fu;
    } else if (a >= 0x43E00000u) {  // 448.0f
        code = 0x7Eu;
    } else if (a >= 0x3C800000u) {  // 2^-6, the smallest normal: round the mantissa at bit 20, re-bias 127 -> 7
        const uint32_t r = a + 0x7FFFFu + ((a >> 20) & 1u);
        code = (r >> 20) - (120u << 3);
    } else {                        // subnormal codes are multiples of 2^-9 (8 is the smallest normal's code)
        code = (uint32_t)__builtin_rintf(__builtin_bit_cast(float, a) * 512.0f);
    }
    return sign | code;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits) { return __builtin_bit_cast(float, bits << 16); }

// Zeroes the bf16 elements e of a granule of 8 tokens whose position first + e is >= kv_total (never written).
__device__ __forceinline__ u32x4 zero_unwritten(u32x4 v, int first, int kv_total) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (first + e >= kv_total) v[e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
    return v;
}

// ---------------------------------------------------------------------------------------------------
// MFMA row-block tile: up to kMfmaCols query columns (rows x G heads of one KV head) against keys
// [kv_begin, kv_end).  kWaves waves x 32 columns; key tiles of 64 tokens (4 pages); v_mfma_f32_32x32x16_bf16 for
// both products.  K and V tiles go from the pool straight into LDS (global_load_lds, 16 bytes per lane, no
// staging registers), each in a ring.  With NS = kStages tiles of prefetch distance and rings of NS + 1 stages:
//   iteration i:  loads K(i+NS) -> Kring[(i+NS) % (NS+1)], V(i+NS-1) -> Vring[(i+NS-1) % (NS+1)]
//                 vector phase on S^T(i); matrix phase reads V(i) and K(i+1)
//   one barrier per iteration, after K(i+2) and V(i+1) have landed (loads issued in the last NS-2 iterations may
//   still be in flight); half of the waves take it between their two phases (see the loop).
// ---------------------------------------------------------------------------------------------------
// 16 bytes per lane from global memory straight into LDS: lane i of the wave writes lds_base + 16*i
// (lds_base is wave-uniform and travels in M0).  Written as inline asm so that the compiler's wait-count pass
// does not see an LDS write it would have to order every later LDS read behind (it would drain the memory
// counter before the first operand read of each tile); completion is awaited explicitly with s_waitcnt vmcnt.
// The global address is a wave-uniform base (scalar register pair) plus a 32-bit byte offset per lane.
__device__ __forceinline__ void lds_direct_load16(const void* gbase, uint32_t lane_off, const char* lds_base) {
    const uint32_t lds_off = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lds_base;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_off), "s"(gbase), "s"(__builtin_amdgcn_readfirstlane(lds_off))
                 : "memory", "m0");
}

// HALF = false: the vector phase covers the 64 keys of a tile, then the matrix phase (the loop described above).
// HALF = true: the same tile is worked in two halves of 32 keys -- vector phase, matrix phase, vector phase, matrix
// phase -- with S^T of 32 keys and half of the packed probabilities live at a time: 24 registers less per lane,
// which is what lets two such waves and a stream wave share a SIMD (three waves of 168 registers).  The late waves
// then take the loop barrier between the second vector phase and the second matrix phase.
// LDS byte address of p as an opaque 32-bit register value: operand reads then address LDS as this register plus a
// compile-time offset below 64 KiB, which fits the instruction's offset field (left to itself the compiler folds
// ring and stage offsets into constants beyond that field and spends one vector add per read).
// (x + k) mod N for 0 <= x, k < N
template <int N>
__device__ __forceinline__ int ring_add(int x, int k) {
    if constexpr ((N & (N - 1)) == 0) return (x + k) & (N - 1);
    const int y = x + k;
    return y >= N ? y - N : y;
}
// The same with the LDS byte address given as a wave-uniform integer (no pointer cast per load).
__device__ __forceinline__ void lds_direct_load16_at(const void* gbase, uint32_t lane_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_off), "s"(gbase), "s"(lds_addr)
                 : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_base(const char* p) {
    uint32_t a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
    asm volatile("" : "+v"(a));
    return a;
}
__device__ __forceinline__ u32x4 lds_read16(uint32_t base, int offset) {
    return *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(base + (uint32_t)offset);
}

// FP8 (pages of one-byte codes): the loads land the tile's codes in a staging ring of their own (half the bytes, NS - 1
// stages of K and of V), and at the end of the iteration before a tile is first read every thread turns the 16 codes it
// loaded itself into bf16 in the operand rings -- once per workgroup, not once per wave and operand read -- so the
// loop's matrix and vector phases are the ones of bf16 pages.  The operand rings then need three stages each (the tile
// being written, the one the early waves read and the one the late waves read), which with the staging ring is the same
// LDS as the four-stage rings of bf16 pages.
template <int HD, bool HALF, bool FP8 = false>
__device__ __forceinline__ void mfma_item(const KParams& P, const ppd_work_item& it, char* smem) {
    static_assert(!(FP8 && HALF), "FP8 pages are read by the full-tile loop only");
    static_assert(!FP8 || kStages == 3, "the staging of FP8 tiles is written for a prefetch distance of 3");
    constexpr int EB = FP8 ? 1 : 2;            // bytes per pool element
    constexpr int PB = kPage * HD * 2;         // bytes of one (page, head) block of K or of V as bf16 operands in LDS
    constexpr int GPP = PB / 16;               // 16-byte granules per such block
    constexpr int KBYTES = 4 * PB;             // one stage: 4 pages of K (or of V)
    constexpr int NS = kStages;
    constexpr int NSV = FP8 ? 3 : kStages + (PPD_PINGPONG ? 1 : 0);  // the late half of the waves reads V one barrier later
    constexpr int NSK = FP8 ? 3 : kStages + (PPD_PINGPONG ? 1 : 0);  // ... and K as well
    constexpr int VRING = NSK * KBYTES;        // LDS: K ring at 0, V ring behind it
    constexpr int LPB = PB / 2 * EB;           // bytes of a block as the loads move it
    constexpr int LGPP = LPB / 16;             // 16-byte granules per loaded block
    constexpr int LBYTES = 4 * LPB;            // one loaded tile of K (or of V)
    constexpr int LOADERS = 4 * LGPP < kThreads ? 4 * LGPP : kThreads;  // threads that load (all, or the first waves)
    constexpr int ROUNDS = 4 * LGPP / LOADERS; // granules of K (and of V) each loading thread moves per tile
    constexpr int NST = NS - 1;                // FP8: stages of the staging ring of K, and of V
    constexpr int STAGE_K = (NSK + NSV) * KBYTES, STAGE_V = STAGE_K + NST * LBYTES;
    constexpr int IDS_AT = (NSK + NSV) * KBYTES + (FP8 ? 2 * NST * LBYTES : 0);
    static_assert(IDS_AT <= (2 * kStages + 2 * (PPD_PINGPONG ? 1 : 0)) * KBYTES, "the kernel's LDS is sized for the bf16 rings");
    constexpr int KS = HD / 16;                // k-steps of S^T = K Q^T
    constexpr int DB = HD / 32;                // 32-row d blocks of O^T

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5;
    const int l32 = lane & 31;
    const int G = P.G;
    const int ncols = it.nrows * G;
    const int col = wave * 32 + l32;
    const int colc = col < ncols ? col : ncols - 1;
    const int jrow = col_row(colc, P.invG);
    const int head = it.kvh * G + (colc - jrow * G);
    const int limit = it.L + it.row0 + jrow;  // last key position this column may see
    const bool wave_active = wave * 32 < ncols;
    const int wmin_limit = it.L + it.row0 + col_row((wave * 32) < ncols ? wave * 32 : ncols - 1, P.invG);

    // Q^T operand: column = lane % 32, d = ks*16 + (lane/32)*8 .. +8
    bf16x8 qreg[KS];
    {
        const uint16_t* qp = P.q + ((int64_t)(it.grow0 + jrow) * P.Hq + head) * HD + h * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4*>(qp + ks * 16));
    }

    const int32_t* pt_row = P.page_tables + (int64_t)it.seq * P.max_pages;
    const int last_page = (it.kv_total - 1) >> 4;
    const int first_page = it.kv_begin >> 4;
    const int ntiles = (it.kv_end - it.kv_begin + kTileTokens - 1) / kTileTokens;
    const int64_t head_off = (int64_t)it.kvh * (kPage * HD);
    const int64_t v_off = (int64_t)P.Hkv * (kPage * HD);

    // Page ids of the whole key range go to LDS once, checked, before the loop (at most 2048: the planner
    // caps a row-block tile at kMaxMfmaChunk keys); a tile reads its four ids with one broadcast LDS read.  Nothing in
    // the loop then depends on a page-table load, so no wait on the memory counter is needed there.
    // Granule gid = r*256 + tid ... of the tile's 4 page blocks goes to LDS byte gid*16 of the stage: a wave writes
    // 1 KiB contiguous per round, which is what a wave-wide LDS-direct load does.  The page a wave reads in
    // round r is wave-uniform, s = r * (kThreads / GPP) + (wave * 64) / GPP, and the lane's offset inside the
    // page block is the same in every round: the load's address is a scalar base plus a per-lane constant.
    constexpr int PAGES_PER_ROUND = LOADERS / LGPP;
    static_assert(LOADERS % 64 == 0 && LOADERS % LGPP == 0 && ROUNDS * PAGES_PER_ROUND == 4, "one round covers whole page blocks");
    static_assert(!FP8 || ROUNDS == 1, "a thread stages one granule of codes per tile");
    const bool loader = LOADERS == kThreads || tid < LOADERS;  // wave-uniform
    const int page_sel = loader ? (wave * 64) / LGPP : 0;
    const uint32_t lane_off = (uint32_t)(tid % LGPP) * 16u;
    // The pages this wave loads from, one per round, as byte offsets of the page in the pool: the id read from LDS
    // becomes a scalar and the 64-bit product is made once per tile on the scalar unit (a page is at most 8 MiB, so
    // its size fits 32 bits); a load then costs two scalar additions for its global address and two for its LDS
    // address.
    struct TilePages { uint32_t lo[ROUNDS], hi[ROUNDS]; };
    int* lds_ids = reinterpret_cast<int*>(smem + IDS_AT);
    for (int i = tid; i < ntiles * 4; i += kThreads)
        lds_ids[i] = (int)checked_page(P, load_page_id(pt_row, first_page + i, last_page));
    struct RawPages { int p[ROUNDS]; };  // the ids as they come from LDS (vector registers)
    const uint32_t page_bytes = (uint32_t)P.page_stride * EB;
    auto tile_pages_raw = [&](int ti) {
        RawPages t;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) t.p[r] = lds_ids[ti * 4 + r * PAGES_PER_ROUND + page_sel];
        return t;
    };
    auto to_scalar = [&](const RawPages& v) {
        TilePages t;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const uint32_t id = (uint32_t)__builtin_amdgcn_readfirstlane(v.p[r]);
            if constexpr (FP8) {  // this kernel has no scalar registers to spare for the pair: the product is made at the load
                t.lo[r] = id;
                t.hi[r] = 0;
            } else {
                const uint64_t off = (uint64_t)id * page_bytes;
                t.lo[r] = (uint32_t)off;
                t.hi[r] = (uint32_t)(off >> 32);
            }
        }
        return t;
    };
    auto tile_pages = [&](int ti) { return to_scalar(tile_pages_raw(ti)); };
    // Workgroup barrier for LDS traffic only: unlike __syncthreads() it does not drain the memory counter, so
    // LDS-direct loads of later tiles stay in flight across it.
    auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    const char* const pool_k = reinterpret_cast<const char*>(P.pool) + head_off * EB;  // this KV head's K block of page 0
    const char* const pool_v = pool_k + v_off * EB;                                    // ... and its V block
    const uint32_t smem_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)smem) + (uint32_t)wave * 1024u;
    auto load_block = [&](const TilePages& t, int lds_byte, bool is_v) {
        if (!loader) return;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const uint64_t off = FP8 ? (uint64_t)t.lo[r] * page_bytes : (((uint64_t)t.hi[r] << 32) | t.lo[r]);
            const char* base = (is_v ? pool_v : pool_k) + off;
            lds_direct_load16_at(base, lane_off, smem_addr + (uint32_t)(lds_byte + r * (kThreads * 16)));
        }
    };
    // FP8: the 16 codes this thread staged at src_byte become two bf16 granules of the operand tile at dst_byte (the
    // element order of a tile is the same in both); V rows of positions >= kv_total were never written and become 0.
    auto convert_staged = [&](int src_byte, int dst_byte, bool is_v, int tile) {
        if (!loader) return;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(smem + src_byte + tid * 16);
        u32x4 lo = fp8x8_to_bf16x8(u32x2{raw[0], raw[1]}), hi = fp8x8_to_bf16x8(u32x2{raw[2], raw[3]});
        if (is_v) {
            const int tile_base = it.kv_begin + tile * kTileTokens;
            if (tile_base + kTileTokens > it.kv_total) {
                const int g0 = 2 * tid, g1 = 2 * tid + 1;  // bf16 granules of the tile: page g / GPP, (octet, d) = g % GPP
                lo = zero_unwritten(lo, tile_base + (g0 / GPP) * 16 + ((g0 % GPP) / HD) * 8, it.kv_total);
                hi = zero_unwritten(hi, tile_base + (g1 / GPP) * 16 + ((g1 % GPP) / HD) * 8, it.kv_total);
            }
        }
        u32x4* dst = reinterpret_cast<u32x4*>(smem + dst_byte + tid * 32);
        dst[0] = lo;
        dst[1] = hi;
    };
    // V rows of positions >= kv_total were never written: zero them in LDS (each thread fixes the granules it
    // loaded itself, after its own loads have landed).  Only the sequence's last tile needs it.
    auto fix_v_tail = [&](int ti, int lds_byte) {
        const int tile_base = it.kv_begin + ti * kTileTokens;
        if (tile_base + kTileTokens > it.kv_total) {
#pragma unroll
            for (int r = 0; r < ROUNDS; ++r) {
                const int gid = r * kThreads + tid;
                const int s = gid / GPP, within = gid % GPP;
                u32x4* cell = reinterpret_cast<u32x4*>(smem + lds_byte + gid * 16);
                *cell = zero_unwritten(*cell, tile_base + s * 16 + (within / HD) * 8, it.kv_total);
            }
        }
    };
    // Loads retire in order: waiting until at most `newer` are outstanding guarantees everything issued
    // before those has landed in LDS.
    auto wait_all_loads = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
    // all but the loads of the last NS - 2 iterations (2*ROUNDS each): K(ti+2) and V(ti+1) were issued before those
    auto wait_older_loads = [&]() {
        constexpr int kKeep = (NS - 2) * 2 * ROUNDS;
        static_assert(kKeep < 64, "the memory counter has six bits");
        // s_waitcnt immediate on gfx9: vmcnt in bits 3:0 and 15:14, expcnt (7 = no wait) in 6:4, lgkmcnt (15) in 11:8
        __builtin_amdgcn_s_waitcnt((kKeep & 15) | ((kKeep >> 4) << 14) | (7 << 4) | (15 << 8));
        asm volatile("" ::: "memory");
    };

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m_run = NEG_INF, l_run = 0.f;
    const float c = P.scale_log2e;

    // K operand row of this lane inside a 32-token block: MFMA row r holds token
    //   page = bit4(r), token-in-page = 8*bit2(r) + 4*bit3(r) + (r & 3)
    // so that accumulator registers 8*s2 .. 8*s2+7 of a lane are 8 consecutive tokens of one page.
    const int k_tok = ((l32 >> 2) & 1) * 8 + ((l32 >> 3) & 1) * 4 + (l32 & 3);
    const int k_lane_off = (l32 >> 4) * PB + k_tok * 16 + h * 256;  // + stage + tb*2*PB + ks*512
    const int v_lane_off = VRING + (h * HD + l32) * 16;             // + stage + s*PB + db*512

    auto qk_tile = [&](int stage, f32x16 (&sacc)[2]) {
        const uint32_t kb = lds_base(smem + stage * KBYTES + k_lane_off);
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[tb][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
                bf16x8 a = as_bf16x8(lds_read16(kb, tb * 2 * PB + ks * 512));
                sacc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sacc[tb], 0, 0, 0);
            }
    };

    // prologue: K(0..NS-1) and V(0..NS-2) are issued, K(0), K(1), V(0) must land; S^T of tile 0
    __syncthreads();  // page ids are in LDS
    if constexpr (FP8) {
        // K(0), K(1) and V(0) are staged and converted; K(2) and V(1) are then issued into the slots of K(0) and beside V(0)
        const TilePages tp0 = tile_pages(0), tp1 = tile_pages(1 < ntiles ? 1 : 0);
        load_block(tp0, STAGE_K, false);
        load_block(tp0, STAGE_V, true);
        if (1 < ntiles) load_block(tp1, STAGE_K + LBYTES, false);
        wait_all_loads();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(qreg[ks]));
        convert_staged(STAGE_K, 0, false, 0);
        if (1 < ntiles) convert_staged(STAGE_K + LBYTES, KBYTES, false, 1);
        convert_staged(STAGE_V, VRING, true, 0);
        if (2 < ntiles) load_block(tile_pages(2), STAGE_K, false);
        if (1 < ntiles) load_block(tp1, STAGE_V + LBYTES, true);
    } else {
#pragma unroll
        for (int t = 0; t < NS; ++t) {
            if (t < ntiles) {
                const TilePages tp = tile_pages(t);
                load_block(tp, t * KBYTES, false);
                if (t < NS - 1) load_block(tp, VRING + t * KBYTES, true);
            }
        }
        wait_all_loads();
        // The compiler does not count the asm loads; make it settle its own pending loads (the Q operand) here, or
        // it would place ever-decreasing memory-counter waits at their first use inside the loop and drain the
        // LDS-direct loads in flight there.
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(qreg[ks]));
#pragma unroll
        for (int t = 0; t < NS - 1; ++t)
            if (t < ntiles) fix_v_tail(t, VRING + t * KBYTES);
    }
    lds_barrier();
    if constexpr (!HALF) {
    f32x16 s_cur[2];
    if (wave_active) qk_tile(0, s_cur);
    lds_barrier();  // with rings of NS stages the first iteration's loads overwrite K stage 0
    int st_cur = 0;   // ti % NS
    int sv_cur = 0;   // ti % NSV: V stage of tile ti
    // Two waves share a SIMD, and a wave issues in order.  An iteration is a vector phase (mask, max, rescale, the
    // tile's exponentials, packed to bf16) followed by a matrix phase (O^T += V^T P^T of this tile, then S^T of the
    // next tile into the registers the probabilities have left), each pure, so that one wave's matrix phase can
    // run under the other's vector phase.  Left alone the two waves would run the same phase at the same time
    // (the loop barrier aligns them); the "late" half of the waves therefore takes the barrier between its two
    // phases instead of at the end of the iteration, which locks it half an iteration behind the other half.
    // A late wave reads V(ti) and K(ti+1) after the barrier at which the early waves start loading V(ti+NS) and
    // K(ti+1+NS): one more stage in each ring (measured: +4.5 % with the shift, -9 % with pure phases alone).
#if PPD_PINGPONG
    const bool late = wave >= kWaves / 2;  // waves w and w + 4 share a SIMD
#else
    const bool late = false;
#endif

    u32x4 pw[4];  // the tile's probabilities as bf16, B operand of the four 16-key steps of the PV product
    TilePages tp_v = tile_pages(NS - 1 < ntiles ? NS - 1 : ntiles - 1);  // pages of the loads the first iteration issues
    TilePages tp_k = tile_pages(NS < ntiles ? NS : ntiles - 1);
    for (int ti = 0; ti < ntiles; ++ti) {
        const int st_nxt = st_cur + 1 == NSK ? 0 : st_cur + 1;           // (ti + 1) % NSK
        const int st_far = ring_add<NSK>(st_cur, NS % NSK);                           // (ti + NS) % NSK
        const int sv_nxt = sv_cur + 1 == NSV ? 0 : sv_cur + 1;           // (ti + 1) % NSV
        const int sv_far = ring_add<NSV>(sv_cur, (NS - 1) % NSV);                       // (ti + NS - 1) % NSV
        const bool full_issue = ti + NS < ntiles;
        if constexpr (FP8) {  // tile t of K or of V is staged in slot t % 2
            if (ti + NS - 1 < ntiles) load_block(tp_v, STAGE_V + (ti & 1) * LBYTES, true);
            if (full_issue) load_block(tp_k, STAGE_K + ((ti + 1) & 1) * LBYTES, false);
        } else {
            if (ti + NS - 1 < ntiles) load_block(tp_v, VRING + sv_far * KBYTES, true);
            if (full_issue) load_block(tp_k, st_far * KBYTES, false);
        }
        // The V tile of the next iteration is this iteration's K tile; the ids of its K tile are read from LDS
        // now and turned into scalars at the end of the iteration: under the other waves' operand reads that
        // small LDS read takes hundreds of cycles, which nothing waits for this way.
        tp_v = tp_k;
        const RawPages tp_raw = tile_pages_raw(ti + 1 + NS < ntiles ? ti + 1 + NS : ntiles - 1);
        // K(ti+2) and V(ti+1) must have landed before the barrier; with NS = 3 the loads issued in this iteration
        // may stay in flight
        auto close_iteration = [&]() {
            if (full_issue)  // then the last NS - 2 iterations all issued their full share
                wait_older_loads();
            else
                wait_all_loads();
            if constexpr (FP8) {
                if (ti + 2 < ntiles) convert_staged(STAGE_K + (ti & 1) * LBYTES, ring_add<NSK>(st_cur, 2 % NSK) * KBYTES, false, ti + 2);
                if (ti + 1 < ntiles) convert_staged(STAGE_V + ((ti + 1) & 1) * LBYTES, VRING + sv_nxt * KBYTES, true, ti + 1);
            } else {
                if (ti + 1 < ntiles) fix_v_tail(ti + 1, VRING + sv_nxt * KBYTES);
            }
            lds_barrier();
        };
        float mc = 0.f;
        if (wave_active) {
            const int tile_base = it.kv_begin + ti * kTileTokens;
            if (tile_base + kTileTokens - 1 > wmin_limit) {  // causal boundary crosses this tile
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int pos = tile_base + (tb * 2 + (i >> 3)) * 16 + h * 8 + (i & 7);
                        if (pos > limit) s_cur[tb][i] = NEG_INF;
                    }
            }
            float mx = s_cur[0][0];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s_cur[tb][i]);
            mx = max_halves(mx);
            const float m_new = fmaxf(m_run, mx);
            if (__any((m_new - m_run) * c > kLazyRescale)) {  // -inf -> finite counts; -inf -> -inf does not
                const float m_use = m_new == NEG_INF ? 0.f : m_new;
                const float alpha = fast_exp2(m_run * c - m_use * c);  // m_run = -inf gives 0
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
                m_run = m_new;
            }
            mc = m_run == NEG_INF ? 0.f : m_run * c;
            // Vector phase: all exponentials of this tile, packed to bf16 at once.  Nothing for the matrix pipe in
            // it, and nothing for the vector pipe in the matrix phase below, so that the late waves (half an
            // iteration behind) run their matrix phase under this vector phase and the other way round.
            float psum = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i0 = (s & 1) * 8 + 2 * e;
                    const float p0 = fast_exp2(__builtin_fmaf(s_cur[s >> 1][i0], c, -mc));
                    const float p1 = fast_exp2(__builtin_fmaf(s_cur[s >> 1][i0 + 1], c, -mc));
                    psum += p0 + p1;
                    pw[s][e] = pack_bf16(p0, p1);
                }
            l_run += psum;
        }
        __builtin_amdgcn_sched_barrier(0);
        if (late) close_iteration();
        if (wave_active) {
            // Matrix phase: O^T += V^T P^T of this tile, then S^T of the next one into the registers the
            // probabilities have left.
            const uint32_t vb = lds_base(smem + sv_cur * KBYTES + v_lane_off);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 pb = as_bf16x8(pw[s]);
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    bf16x8 a = as_bf16x8(lds_read16(vb, s * PB + db * 512));
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, oacc[db], 0, 0, 0);
                }
            }
            if (ti + 1 < ntiles) qk_tile(st_nxt, s_cur);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (!late) close_iteration();
        tp_k = to_scalar(tp_raw);
        st_cur = st_nxt;
        sv_cur = sv_nxt;
    }

    } else {
    // S^T of 32 keys: the tb-th pair of pages of a K stage
    auto qk_half = [&](int stage, int tb, f32x16& sacc) {
        const uint32_t kb = lds_base(smem + stage * KBYTES + k_lane_off + tb * 2 * PB);
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 a = as_bf16x8(lds_read16(kb, ks * 512));
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sacc, 0, 0, 0);
        }
    };
    f32x16 s_half;
    if (wave_active) qk_half(0, 0, s_half);
    lds_barrier();  // with rings of NS stages the first iteration's loads overwrite K stage 0
    int st_cur = 0;   // ti % NSK
    int sv_cur = 0;   // ti % NSV: V stage of tile ti
#if PPD_PINGPONG
    const bool late = wave >= kWaves / 2;  // waves w and w + 4 share a SIMD
#else
    const bool late = false;
#endif
    TilePages tp_v = tile_pages(NS - 1 < ntiles ? NS - 1 : ntiles - 1);  // pages of the loads the first iteration issues
    TilePages tp_k = tile_pages(NS < ntiles ? NS : ntiles - 1);
    for (int ti = 0; ti < ntiles; ++ti) {
        const int st_nxt = st_cur + 1 == NSK ? 0 : st_cur + 1;           // (ti + 1) % NSK
        const int st_far = ring_add<NSK>(st_cur, NS % NSK);                           // (ti + NS) % NSK
        const int sv_nxt = sv_cur + 1 == NSV ? 0 : sv_cur + 1;           // (ti + 1) % NSV
        const int sv_far = ring_add<NSV>(sv_cur, (NS - 1) % NSV);                       // (ti + NS - 1) % NSV
        const bool full_issue = ti + NS < ntiles;
        if (ti + NS - 1 < ntiles) load_block(tp_v, VRING + sv_far * KBYTES, true);
        if (full_issue) load_block(tp_k, st_far * KBYTES, false);
        tp_v = tp_k;
        const RawPages tp_raw = tile_pages_raw(ti + 1 + NS < ntiles ? ti + 1 + NS : ntiles - 1);
        auto close_iteration = [&]() {
            if (full_issue)  // then the last NS - 2 iterations all issued their full share
                wait_older_loads();
            else
                wait_all_loads();
            if (ti + 1 < ntiles) fix_v_tail(ti + 1, VRING + sv_nxt * KBYTES);
            lds_barrier();
        };
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            u32x4 pw[2];  // the half's probabilities as bf16, B operand of its two 16-key steps of the PV product
            if (wave_active) {
                const int half_base = it.kv_begin + ti * kTileTokens + hb * 32;
                if (half_base + 31 > wmin_limit) {  // causal boundary crosses this half
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int pos = half_base + (i >> 3) * 16 + h * 8 + (i & 7);
                        if (pos > limit) s_half[i] = NEG_INF;
                    }
                }
                float mx = s_half[0];
#pragma unroll
                for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s_half[i]);
                mx = max_halves(mx);
                const float m_new = fmaxf(m_run, mx);
                if (__any((m_new - m_run) * c > kLazyRescale)) {  // -inf -> finite counts; -inf -> -inf does not
                    const float m_use = m_new == NEG_INF ? 0.f : m_new;
                    const float alpha = fast_exp2(m_run * c - m_use * c);  // m_run = -inf gives 0
                    l_run *= alpha;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
                    m_run = m_new;
                }
                const float mc = m_run == NEG_INF ? 0.f : m_run * c;
                float psum = 0.f;
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i0 = s2 * 8 + 2 * e;
                        const float p0 = fast_exp2(__builtin_fmaf(s_half[i0], c, -mc));
                        const float p1 = fast_exp2(__builtin_fmaf(s_half[i0 + 1], c, -mc));
                        psum += p0 + p1;
                        pw[s2][e] = pack_bf16(p0, p1);
                    }
                l_run += psum;
            }
            __builtin_amdgcn_sched_barrier(0);
            if (hb == 1 && late) close_iteration();
            if (wave_active) {
                // O^T += V^T P^T of this half, then S^T of the next half into the registers the probabilities left
                const uint32_t vb = lds_base(smem + sv_cur * KBYTES + v_lane_off + hb * 2 * PB);
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const bf16x8 pb = as_bf16x8(pw[s2]);
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        bf16x8 a = as_bf16x8(lds_read16(vb, s2 * PB + db * 512));
                        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, oacc[db], 0, 0, 0);
                    }
                }
                if (hb == 0)
                    qk_half(st_cur, 1, s_half);
                else if (ti + 1 < ntiles)
                    qk_half(st_nxt, 0, s_half);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (!late) close_iteration();
        tp_k = to_scalar(tp_raw);
        st_cur = st_nxt;
        sv_cur = sv_nxt;
    }

    }
    // epilogue: O^T register i of block db is d = db*32 + (i/4)*8 + h*4 + i%4 of column `col`
    const float l_tot = sum_halves(l_run);
    if (col < ncols) {
        if (it.part_off < 0) {
            const float inv = P.v_scale / l_tot;
            uint16_t* op = P.out + ((int64_t)(it.grow0 + jrow) * P.Hq + head) * HD + h * 4;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    u32x2 w;
                    w[0] = pack_bf16(oacc[db][i4 * 4 + 0] * inv, oacc[db][i4 * 4 + 1] * inv);
                    w[1] = pack_bf16(oacc[db][i4 * 4 + 2] * inv, oacc[db][i4 * 4 + 3] * inv);
                    *reinterpret_cast<u32x2*>(op + db * 32 + i4 * 8) = w;
                }
        } else {
            float* pp = P.partials + it.part_off;
            float* po = pp + (int64_t)col * HD + h * 4;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    f32x4 w = {oacc[db][i4 * 4 + 0], oacc[db][i4 * 4 + 1], oacc[db][i4 * 4 + 2], oacc[db][i4 * 4 + 3]};
                    *reinterpret_cast<f32x4*>(po + db * 32 + i4 * 8) = w;
                }
            if (h == 0) {
                float* ml = pp + (int64_t)ncols * HD + col * 2;
                ml[0] = m_run;
                ml[1] = l_tot;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Narrow tile: rows*G <= 16 query columns (decode: 1 row x G heads).  HBM-bound: each of the NW waves
// streams its own share of the key range straight from the pool into MFMA operand registers
// (v_mfma_f32_16x16x32_bf16 for S^T, v_mfma_f32_16x16x16_bf16 for O^T; one page per step; NK register sets for
// K and NV <= NK for V rotate, so that K of NK - 1 and V of NV - 1 pages per wave are in flight while one page is
// computed), then the waves' (o, m, l) are combined through LDS, CB columns per pass.
// ---------------------------------------------------------------------------------------------------
template <int NW>
struct NarrowCombine {
    static constexpr int CB = NW >= 8 ? kNarrowCols : 8;  // columns per combine pass
    static constexpr size_t bytes(int head_dim) { return (size_t)NW * CB * (head_dim + 2) * sizeof(float); }
};

// SOLO: the calling wave runs the whole tile on its own (NW = 1): no LDS, no barrier, the result is written from the
// accumulator registers; the other waves of the workgroup run other tiles at the same time.
// (bf16 pages; FP8 pages are read by narrow_item_wide.)
template <int HD, int NW, int NK, int NV, bool SOLO = false>
__device__ __forceinline__ void narrow_item(const KParams& P, const ppd_work_item& it, char* smem) {
    static_assert(!SOLO || NW == 1, "a solo tile is one wave");
    constexpr int EB = 2;  // bytes per pool element
    using KVec = u32x4;    // 8 elements
    using VVec = u32x2;    // 4 elements
    constexpr int KS = HD / 32;   // k-steps of S^T
    constexpr int DBN = HD / 16;  // 16-row d blocks of O^T
    constexpr int CB = NarrowCombine<NW>::CB;
    constexpr int WSTRIDE = CB * (HD + 2);  // floats per wave in the combine buffer
    constexpr int NT = NW * 64;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = SOLO ? 0 : __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c16 = lane & 15;
    const int g4 = lane >> 4;
    const int G = P.G;
    const int ncols = it.nrows * G;
    const int colc = c16 < ncols ? c16 : ncols - 1;
    const int jrow = col_row(colc, P.invG);
    const int head = it.kvh * G + (colc - jrow * G);
    const int limit = it.L + it.row0 + jrow;
    const int min_limit = it.L + it.row0;

    bf16x8 qreg[KS];
    {
        const uint16_t* qp = P.q + ((int64_t)(it.grow0 + jrow) * P.Hq + head) * HD + g4 * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 w = *reinterpret_cast<const u32x4*>(qp + ks * 32);
            if (c16 >= ncols) w = u32x4{0, 0, 0, 0};
            qreg[ks] = as_bf16x8(w);
        }
    }

    const int32_t* pt_row = P.page_tables + (int64_t)it.seq * P.max_pages;
    const int last_page = (it.kv_total - 1) >> 4;
    const int nsteps = (it.kv_end - it.kv_begin + kPage - 1) >> 4;  // one page per step
    const int s_lo = wave * nsteps / NW, s_hi = (wave + 1) * nsteps / NW;
    const int wave_first_page = (it.kv_begin >> 4) + s_lo;
    const int64_t head_off = (int64_t)it.kvh * (kPage * HD);
    const int64_t v_off = (int64_t)P.Hkv * (kPage * HD);

    f32x4 oacc[DBN];
#pragma unroll
    for (int db = 0; db < DBN; ++db) oacc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = NEG_INF, l_run = 0.f;
    const float c = P.scale_log2e;

    // lane i of `ids_*` holds the page of logical page (batch*64 + i) of this wave's range.  K loads run NK - 1 steps
    // ahead of the computation and drive the rotation of the id batches; V loads run NV - 1 <= NK - 1 steps ahead
    // and may still be in the batch before (ids_old).
    int ids_old = 0, ids_cur = 0, ids_nxt = 0, k_batch = 0;
    auto load_ids = [&](int batch) { return load_page_id(pt_row, wave_first_page + batch * 64 + lane, last_page); };
    struct KRegs { KVec k[KS]; };   // K operand of the page: 16 tokens x 32 d per k-step
    struct VRegs { VVec v[DBN]; };  // V^T operand: 4 tokens of one d, one per 16-row d block
    KRegs rk[NK];
    VRegs rv[NV];
    const int my_steps = s_hi - s_lo;
    const uint32_t k_lane_bytes = (uint32_t)(g4 * 128 + c16 * 8) * EB;                          // + ks * 512 elements
    const uint32_t v_lane_bytes = (uint32_t)(((g4 >> 1) * HD + c16) * 8 + (g4 & 1) * 4) * EB;  // + db * 128 elements
    // K and V are read once: non-temporal loads (no reuse to keep in the caches) stream ~12 % faster than plain
    // ones on this pattern.  Address = wave-uniform base of the (page, head) block + one 32-bit byte offset per lane.
    auto issue_k = [&](int k, KRegs& r) {  // k = step index relative to s_lo
        if ((k & 63) == 0 && k > 0) {
            ids_old = ids_cur;
            ids_cur = ids_nxt;
            k_batch = k >> 6;
            if (k + 64 < my_steps) ids_nxt = load_ids(k_batch + 1);
        }
        const int64_t pa = checked_page(P, __builtin_amdgcn_readlane(ids_cur, k & 63));
        const char* kb = reinterpret_cast<const char*>(P.pool) + (pa * P.page_stride + head_off) * EB;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            r.k[ks] = __builtin_nontemporal_load(reinterpret_cast<const KVec*>(kb + k_lane_bytes + ks * (512 * EB)));
    };
    auto issue_v = [&](int k, VRegs& r) {
        const int ids = (k >> 6) == k_batch ? ids_cur : ids_old;
        const int64_t pa = checked_page(P, __builtin_amdgcn_readlane(ids, k & 63));
        const char* vb = reinterpret_cast<const char*>(P.pool) + (pa * P.page_stride + head_off + v_off) * EB;
#pragma unroll
        for (int db = 0; db < DBN; ++db)
            r.v[db] = __builtin_nontemporal_load(reinterpret_cast<const VVec*>(vb + v_lane_bytes + db * (128 * EB)));
    };
    auto compute_step = [&](int k, KRegs& rs, VRegs& rw) {
        f32x4 sa = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(rs.k[ks]), qreg[ks], sa, 0, 0, 0);
        // sa[i]: token 4*g4 + i of the page
        const int t0 = it.kv_begin + (s_lo + k) * kPage;
        const bool masked = t0 + kPage - 1 > min_limit || t0 + kPage > it.kv_end;
        if (masked) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int pa = t0 + 4 * g4 + i;
                if (pa > limit || pa >= it.kv_end) sa[i] = NEG_INF;
            }
            if (t0 + kPage > it.kv_total) {  // rows of the last page that were never written
#pragma unroll
                for (int db = 0; db < DBN; ++db) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int pos = t0 + 4 * g4 + e;
                        if (pos >= it.kv_total) rw.v[db][e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
                    }
                }
            }
        }
        float mx = fmaxf(fmaxf(sa[0], sa[1]), fmaxf(sa[2], sa[3]));
        mx = fmaxf(mx, xor_shuffle(mx, 16));
        mx = max_halves(mx);
        const float m_new = fmaxf(m_run, mx);
        if (__any((m_new - m_run) * c > kLazyRescale)) {
            const float m_use = m_new == NEG_INF ? 0.f : m_new;
            const float alpha = fast_exp2(m_run * c - m_use * c);
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < DBN; ++db) oacc[db] *= alpha;
            m_run = m_new;
        }
        const float mc = m_run == NEG_INF ? 0.f : m_run * c;
        float p[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] = fast_exp2(__builtin_fmaf(sa[i], c, -mc));
        l_run += (p[0] + p[1]) + (p[2] + p[3]);
        const u32x2 pw = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3])};
        const s16x4 pb4 = __builtin_bit_cast(s16x4, pw);
#pragma unroll
        for (int db = 0; db < DBN; ++db)
            oacc[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, rw.v[db]), pb4, oacc[db], 0, 0, 0);
    };

    // K of NK - 1 pages and V of NV - 1 pages (4 KiB each at D = 128) are in flight per wave while one page is being
    // computed; the register sets rotate (period = NK * NV steps, unrolled).  The loads sit under conditions, so at
    // the points where paths meet the compiler's waits on the memory counter assume the path with the fewest loads
    // issued and mostly drain what was just issued.  That costs nothing here: a loop without any conditional load
    // (waits of 36..47 outstanding loads in its steady state) was built and measured the same -- a compute unit
    // pulls at most ~58 GB/s from HBM however much it keeps in flight (a load-only kernel with 4 KiB or 28 KiB in
    // flight per wave, 8 or 16 waves: 54..60 GB/s per unit), and eight waves with one page each are already there.
    if (my_steps > 0) {
        ids_cur = load_ids(0);
        if (my_steps > 64) ids_nxt = load_ids(1);
#pragma unroll
        for (int j = 0; j < NK - 1; ++j)
            if (j < my_steps) issue_k(j, rk[j]);
#pragma unroll
        for (int j = 0; j < NV - 1; ++j)
            if (j < my_steps) issue_v(j, rv[j]);
    }
    constexpr int PERIOD = NK == NV ? NK : NK * NV;
    for (int k = 0; k < my_steps; k += PERIOD) {
#pragma unroll
        for (int j = 0; j < PERIOD; ++j) {
            if (k + j < my_steps) {
                if (k + j + NK - 1 < my_steps) issue_k(k + j + NK - 1, rk[(j + NK - 1) % NK]);
                if (k + j + NV - 1 < my_steps) issue_v(k + j + NV - 1, rv[(j + NV - 1) % NV]);
                compute_step(k + j, rk[j % NK], rv[j % NV]);
            }
        }
    }
    l_run += xor_shuffle(l_run, 16);
    l_run = sum_halves(l_run);

    if constexpr (SOLO) {
        // O^T register i of block db is d = db*16 + 4*g4 + i of column c16; m and l are the column's in every lane
        if (c16 < ncols) {
            if (it.part_off < 0) {
                const float inv = P.v_scale / l_run;
                uint16_t* op = P.out + ((int64_t)(it.grow0 + jrow) * P.Hq + head) * HD + 4 * g4;
#pragma unroll
                for (int db = 0; db < DBN; ++db) {
                    u32x2 w;
                    w[0] = pack_bf16(oacc[db][0] * inv, oacc[db][1] * inv);
                    w[1] = pack_bf16(oacc[db][2] * inv, oacc[db][3] * inv);
                    *reinterpret_cast<u32x2*>(op + db * 16) = w;
                }
            } else {
                float* pp = P.partials + it.part_off;
#pragma unroll
                for (int db = 0; db < DBN; ++db)
                    *reinterpret_cast<f32x4*>(pp + (int64_t)c16 * HD + db * 16 + 4 * g4) = oacc[db];
                if (g4 == 0) {
                    pp[(int64_t)ncols * HD + c16 * 2] = m_run;
                    pp[(int64_t)ncols * HD + c16 * 2 + 1] = l_run;
                }
            }
        }
        return;
    }
    // combine the waves, CB columns per pass: O^T register i of block db is d = db*16 + 4*g4 + i of column c16
    float* wbuf = reinterpret_cast<float*>(smem) + wave * WSTRIDE;
    const float* all = reinterpret_cast<const float*>(smem);
    for (int c0 = 0; c0 < ncols; c0 += CB) {
        if (c0 > 0) __syncthreads();  // the previous pass has been read
        if (c16 >= c0 && c16 < c0 + CB) {
#pragma unroll
            for (int db = 0; db < DBN; ++db)
                *reinterpret_cast<f32x4*>(wbuf + (c16 - c0) * HD + db * 16 + 4 * g4) = oacc[db];
            if (g4 == 0) {
                wbuf[CB * HD + (c16 - c0) * 2] = m_run;
                wbuf[CB * HD + (c16 - c0) * 2 + 1] = l_run;
            }
        }
        __syncthreads();
        const int nc = ncols - c0 < CB ? ncols - c0 : CB;
        for (int idx = tid; idx < nc * HD; idx += NT) {
            const int cl = idx / HD, d = idx % HD;
            const int col = c0 + cl;
            float mw[NW], mm = NEG_INF;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                mw[w] = all[w * WSTRIDE + CB * HD + cl * 2];
                mm = fmaxf(mm, mw[w]);
            }
            float o = 0.f, l = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float f = mw[w] == NEG_INF ? 0.f : fast_exp2((mw[w] - mm) * c);
                o += f * all[w * WSTRIDE + cl * HD + d];
                l += f * all[w * WSTRIDE + CB * HD + cl * 2 + 1];
            }
            if (it.part_off < 0) {
                const int crow = col_row(col, P.invG);
                const int64_t orow = (int64_t)(it.grow0 + crow) * P.Hq + it.kvh * G + (col - crow * G);
                const float val = (o / l) * P.v_scale;
                const float other = __shfl_xor(val, 1, 64);  // d and d^1 sit in neighbouring lanes
                if ((d & 1) == 0) *reinterpret_cast<uint32_t*>(P.out + orow * HD + d) = pack_bf16(val, other);
            } else {
                float* pp = P.partials + it.part_off;
                pp[(int64_t)col * HD + d] = o;
                if (d == 0) {
                    pp[(int64_t)ncols * HD + col * 2] = mm;
                    pp[(int64_t)ncols * HD + col * 2 + 1] = l;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Narrow tile on the operand shapes of the row-block tile: v_mfma_f32_32x32x16_bf16 for both products, two pages (32
// keys) per step, operands loaded from the pool straight into registers.  A lane then loads whole granules -- 8 d of one
// key for K, 8 tokens of one d for V -- in runs of 256 and 512 contiguous bytes per half-wave, where the 16x16 shapes of
// narrow_item make a lane own 4 tokens of a d (half a granule).  For FP8 pages that is 8 bytes per lane instead of 4 in
// V, and a compute unit streams a third more (measured with loads alone: 45 against 33 GB/s; bf16 pages 53 against 48).
// Half of the 32 columns of every product are unused (a narrow tile has at most 16), which costs matrix time the
// memory-bound tile has to spare.  Used for FP8 pages.
//   S^T rows: MFMA row r is key (page r >> 4 of the pair, token 8*bit2(r) + 4*bit3(r) + (r & 3)), so that accumulator
//   registers 0..7 of a lane are tokens 8h..8h+7 of the first page and 8..15 those of the second (h = lane / 32):
//   the octet the lane's V granules hold.
// NS register sets of one page pair each rotate: NS - 1 pairs are in flight per wave.
// ---------------------------------------------------------------------------------------------------
template <int HD, int NW, int NS, bool SOLO, bool FP8>
__device__ __forceinline__ void narrow_item_wide(const KParams& P, const ppd_work_item& it, char* smem) {
    static_assert(!SOLO || NW == 1, "a solo tile is one wave");
    constexpr int EB = FP8 ? 1 : 2;                       // bytes per pool element
    using Vec = std::conditional_t<FP8, u32x2, u32x4>;    // a granule: 8 elements
    constexpr int KS = HD / 16;   // k-steps of S^T
    constexpr int DB = HD / 32;   // 32-row d blocks of O^T
    constexpr int CB = NarrowCombine<NW>::CB;
    constexpr int WSTRIDE = CB * (HD + 2);
    constexpr int NT = NW * 64;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = SOLO ? 0 : __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31;   // column of the products' B operands and results; key row / d row of the A operands
    const int h = lane >> 5;
    const int G = P.G;
    const int ncols = it.nrows * G;
    const int colc = r < ncols ? r : ncols - 1;
    const int jrow = col_row(colc, P.invG);
    const int head = it.kvh * G + (colc - jrow * G);
    const int limit = it.L + it.row0 + jrow;
    const int min_limit = it.L + it.row0;

    bf16x8 qreg[KS];  // Q^T operand: column r, d = ks*16 + h*8 .. +8; zero for the unused columns
    {
        const uint16_t* qp = P.q + ((int64_t)(it.grow0 + jrow) * P.Hq + head) * HD + h * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 w = *reinterpret_cast<const u32x4*>(qp + ks * 16);
            if (r >= ncols) w = u32x4{0, 0, 0, 0};
            qreg[ks] = as_bf16x8(w);
        }
    }

    const int32_t* pt_row = P.page_tables + (int64_t)it.seq * P.max_pages;
    const int last_page = (it.kv_total - 1) >> 4;
    const int npages = (it.kv_end - it.kv_begin + kPage - 1) >> 4;
    const int s_lo = wave * npages / NW, s_hi = (wave + 1) * npages / NW;
    const int my_pages = s_hi - s_lo;
    const int my_steps = (my_pages + 1) >> 1;  // page pairs; the last may lack its second page
    const int wave_first_page = (it.kv_begin >> 4) + s_lo;
    const int64_t head_off = (int64_t)it.kvh * (kPage * HD);
    const int64_t v_off = (int64_t)P.Hkv * (kPage * HD);

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m_run = NEG_INF, l_run = 0.f;
    const float c = P.scale_log2e;

    // lane i of ids_cur holds the page of logical page (batch*64 + i) of this wave's range; a pair never straddles batches
    int ids_cur = 0, ids_nxt = 0;
    auto load_ids = [&](int batch) { return load_page_id(pt_row, wave_first_page + batch * 64 + lane, last_page); };
    struct Set {
        Vec k[KS];      // K operand of the pair: 32 keys x 16 d per k-step
        Vec v[2][DB];   // V^T operand of each page: 32 d x 8 tokens (the lane's octet) per d block
    };
    Set rs[NS];
    const int k_tok = ((r >> 2) & 1) * 8 + ((r >> 3) & 1) * 4 + (r & 3);
    const uint32_t k_lane_bytes = (uint32_t)(h * 128 + k_tok * 8) * EB;   // + ks * 256 elements
    const uint32_t v_lane_bytes = (uint32_t)((h * HD + r) * 8) * EB;      // + db * 256 elements
    auto issue = [&](int j, Set& s) {  // j = pair index relative to s_lo
        const int pg0 = 2 * j;
        if ((pg0 & 63) == 0 && pg0 > 0) {
            ids_cur = ids_nxt;
            if (pg0 + 64 < my_pages) ids_nxt = load_ids((pg0 >> 6) + 1);
        }
        const int id_a = __builtin_amdgcn_readlane(ids_cur, pg0 & 63);
        const int id_b = pg0 + 1 < my_pages ? __builtin_amdgcn_readlane(ids_cur, (pg0 + 1) & 63) : id_a;  // absent: re-read the first
        const char* base_a = reinterpret_cast<const char*>(P.pool) + (checked_page(P, id_a) * P.page_stride + head_off) * EB;
        const char* base_b = reinterpret_cast<const char*>(P.pool) + (checked_page(P, id_b) * P.page_stride + head_off) * EB;
        const char* kb = ((r & 16) ? base_b : base_a) + k_lane_bytes;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s.k[ks] = __builtin_nontemporal_load(reinterpret_cast<const Vec*>(kb + ks * (256 * EB)));
        const char* va = base_a + v_off * EB + v_lane_bytes;
        const char* vb = base_b + v_off * EB + v_lane_bytes;
#pragma unroll
        for (int db = 0; db < DB; ++db) s.v[0][db] = __builtin_nontemporal_load(reinterpret_cast<const Vec*>(va + db * (256 * EB)));
#pragma unroll
        for (int db = 0; db < DB; ++db) s.v[1][db] = __builtin_nontemporal_load(reinterpret_cast<const Vec*>(vb + db * (256 * EB)));
    };
    auto operand = [&](Vec v) {
        if constexpr (FP8) return as_bf16x8(fp8x8_to_bf16x8(v)); else return as_bf16x8(v);
    };
    auto compute_step = [&](int j, Set& s) {
        f32x16 sa;
#pragma unroll
        for (int i = 0; i < 16; ++i) sa[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(operand(s.k[ks]), qreg[ks], sa, 0, 0, 0);
        // sa[i]: token 8*h + (i & 7) of page i >> 3 of the pair
        const int t0 = it.kv_begin + (s_lo + 2 * j) * kPage;
        const bool has_b = 2 * j + 1 < my_pages;
        if (t0 + 2 * kPage - 1 > min_limit || t0 + 2 * kPage > it.kv_end || !has_b) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int pos = t0 + (i >> 3) * kPage + h * 8 + (i & 7);
                if (pos > limit || pos >= it.kv_end || ((i >> 3) && !has_b)) sa[i] = NEG_INF;
            }
            if (t0 + 2 * kPage > it.kv_total || !has_b) {  // rows never written, or the page that is not there
#pragma unroll
                for (int pg = 0; pg < 2; ++pg)
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int pos = t0 + pg * kPage + h * 8 + e;
                            if (pos >= it.kv_total || (pg && !has_b)) {
                                if constexpr (FP8) s.v[pg][db][e >> 2] &= ~(0xFFu << (8 * (e & 3)));  // code 0 is 0.0
                                else s.v[pg][db][e >> 1] &= (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
                            }
                        }
            }
        }
        float mx = sa[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sa[i]);
        mx = max_halves(mx);
        const float m_new = fmaxf(m_run, mx);
        if (__any((m_new - m_run) * c > kLazyRescale)) {
            const float m_use = m_new == NEG_INF ? 0.f : m_new;
            const float alpha = fast_exp2(m_run * c - m_use * c);
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
            m_run = m_new;
        }
        const float mc = m_run == NEG_INF ? 0.f : m_run * c;
        u32x4 pw[2];
        float psum = 0.f;
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float p0 = fast_exp2(__builtin_fmaf(sa[pg * 8 + 2 * e], c, -mc));
                const float p1 = fast_exp2(__builtin_fmaf(sa[pg * 8 + 2 * e + 1], c, -mc));
                psum += p0 + p1;
                pw[pg][e] = pack_bf16(p0, p1);
            }
        l_run += psum;
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int db = 0; db < DB; ++db)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(operand(s.v[pg][db]), as_bf16x8(pw[pg]), oacc[db], 0, 0, 0);
    };

    if (my_steps > 0) {
        ids_cur = load_ids(0);
        if (my_pages > 64) ids_nxt = load_ids(1);
#pragma unroll
        for (int j = 0; j < NS - 1; ++j)
            if (j < my_steps) issue(j, rs[j]);
    }
    for (int k = 0; k < my_steps; k += NS) {
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            if (k + j < my_steps) {
                if (k + j + NS - 1 < my_steps) issue(k + j + NS - 1, rs[(j + NS - 1) % NS]);
                compute_step(k + j, rs[j]);
            }
        }
    }
    const float l_tot = sum_halves(l_run);

    // O^T register i of block db is d = db*32 + (i/4)*8 + h*4 + i%4 of column r; m and l_tot are the column's in both halves
    if constexpr (SOLO) {
        if (r < ncols) {
            if (it.part_off < 0) {
                const float inv = P.v_scale / l_tot;
                uint16_t* op = P.out + ((int64_t)(it.grow0 + jrow) * P.Hq + head) * HD + h * 4;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        u32x2 w;
                        w[0] = pack_bf16(oacc[db][i4 * 4 + 0] * inv, oacc[db][i4 * 4 + 1] * inv);
                        w[1] = pack_bf16(oacc[db][i4 * 4 + 2] * inv, oacc[db][i4 * 4 + 3] * inv);
                        *reinterpret_cast<u32x2*>(op + db * 32 + i4 * 8) = w;
                    }
            } else {
                float* pp = P.partials + it.part_off;
                float* po = pp + (int64_t)r * HD + h * 4;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const f32x4 w = {oacc[db][i4 * 4 + 0], oacc[db][i4 * 4 + 1], oacc[db][i4 * 4 + 2], oacc[db][i4 * 4 + 3]};
                        *reinterpret_cast<f32x4*>(po + db * 32 + i4 * 8) = w;
                    }
                if (h == 0) {
                    pp[(int64_t)ncols * HD + r * 2] = m_run;
                    pp[(int64_t)ncols * HD + r * 2 + 1] = l_tot;
                }
            }
        }
        return;
    }
    // combine the waves through LDS, CB columns per pass (the buffer and the second half are those of narrow_item)
    float* wbuf = reinterpret_cast<float*>(smem) + wave * WSTRIDE;
    const float* all = reinterpret_cast<const float*>(smem);
    for (int c0 = 0; c0 < ncols; c0 += CB) {
        if (c0 > 0) __syncthreads();  // the previous pass has been read
        if (r >= c0 && r < c0 + CB && r < ncols) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x4 w = {oacc[db][i4 * 4 + 0], oacc[db][i4 * 4 + 1], oacc[db][i4 * 4 + 2], oacc[db][i4 * 4 + 3]};
                    *reinterpret_cast<f32x4*>(wbuf + (r - c0) * HD + db * 32 + i4 * 8 + h * 4) = w;
                }
            if (h == 0) {
                wbuf[CB * HD + (r - c0) * 2] = m_run;
                wbuf[CB * HD + (r - c0) * 2 + 1] = l_tot;
            }
        }
        __syncthreads();
        const int nc = ncols - c0 < CB ? ncols - c0 : CB;
        for (int idx = tid; idx < nc * HD; idx += NT) {
            const int cl = idx / HD, d = idx % HD;
            const int col = c0 + cl;
            float mw[NW], mm = NEG_INF;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                mw[w] = all[w * WSTRIDE + CB * HD + cl * 2];
                mm = fmaxf(mm, mw[w]);
            }
            float o = 0.f, l = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float f = mw[w] == NEG_INF ? 0.f : fast_exp2((mw[w] - mm) * c);
                o += f * all[w * WSTRIDE + cl * HD + d];
                l += f * all[w * WSTRIDE + CB * HD + cl * 2 + 1];
            }
            if (it.part_off < 0) {
                const int crow = col_row(col, P.invG);
                const int64_t orow = (int64_t)(it.grow0 + crow) * P.Hq + it.kvh * G + (col - crow * G);
                const float val = (o / l) * P.v_scale;
                const float other = __shfl_xor(val, 1, 64);  // d and d^1 sit in neighbouring lanes
                if ((d & 1) == 0) *reinterpret_cast<uint32_t*>(P.out + orow * HD + d) = pack_bf16(val, other);
            } else {
                float* pp = P.partials + it.part_off;
                pp[(int64_t)col * HD + d] = o;
                if (d == 0) {
                    pp[(int64_t)ncols * HD + col * 2] = mm;
                    pp[(int64_t)ncols * HD + col * 2 + 1] = l;
                }
            }
        }
    }
}

// Claims the next tile of queue q: its index in the work list, or -1 when the queue is exhausted.  A claim on the
// wave-tile queue covers kWaves consecutive tiles and returns the index of the first.
__device__ __forceinline__ int claim_from(const KParams& P, int q) {
    const int got = (int)atomicAdd(&P.counters[kCursorBase + q * kCursorStride], 1u) * (q == kWaveQueue ? kWaves : 1);
    return got < P.queue_begin[q + 1] - P.queue_begin[q] ? P.queue_begin[q] + got : -1;
}

// The last workgroup of a kernel to run out of work re-arms the cursors of queues [q0, q1) and the kernel's own
// count of finished workgroups (word `done_word`) for the next launch.
__device__ __forceinline__ void rearm_cursors(const KParams& P, int q0, int q1, int done_word) {
    const unsigned done = atomicAdd(&P.counters[done_word], 1u);
    if (done == gridDim.x - 1) {
        for (int q = q0; q < q1; ++q)
            __hip_atomic_store(&P.counters[kCursorBase + q * kCursorStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&P.counters[done_word], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int HD, bool FP8>
__global__ __launch_bounds__(kThreads, 2) void ppd_mixed_kernel(const KParams P) {
    constexpr int NSETS = 4;  // rotating register sets (one page each) of a streaming wave on bf16 pages
    // Dynamic LDS: rings of kStages + 1 stages of 4 pages of K and as many of V, then the page ids of a tile's key
    // range, for the MFMA path (136 KiB at HD = 128); the narrow path's combine buffer (kWaves * 16 * (HD+2)
    // floats) uses the front of it.
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ int s_next_slot;
    volatile int* s_next = &s_next_slot;
    const int tid = threadIdx.x;
    // Ten queues in one list: MFMA row-block tiles in eight queues, one per XCD (tiles that read the same K/V
    // sit in the same queue, next to each other, so the workgroups of one XCD find them in their L2), and one
    // queue of narrow tiles run by the whole workgroup and one of short narrow tiles run one per wave; each longest tile
    // first.  A workgroup prefers one kind, chosen by the compute
    // unit it runs on (narrow_cus of the 32 units of every XCD take narrow tiles, spread evenly over the shader
    // engines; the planner sizes the split so that both kinds finish together): workgroups that share a unit
    // then run the same kind, and HBM-bound and MFMA-bound tiles run side by side on different units.
    // It takes MFMA tiles from its own XCD's queue first, and steals from the other queues when its own run dry.
    int pref;
    switch (P.pref_mode) {
        case 1: pref = (blockIdx.x >> 3) & 1; break;
        case 2: {
            // HW_REG_HW_ID: cu_id in bits 11:8, se_id in bits 15:13 (eight active units per shader engine, ids
            // 0..8 with one gap, so the low three bits tell them apart)
            const unsigned hw = __builtin_amdgcn_s_getreg((15 << 11) | (0 << 6) | 4);
            const int unit = (int)(((hw >> 8) & 7) << 2 | ((hw >> 13) & 3));
            pref = unit < P.narrow_cus ? 1 : 0;
            break;
        }
        case 3: pref = 1; break;
        default: pref = 0; break;
    }
    const int xcd = (int)(__builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20) & (kXcds - 1));  // HW_REG_XCC_ID
    // bit q: queue q is exhausted (only thread 0 uses it).  Queues that are empty by construction never cost an
    // atomic; when a claim finds a queue exhausted, one batch of plain loads of all nine cursors tells which
    // others are, instead of one failing atomic (a round trip to the L2 each, one after the other) per queue --
    // that chain used to be the last ~10 us of every workgroup, and so of every launch.
    unsigned dry = 0;
#pragma unroll
    for (int q = 0; q < kQueues; ++q)
        if (P.queue_begin[q + 1] == P.queue_begin[q]) dry |= 1u << q;
    constexpr unsigned kAllDry = (1u << kQueues) - 1;
    auto look_at_cursors = [&]() {
        unsigned cur[kQueues];
#pragma unroll
        for (int q = 0; q < kQueues; ++q)
            cur[q] = __hip_atomic_load(&P.counters[kCursorBase + q * kCursorStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int q = 0; q < kQueues; ++q)
            if ((int)(cur[q] * (q == kWaveQueue ? kWaves : 1)) >= P.queue_begin[q + 1] - P.queue_begin[q]) dry |= 1u << q;
    };
    for (;;) {
        if (tid == 0) {
            int idx = -1;
#pragma unroll
            for (int attempt = 0; attempt < 2 && idx < 0; ++attempt) {
                const bool want_narrow = (attempt == 0) == (pref == 1);
                if (want_narrow) {
                    // whole-workgroup tiles first (the long ones), then the very short ones, eight to a claim
                    for (int q = kNarrowQueue; q <= kWaveQueue && idx < 0; ++q) {
                        if (dry & (1u << q)) continue;
                        idx = claim_from(P, q);
                        if (idx < 0) {
                            dry |= 1u << q;
                            if (dry != kAllDry) look_at_cursors();
                        }
                    }
                } else {
                    for (int a = 0; a < kXcds && idx < 0; ++a) {
                        const int q = (xcd + a) & (kXcds - 1);
                        if (dry & (1u << q)) continue;
                        idx = claim_from(P, q);
                        if (idx < 0) {
                            dry |= 1u << q;
                            if (dry != kAllDry) look_at_cursors();
                        }
                    }
                }
            }
            *s_next = idx;
        }
        __syncthreads();
        const int idx = __builtin_amdgcn_readfirstlane(*s_next);
        __syncthreads();  // everyone has read s_next, and the previous tile's LDS use is over
        if (idx < 0) break;
        if (idx >= P.queue_begin[kWaveQueue]) {
            // a claim on the wave-tile queue: wave w runs tile idx + w on its own
            const int mine = idx + __builtin_amdgcn_readfirstlane(tid >> 6);
            if (mine < P.queue_begin[kQueues]) {
                const ppd_work_item it = P.items[mine];
                if constexpr (FP8) narrow_item_wide<HD, 1, kFp8StreamSets, true, true>(P, it, smem);
                else narrow_item<HD, 1, NSETS, NSETS, true>(P, it, smem);
            }
            continue;
        }
        const ppd_work_item it = P.items[idx];
        if (it.kind == 0) {
            if constexpr (FP8) narrow_item_wide<HD, kWaves, kFp8StreamSets, false, true>(P, it, smem);
            else narrow_item<HD, kWaves, NSETS, NSETS, false>(P, it, smem);
        } else {
            mfma_item<HD, false, FP8>(P, it, smem);
        }
    }
    if (tid == 0) rearm_cursors(P, 0, kCursors, 10);
}

// ---------------------------------------------------------------------------------------------------
// A launch that holds narrow tiles only (a decode-only step).  Same tile code as in ppd_mixed_kernel, handed out
// differently: a small launch of the mixed kernel spends 1.7 us on its first claim and ~5 us finding out, claim by
// failing claim, that nothing is left, which is a quarter of a 25 us decode step.  Here the whole-workgroup tiles
// (longest first) and then the one-wave tiles, NW to a slot, form one row of slots; workgroup b takes slot b
// without asking, and only a launch with more slots than workgroups claims further ones (from gridDim.x on) with the
// cursor of the narrow queue, which the last workgroup to finish re-arms.  The host launches no more workgroups than
// there are slots.  Measured and not kept: claiming the next slot before running the current one (hides the round
// trip but holds a slot that an idle workgroup could have run: cfg2 186 -> 206 us), and handing out all slots by
// index, rounds running alternately up and down the workgroups (no atomics at all: same step time on short tiles,
// +3 % on long ones).
// ---------------------------------------------------------------------------------------------------
template <int HD, bool FP8, int NW>
__global__ __launch_bounds__(64 * NW, 2) void ppd_narrow_kernel(const KParams P) {
    constexpr int NSETS = 4;  // rotating register sets (one page each) of a streaming wave on bf16 pages
    extern __shared__ __attribute__((aligned(16))) char smem[];  // the combine buffer
    __shared__ int s_next_slot;
    volatile int* s_next = &s_next_slot;
    const int tid = threadIdx.x;
    const int wg_begin = P.queue_begin[kNarrowQueue], wave_begin = P.queue_begin[kWaveQueue], end = P.queue_begin[kQueues];
    const int n_wg = wave_begin - wg_begin;
    const int slots = n_wg + (end - wave_begin + NW - 1) / NW;
    const bool claims = slots > (int)gridDim.x;  // the same for every workgroup of the launch
    int slot = blockIdx.x;
    while (slot < slots) {
        if (slot < n_wg) {
            const ppd_work_item it = P.items[wg_begin + slot];
            if constexpr (FP8) narrow_item_wide<HD, NW, kFp8StreamSets, false, true>(P, it, smem);
            else narrow_item<HD, NW, NSETS, NSETS, false>(P, it, smem);
        } else {
            const int mine = wave_begin + (slot - n_wg) * NW + __builtin_amdgcn_readfirstlane(tid >> 6);
            if (mine < end) {
                const ppd_work_item it = P.items[mine];
                if constexpr (FP8) narrow_item_wide<HD, 1, kFp8StreamSets, true, true>(P, it, smem);
                else narrow_item<HD, 1, NSETS, NSETS, true>(P, it, smem);
            }
        }
        if (!claims) break;
        if (tid == 0) *s_next = (int)gridDim.x + (int)atomicAdd(&P.counters[kCursorBase + kNarrowQueue * kCursorStride], 1u);
        __syncthreads();
        slot = __builtin_amdgcn_readfirstlane(*s_next);
        __syncthreads();  // everyone has read s_next, and the previous tile's combine is over
    }
    if (claims && tid == 0) rearm_cursors(P, kNarrowQueue, kNarrowQueue + 1, 10);
}

// ---------------------------------------------------------------------------------------------------
// The co-resident pair.  A step that holds both kinds of tiles is launched as two kernels on two streams, sized so
// that one workgroup of each fits on every compute unit at the same time: the row-block kernel (8 waves, two per
// SIMD, 168 registers each, the K/V rings in LDS) keeps the matrix cores busy while the stream kernel (4 waves, one
// per SIMD, 168 registers, a small combine buffer) keeps HBM busy from the same unit -- a compute unit streams
// about 50 GB/s at most, whatever is in flight, so memory-bound tiles need most of the chip's units and so do the
// matrix-bound ones.  Each kernel has its own queues, cursors and count of finished workgroups.
// ---------------------------------------------------------------------------------------------------
template <int HD>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void ppd_mfma_kernel(const KParams P) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ int s_next_slot;
    volatile int* s_next = &s_next_slot;
    const int tid = threadIdx.x;
    const int xcd = (int)(__builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20) & (kXcds - 1));  // HW_REG_XCC_ID
    unsigned dry = 0;  // bit q: queue q is exhausted (only thread 0 uses it)
#pragma unroll
    for (int q = 0; q < kXcds; ++q)
        if (P.queue_begin[q + 1] == P.queue_begin[q]) dry |= 1u << q;
    for (;;) {
        if (tid == 0) {
            int idx = -1;
            for (int a = 0; a < kXcds && idx < 0; ++a) {
                const int q = (xcd + a) & (kXcds - 1);
                if (dry & (1u << q)) continue;
                idx = claim_from(P, q);
                if (idx < 0) {
                    dry |= 1u << q;
                    if (dry != (1u << kXcds) - 1) {  // one batch of plain loads tells which other queues are exhausted
                        unsigned cur[kXcds];
#pragma unroll
                        for (int j = 0; j < kXcds; ++j)
                            cur[j] = __hip_atomic_load(&P.counters[kCursorBase + j * kCursorStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                        for (int j = 0; j < kXcds; ++j)
                            if ((int)cur[j] >= P.queue_begin[j + 1] - P.queue_begin[j]) dry |= 1u << j;
                    }
                }
            }
            *s_next = idx;
        }
        __syncthreads();
        const int idx = __builtin_amdgcn_readfirstlane(*s_next);
        __syncthreads();
        if (idx < 0) break;
        const ppd_work_item it = P.items[idx];
        mfma_item<HD, true>(P, it, smem);
    }
    if (tid == 0) rearm_cursors(P, 0, kXcds, 10);
}

template <int HD>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void ppd_stream_kernel(const KParams P) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ int s_next_slot;
    volatile int* s_next = &s_next_slot;
    const int tid = threadIdx.x;
    for (;;) {
        if (tid == 0) *s_next = claim_from(P, kNarrowQueue);
        __syncthreads();
        const int idx = __builtin_amdgcn_readfirstlane(*s_next);
        __syncthreads();  // everyone has read s_next, and the previous tile's combine is over
        if (idx < 0) break;
        const ppd_work_item it = P.items[idx];
        narrow_item<HD, kStreamWaves, kStreamKSets, kStreamVSets>(P, it, smem);
    }
    if (tid == 0) rearm_cursors(P, kNarrowQueue, kNarrowQueue + 1, 11);
}

// ---------------------------------------------------------------------------------------------------
// Log-sum-exp merge of split partials: out = sum_j o_j 2^{(m_j - m*) c} / sum_j l_j 2^{(m_j - m*) c},
// splits taken in index order (deterministic).  Block b takes the kMergeCols columns starting at units[b].col0 of
// group units[b].group, each wave kMergeCols / 4 of them.  A wave moves little data, so its time is its chain of
// dependent loads: the loads of all its columns (four splits at a time) are issued before the first use.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSmallThreads) void ppd_merge_kernel(const MergeParams M) {
    constexpr int CPW = kMergeCols / (kSmallThreads / 64);  // columns per wave
    const MergeUnit u = M.units[blockIdx.x];
    const MergeGroup g = M.groups[u.group];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ncols = g.nrows * M.G;
    const int D = M.D;
    const int d = lane * 2;
    const bool live = d < D;
    const float* base = M.partials + g.part_off;
    float o0[CPW], o1[CPW], l[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int colr = u.col0 + wave * CPW + c;
        const int col = colr < ncols ? colr : ncols - 1;  // columns past the end redo the last one and store nothing
        const int64_t ml_off = (int64_t)ncols * D + col * 2;
        const int64_t v_off = (int64_t)col * D + (live ? d : 0);
        float mm = NEG_INF;
        o0[c] = o1[c] = l[c] = 0.f;
        if (g.nsplit <= 4) {
            float m4[4], l4[4];
            f32x2 v4[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float* pp = base + g.part_stride * (t < g.nsplit ? t : 0);
                m4[t] = pp[ml_off];
                l4[t] = pp[ml_off + 1];
                v4[t] = *reinterpret_cast<const f32x2*>(pp + v_off);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (t < g.nsplit) mm = fmaxf(mm, m4[t]);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (t < g.nsplit) {
                    const float f = m4[t] == NEG_INF ? 0.f : fast_exp2((m4[t] - mm) * M.scale_log2e);
                    l[c] += f * l4[t];
                    o0[c] += f * v4[t][0];
                    o1[c] += f * v4[t][1];
                }
            }
        } else {
            for (int j0 = 0; j0 < g.nsplit; j0 += 4) {
                float m4[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) m4[t] = base[g.part_stride * (j0 + t < g.nsplit ? j0 + t : j0) + ml_off];
#pragma unroll
                for (int t = 0; t < 4; ++t) mm = fmaxf(mm, m4[t]);
            }
            for (int j0 = 0; j0 < g.nsplit; j0 += 4) {
                float m4[4], l4[4];
                f32x2 v4[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float* pp = base + g.part_stride * (j0 + t < g.nsplit ? j0 + t : j0);
                    m4[t] = pp[ml_off];
                    l4[t] = pp[ml_off + 1];
                    v4[t] = *reinterpret_cast<const f32x2*>(pp + v_off);
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (j0 + t < g.nsplit) {
                        const float f = m4[t] == NEG_INF ? 0.f : fast_exp2((m4[t] - mm) * M.scale_log2e);
                        l[c] += f * l4[t];
                        o0[c] += f * v4[t][0];
                        o1[c] += f * v4[t][1];
                    }
                }
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int col = u.col0 + wave * CPW + c;
        if (live && col < ncols) {
            const int crow = col_row(col, M.invG);
            const int64_t orow = (int64_t)(g.grow0 + crow) * M.Hq + g.kvh * M.G + (col - crow * M.G);
            *reinterpret_cast<uint32_t*>(M.out + orow * D + d) = pack_bf16((o0[c] / l[c]) * M.v_scale, (o1[c] / l[c]) * M.v_scale);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Paged KV append (and, with several layers in one launch, the landing of transferred KV).  One workgroup
// moves 8 consecutive tokens of the batch for one KV head of one layer.
// K: 16-byte granules (8 d of one token), lanes ordered token-minor so that tokens in consecutive slots
//    write 128 contiguous bytes.
// V: a granule is 8 tokens of one d, i.e. 8 consecutive slots starting at a multiple of 8.  The new tokens of a
//    sequence sit in consecutive slots but start anywhere (at its cached length), so the workgroup's own 8
//    tokens rarely fill one granule; run of 8 batch tokens that do ("octets") are found in a window of slots
//    around the workgroup's tokens instead: the workgroup writes, as whole 16-byte granules, the octet that
//    STARTS at one of its tokens (there is at most one; its tokens may reach into the next workgroup's range,
//    which only reads them), and element by element those of its tokens that belong to no octet (heads and tails
//    of runs, skipped neighbours).  Every token is written exactly once.
// ---------------------------------------------------------------------------------------------------
// source and pool are each touched once: non-temporal loads and stores (the landing of a whole request runs 7 %
// faster with them)
#define APPEND_LOAD(p) __builtin_nontemporal_load(p)
#define APPEND_STORE(v, p) __builtin_nontemporal_store(v, p)
// FP8: the pool's elements are bytes; element x of K is stored as the code of x * inv_k (of V: x * inv_v), one
// binary32 product each.
template <bool FP8>
__global__ __launch_bounds__(kSmallThreads) void ppd_kv_append_kernel(const uint16_t* __restrict__ k,
                                                                 const uint16_t* __restrict__ v,
                                                                 std::conditional_t<FP8, uint8_t, uint16_t>* __restrict__ pool,
                                                                 const int64_t* __restrict__ slots, int64_t T,
                                                                 int Hkv, int D, int64_t num_pages,
                                                                 int64_t pool_layer_stride, uint32_t* err_flags,
                                                                 float inv_k, float inv_v) {
    auto code_pair = [](uint32_t two_bf16, float inv) {  // the codes of the two bf16 of a dword, low one first
        return e4m3_code(bf16_bits_to_f32(two_bf16 & 0xFFFFu) * inv) | (e4m3_code(bf16_bits_to_f32(two_bf16 >> 16) * inv) << 8);
    };
    // blockIdx.z = layer: source layers are contiguous [layer][T][Hkv][D], pools pool_layer_stride apart
    k += (int64_t)blockIdx.z * T * Hkv * D;
    v += (int64_t)blockIdx.z * T * Hkv * D;
    pool += (int64_t)blockIdx.z * pool_layer_stride;
    const int tid = threadIdx.x;
    const int hh = blockIdx.y;
    const int64_t t0 = (int64_t)blockIdx.x * 8;
    // Window of slots: batch tokens t0-7 .. t0+14, one per lane (lane 7 holds token t0), in every wave; tokens
    // outside the batch and slots outside the pool count as skipped.  What follows is a handful of wave-wide
    // votes: the per-workgroup bookkeeping has to stay far below the cost of moving 8 tokens.
    constexpr int kWin = 22;
    const int lane = tid & 63;
    const int64_t tw = t0 - 7 + lane;
    int64_t ws = -1;
    if (lane < kWin && tw >= 0 && tw < T) ws = slots[tw];
    const bool outside = ws >= num_pages * kPage;
    if (__ballot(outside && lane >= 7 && lane < 15) != 0 && tid == 0 && hh == 0 && blockIdx.z == 0)
        atomicOr(err_flags, 1u);
    if (outside) ws = -1;
    // bit i of `runs`: entry i+1 holds the slot after entry i's; bit c of `octets`: the 8 tokens from entry c on
    // sit in the 8 slots of one V granule, in order
    const int64_t ws_next = __shfl_down(ws, 1);
    const uint64_t runs = __ballot(lane < kWin - 1 && ws_next == ws + 1);
    const uint64_t starts = __ballot(ws >= 0 && (ws & 7) == 0);
    const uint32_t octets = (uint32_t)(starts & runs & (runs >> 1) & (runs >> 2) & (runs >> 3) & (runs >> 4) &
                                       (runs >> 5) & (runs >> 6)) & 0x7FFFu;
    // own tokens: which of them no octet covers (a token with slot s would be entry s % 8 of one), and the
    // octet that starts at one of them
    const int my_start = (ws >= 0 && lane >= 7) ? lane - (int)(ws & 7) : 0;
    const uint32_t single =
        (uint32_t)(__ballot(lane >= 7 && lane < 15 && ws >= 0 && !((octets >> my_start) & 1u)) >> 7) & 0xFFu;
    const uint32_t own_octets = (octets >> 7) & 0xFFu;
    const int oct_tok = own_octets ? __builtin_ctz(own_octets) : 0;
    const int64_t oct_first = __shfl(ws, 7 + oct_tok);
    const int64_t oct_slot = own_octets ? oct_first : -1;
    const int64_t S = 2LL * Hkv * kPage * D;
    const int HD = Hkv * D;
    const int64_t koff = (int64_t)hh * kPage * D;
    const int64_t voff = (int64_t)Hkv * kPage * D + koff;
    // K (lower half of the threads): work unit = (granule c, token), token fastest
    constexpr int kHalf = kSmallThreads / 2;
    const int kunits = (D / 8) * 8;
    for (int u = tid; u < kunits && tid < kHalf; u += kHalf) {
        const int tok = u & 7, c = u >> 3;
        const int64_t s = __shfl(ws, 7 + tok);  // every lane of the wave is here: D is a multiple of 64
        if (s < 0) continue;
        const u32x4 val = APPEND_LOAD(reinterpret_cast<const u32x4*>(k + (t0 + tok) * HD + hh * D + c * 8));
        auto* dst = pool + (s >> 4) * S + koff + c * (kPage * 8) + (int)(s & 15) * 8;
        if constexpr (FP8) {
            const u32x2 codes = {code_pair(val[0], inv_k) | (code_pair(val[1], inv_k) << 16),
                                 code_pair(val[2], inv_k) | (code_pair(val[3], inv_k) << 16)};
            APPEND_STORE(codes, reinterpret_cast<u32x2*>(dst));
        } else {
            APPEND_STORE(val, reinterpret_cast<u32x4*>(dst));
        }
    }
    // V, whole granules (upper half of the threads, at the same time as K): work unit = d
    if (oct_slot >= 0 && tid >= kHalf) {
        const int64_t page = oct_slot >> 4;
        const int half = (int)((oct_slot & 15) >> 3);
        const uint16_t* src = v + (t0 + oct_tok) * HD + hh * D;
        for (int d = tid - kHalf; d < D; d += kHalf) {
            uint32_t g[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t lo = APPEND_LOAD(src + (2 * e) * HD + d);
                const uint32_t hi = APPEND_LOAD(src + (2 * e + 1) * HD + d);
                g[e] = lo | (hi << 16);
            }
            auto* dst = pool + page * S + voff + half * (D * 8) + d * 8;
            if constexpr (FP8) {
                const u32x2 codes = {code_pair(g[0], inv_v) | (code_pair(g[1], inv_v) << 16),
                                     code_pair(g[2], inv_v) | (code_pair(g[3], inv_v) << 16)};
                APPEND_STORE(codes, reinterpret_cast<u32x2*>(dst));
            } else {
                APPEND_STORE((u32x4{g[0], g[1], g[2], g[3]}), reinterpret_cast<u32x4*>(dst));
            }
        }
    }
    // V, element by element: work unit = (token, d)
    if (single) {
        for (int u = tid; u < D * 8; u += kSmallThreads) {
            const int tok = u / D, d = u % D;
            const int64_t s = __shfl(ws, 7 + tok);  // before any lane drops out
            if (!((single >> tok) & 1u)) continue;
            const int off = (int)(s & 15);
            const uint16_t x = v[(t0 + tok) * HD + hh * D + d];
            auto* dst = pool + (s >> 4) * S + voff + (off >> 3) * (D * 8) + d * 8 + (off & 7);
            if constexpr (FP8) *dst = (uint8_t)e4m3_code(bf16_bits_to_f32(x) * inv_v); else *dst = x;
        }
    }
}

// ---------------------------------------------------------------------------------------------------
static size_t ring_lds_bytes(int head_dim) {
    return (size_t)(2 * kStages + (PPD_PINGPONG ? 1 : 0) + (PPD_PINGPONG ? 1 : 0)) * 4 * kPage * head_dim * 2 +
           (kMaxMfmaChunk / kPage) * 4;  // + page ids of one row-block tile
}
static size_t mixed_lds_bytes(int head_dim) {
    const size_t rings = ring_lds_bytes(head_dim), combine = NarrowCombine<kWaves>::bytes(head_dim);
    return rings > combine ? rings : combine;
}

// More than 64 KiB of dynamic LDS has to be allowed per kernel, on the device that is current (ppd_create calls
// this once per context, with the context's device current).
int prepare_mixed_kernels() {
    hipError_t e = hipSuccess;
    auto allow = [&](const void* fn, size_t bytes) {
        if (e == hipSuccess) e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    };
    allow(reinterpret_cast<const void*>(&ppd_mixed_kernel<128, false>), mixed_lds_bytes(128));
    allow(reinterpret_cast<const void*>(&ppd_mixed_kernel<64, false>), mixed_lds_bytes(64));
    allow(reinterpret_cast<const void*>(&ppd_mixed_kernel<128, true>), mixed_lds_bytes(128));
    allow(reinterpret_cast<const void*>(&ppd_mixed_kernel<64, true>), mixed_lds_bytes(64));
    allow(reinterpret_cast<const void*>(&ppd_narrow_kernel<128, false, kNarrowKernelWaves>), NarrowCombine<kNarrowKernelWaves>::bytes(128));
    allow(reinterpret_cast<const void*>(&ppd_narrow_kernel<64, false, kNarrowKernelWaves>), NarrowCombine<kNarrowKernelWaves>::bytes(64));
    allow(reinterpret_cast<const void*>(&ppd_narrow_kernel<128, true, kNarrowKernelWaves>), NarrowCombine<kNarrowKernelWaves>::bytes(128));
    allow(reinterpret_cast<const void*>(&ppd_narrow_kernel<64, true, kNarrowKernelWaves>), NarrowCombine<kNarrowKernelWaves>::bytes(64));
    allow(reinterpret_cast<const void*>(&ppd_mfma_kernel<128>), ring_lds_bytes(128));
    allow(reinterpret_cast<const void*>(&ppd_mfma_kernel<64>), ring_lds_bytes(64));
    return (int)e;
}

int launch_mixed(const KParams& p, int head_dim, int grid, void* stream, bool fp8_pages) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (head_dim == 128 && !fp8_pages)
        hipLaunchKernelGGL((ppd_mixed_kernel<128, false>), dim3(grid), dim3(kThreads), mixed_lds_bytes(128), st, p);
    else if (head_dim == 128)
        hipLaunchKernelGGL((ppd_mixed_kernel<128, true>), dim3(grid), dim3(kThreads), mixed_lds_bytes(128), st, p);
    else if (!fp8_pages)
        hipLaunchKernelGGL((ppd_mixed_kernel<64, false>), dim3(grid), dim3(kThreads), mixed_lds_bytes(64), st, p);
    else
        hipLaunchKernelGGL((ppd_mixed_kernel<64, true>), dim3(grid), dim3(kThreads), mixed_lds_bytes(64), st, p);
    return (int)hipGetLastError();
}

int launch_narrow(const KParams& p, int head_dim, int grid, void* stream, bool fp8_pages) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    constexpr int NW = kNarrowKernelWaves;
    const size_t lds128 = NarrowCombine<NW>::bytes(128), lds64 = NarrowCombine<NW>::bytes(64);
    if (head_dim == 128 && !fp8_pages)
        hipLaunchKernelGGL((ppd_narrow_kernel<128, false, NW>), dim3(grid), dim3(64 * NW), lds128, st, p);
    else if (head_dim == 128)
        hipLaunchKernelGGL((ppd_narrow_kernel<128, true, NW>), dim3(grid), dim3(64 * NW), lds128, st, p);
    else if (!fp8_pages)
        hipLaunchKernelGGL((ppd_narrow_kernel<64, false, NW>), dim3(grid), dim3(64 * NW), lds64, st, p);
    else
        hipLaunchKernelGGL((ppd_narrow_kernel<64, true, NW>), dim3(grid), dim3(64 * NW), lds64, st, p);
    return (int)hipGetLastError();
}

int launch_mfma_only(const KParams& p, int head_dim, int grid, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (head_dim == 128)
        hipLaunchKernelGGL(ppd_mfma_kernel<128>, dim3(grid), dim3(kThreads), ring_lds_bytes(128), st, p);
    else
        hipLaunchKernelGGL(ppd_mfma_kernel<64>, dim3(grid), dim3(kThreads), ring_lds_bytes(64), st, p);
    return (int)hipGetLastError();
}

int launch_stream_only(const KParams& p, int head_dim, int grid, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (head_dim == 128)
        hipLaunchKernelGGL(ppd_stream_kernel<128>, dim3(grid), dim3(kStreamThreads),
                           NarrowCombine<kStreamWaves>::bytes(128), st, p);
    else
        hipLaunchKernelGGL(ppd_stream_kernel<64>, dim3(grid), dim3(kStreamThreads),
                           NarrowCombine<kStreamWaves>::bytes(64), st, p);
    return (int)hipGetLastError();
}

int launch_merge(const MergeParams& p, void* stream) {
    hipLaunchKernelGGL(ppd_merge_kernel, dim3(p.n_units), dim3(kSmallThreads), 0, static_cast<hipStream_t>(stream), p);
    return (int)hipGetLastError();
}

int launch_kv_append(const uint16_t* k, const uint16_t* v, void* pool, const int64_t* slots, int64_t T, int Hkv,
                     int D, int64_t num_pages, int layers, int64_t pool_layer_stride, uint32_t* err_flags,
                     void* stream, bool fp8_pages, float inv_k_scale, float inv_v_scale) {
    const int64_t blocks = (T + 7) / 8;
    const dim3 grid((unsigned)blocks, (unsigned)Hkv, (unsigned)layers);
    if (fp8_pages)
        hipLaunchKernelGGL(ppd_kv_append_kernel<true>, grid, dim3(kSmallThreads), 0, static_cast<hipStream_t>(stream), k, v,
                           static_cast<uint8_t*>(pool), slots, T, Hkv, D, num_pages, pool_layer_stride, err_flags,
                           inv_k_scale, inv_v_scale);
    else
        hipLaunchKernelGGL(ppd_kv_append_kernel<false>, grid, dim3(kSmallThreads), 0, static_cast<hipStream_t>(stream), k, v,
                           static_cast<uint16_t*>(pool), slots, T, Hkv, D, num_pages, pool_layer_stride, err_flags,
                           inv_k_scale, inv_v_scale);
    return (int)hipGetLastError();
}

}  // namespace ppd
