// Internal declarations shared by the host planner, the host API and the kernels of libppd.
#pragma once
#include <stdint.h>

#include <vector>

#include "../../include/ppd.h"

namespace ppd {

constexpr int kPage = 16;            // tokens per page
constexpr int kMaxTiles = 1 << 22;   // work-list entries of one launch (a 128K-token full prefill needs ~10^5)
constexpr int kNarrowCols = 16;      // a narrow tile holds rows*G <= 16 query columns
#ifndef PPD_WAVES
#define PPD_WAVES 8
#endif
#ifndef PPD_STAGES
#define PPD_STAGES 3
#endif
constexpr int kWaves = PPD_WAVES;            // waves per workgroup of the mixed kernel
constexpr int kThreads = 64 * kWaves;
constexpr int kMfmaCols = 32 * kWaves;       // an MFMA row-block tile holds up to 32 query columns per wave
constexpr int kStages = PPD_STAGES;          // prefetch distance of the K tiles (V: one less); the LDS rings have one stage more
constexpr int kWgPerCu = kWaves == 8 ? 1 : 2;  // resident workgroups per compute unit (256 VGPRs per wave)
constexpr int kTileTokens = 64;      // key tile of the MFMA path; every split boundary is a multiple of it
constexpr int kMaxMfmaChunk = 32768;  // keys per MFMA row-block tile at most (its 2048 page ids are staged in LDS)
constexpr int kSmallThreads = 256;   // block size of the append and merge kernels
// The co-resident pair (a step with both kinds of tiles): the stream kernel's workgroup is kStreamWaves waves, one
// per SIMD, each with kStreamKSets rotating register sets for the K half of a page and kStreamVSets for the V half
// (K of kStreamKSets - 1 pages and V of kStreamVSets - 1 pages in flight per wave: what 168 registers hold).
constexpr int kStreamWaves = 4;
constexpr int kStreamThreads = 64 * kStreamWaves;
#ifndef PPD_STREAM_KSETS
#define PPD_STREAM_KSETS 3
#endif
#ifndef PPD_STREAM_VSETS
#define PPD_STREAM_VSETS 2
#endif
constexpr int kStreamKSets = PPD_STREAM_KSETS;
constexpr int kStreamVSets = PPD_STREAM_VSETS;
#ifndef PPD_FP8_SETS
#define PPD_FP8_SETS 2
#endif
constexpr int kFp8StreamSets = PPD_FP8_SETS;  // rotating register sets (one page pair each) of a streaming wave on FP8 pages
// Waves per workgroup of ppd_narrow_kernel.  Two workgroups of four waves per unit (two tiles in flight there) measured
// the same on short tiles and 10 % slower on cfg2, so it runs its tiles exactly as ppd_mixed_kernel does.
constexpr int kNarrowKernelWaves = kWaves;
constexpr int kXcds = 8;             // MFMA tile queues, one per XCD (each XCD has its own L2)
constexpr int kNarrowQueue = kXcds;  // index of the narrow-tile queue
// Very short narrow tiles of a launch that has very many of them are handed out kWaves at a time (one claim), each
// wave running one tile on its own: no combine through LDS, no barrier, and the fixed costs of a tile (claim, work
// item, page ids, first loads) overlap across the eight tiles instead of adding up.  Only worth it while a tile is
// far shorter than the launch: a wave alone streams slowly, so long tiles would stretch the end of the launch.
constexpr int kWaveQueue = kXcds + 1;       // index of that queue; a claim covers kWaves consecutive tiles
constexpr int kQueues = kXcds + 2;
constexpr int kCursors = kQueues;           // one cursor per queue
#ifndef PPD_WAVE_TILE_KEYS
#define PPD_WAVE_TILE_KEYS 384
#endif
constexpr int kWaveTileKeys = PPD_WAVE_TILE_KEYS;  // a narrow tile of at most this many keys may run on one wave
// Device counters of a context: 64 words of flags (word 9: sticky error flags; words 10 and 11: finished
// workgroups of the mixed / row-block kernel and of the stream kernel), then the queue cursors, each in a
// 128-byte line of its own (claims on different queues then do not queue up behind one another at one address
// range of the memory side, where device-scope atomics execute).
constexpr int kCursorBase = 64;    // word index of cursor 0
constexpr int kCursorStride = 32;  // words between cursors
constexpr int kCounterWords = kCursorBase + kCursors * kCursorStride;
constexpr int kMergeCols = 16;     // columns of a merge group one block of the merge kernel takes

// One merge group: a row block whose key range was split over `nsplit` tiles with consecutive partials.
struct MergeGroup {
    int32_t grow0;
    int32_t nrows;
    int32_t kvh;
    int32_t nsplit;
    int64_t part_off;     // float offset of split 0
    int64_t part_stride;  // floats per split = cols * (D + 2)
};

// One workgroup of the merge kernel: kMergeCols consecutive columns of a group (a quarter of them per wave).
struct MergeUnit {
    int32_t group;
    int32_t col0;
};

struct Plan {
    int32_t queue_begin[kQueues + 1];  // items [queue_begin[q], queue_begin[q+1]) belong to queue q
    int32_t narrow_cus = 16;         // of the 32 compute units of an XCD, how many take narrow tiles first
    std::vector<ppd_work_item> items;
    std::vector<MergeGroup> groups;
    std::vector<MergeUnit> units;
    ppd_plan_stats stats;
};

struct PlanOptions {
    int32_t narrow_chunk = 0;
    int32_t mfma_chunk = 0;
    int32_t grid = 0;
    int32_t force_kind = -1;
    int32_t num_cus = 256;
    int32_t pref_mode = 2;
    int32_t narrow_cus = -1;  // -1: from the cost model
    int32_t wave_tiles = -1;  // -1: short narrow tiles run one per wave when the launch has enough of them; 0 never; 1 always
    int32_t kv_elem_bytes = 2;  // bytes per K/V element in the pool: 2 (bf16 pages) or 1 (FP8 E4M3 pages)
};

// Returns PPD_OK or an error code with a message in `err` (may be null).
ppd_status validate_shape(const ppd_shape* s, const char** err);
ppd_status build_plan(const ppd_shape& s, const int32_t* L, const int32_t* n, int32_t B, const PlanOptions& o,
                      Plan* plan, const char** err);

// Kernel arguments (passed by value).
struct KParams {
    const uint16_t* q;
    uint16_t* out;
    const uint16_t* pool;
    const int32_t* page_tables;
    const ppd_work_item* items;
    float* partials;
    uint32_t* counters;   // [9] sticky error flags, [10], [11] finished workgroups; queue cursors from kCursorBase on
    const int32_t* queue_begin;  // device: kQueues + 1 bounds, uploaded behind the plan's tables
    int64_t num_pages;
    int64_t page_stride;  // elements per page = 2 * Hkv * 16 * D
    int32_t n_items;
    int32_t pref_mode;    // how a workgroup picks its preferred queue (see ppd_mixed_kernel)
    int32_t narrow_cus;   // pref_mode 2: compute units per XCD (of 32) that take narrow tiles first
    int32_t max_pages;
    int32_t Hq, Hkv, G, invG;  // invG = 65536 / G + 1: col / G == (col * invG) >> 16
    float scale_log2e;    // softmax scale * log2(e), times the K scale of FP8 pages
    float v_scale;        // factor of the final output: the V scale of FP8 pages, 1 for bf16 pages
};

struct MergeParams {
    const MergeGroup* groups;
    const MergeUnit* units;
    int32_t n_units;
    const float* partials;
    uint16_t* out;
    int32_t n_groups;
    int32_t Hq, G, invG, D;
    float scale_log2e;
    float v_scale;
};

// Launchers (defined in ppd_kernels.hip); stream is a hipStream_t.
int prepare_mixed_kernels();
int launch_mixed(const KParams& p, int head_dim, int grid, void* stream, bool fp8_pages);
// a launch without row-block tiles: grid <= slots, slots = whole-workgroup tiles + ceil(one-wave tiles / kNarrowKernelWaves)
int launch_narrow(const KParams& p, int head_dim, int grid, void* stream, bool fp8_pages);
int launch_mfma_only(const KParams& p, int head_dim, int grid, void* stream);    // row-block tiles of queues 0..7
int launch_stream_only(const KParams& p, int head_dim, int grid, void* stream);  // narrow tiles of queue 8
int launch_merge(const MergeParams& p, void* stream);
// fp8_pages: the pool holds one-byte FP8 E4M3 codes of x * inv_k_scale (K) and x * inv_v_scale (V)
int launch_kv_append(const uint16_t* k, const uint16_t* v, void* pool, const int64_t* slots, int64_t T,
                     int Hkv, int D, int64_t num_pages, int layers, int64_t pool_layer_stride, uint32_t* err_flags,
                     void* stream, bool fp8_pages, float inv_k_scale, float inv_v_scale);

}  // namespace ppd
