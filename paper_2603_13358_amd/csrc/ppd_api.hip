// Host side of libppd: context, argument checks, plan upload and kernel launches behind the C ABI.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "ppd_internal.h"

namespace {

thread_local std::string g_create_error;

constexpr int kStagingSlots = 4;
constexpr size_t kMaxTimedLaunches = 4096;

struct Staging {
    void* host = nullptr;  // pinned
    size_t bytes = 0;
    hipEvent_t done = nullptr;
    bool in_flight = false;
};

}  // namespace

struct ppd_ctx {
    ppd_shape shape;
    int device = 0;
    int num_cus = 256;
    ppd::PlanOptions opts;
    std::string error;
    ppd::Plan plan;
    // device workspace
    void* d_items = nullptr;
    size_t d_items_bytes = 0;
    float* d_partials = nullptr;
    size_t d_partials_floats = 0;
    uint32_t* d_counters = nullptr;  // kCounterWords words: error flags, finished-workgroup counts, queue cursors
    Staging staging[kStagingSlots];
    int next_slot = 0;
    // the plan on the device stays valid while L, n and the planner options do not change (the layers of one
    // engine step call with the same lengths): such calls skip planning and upload
    std::vector<int32_t> plan_L, plan_n;
    ppd::PlanOptions plan_opts;
    bool plan_on_device = false;
    // where that plan lives: 1 = the context's own workspace, 2 = the library's static scratch array
    int plan_where = 0;
    hipStream_t plan_stream = nullptr;  // the stream the plan was uploaded on and the last call ran on
    bool have_plan_stream = false;
    // the co-resident pair: the stream kernel runs on a stream of the context's own, forked from and joined to the
    // caller's stream with these events
    hipStream_t side_stream = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    int launch_mode = 0;  // option "launch_mode"
    bool narrow_kernel = true;  // option "narrow_kernel": launches without row-block tiles run ppd_narrow_kernel
    // element format of the pools (ppd_set_kv_format): FP8 E4M3 codes with one scale per tensor, or bf16
    bool fp8_pages = false;
    float k_scale = 1.f, v_scale = 1.f;
    // debugging aids switched on by environment variables read in ppd_create
    bool log_calls = false;          // PPD_LOG=1: one line per call on stderr
    uint32_t* d_slot_seen = nullptr;  // PPD_DEBUG_SLOTS=1: one bit per pool slot, to find duplicate slots of an append
    // pinned staging of the entry point that allocates nothing (fixed size, allocated with the context)
    void* static_staging = nullptr;
    hipEvent_t static_staging_done = nullptr;
    bool static_staging_in_flight = false;
    // optional timing of the attention kernels alone (option "timing"): one pair of events per call since the option
    // was set or the times were last collected, up to kMaxTimedLaunches
    bool timing = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_pairs;
    size_t ev_used = 0;
};

namespace {

ppd_status fail(ppd_ctx* ctx, ppd_status st, const std::string& msg) {
    if (ctx) ctx->error = msg; else g_create_error = msg;
    return st;
}

ppd_status hip_fail(ppd_ctx* ctx, hipError_t e, const char* what) {
    return fail(ctx, PPD_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define PPD_HIP(ctx, call)                                         \
    do {                                                           \
        hipError_t e_ = (call);                                    \
        if (e_ != hipSuccess) return hip_fail((ctx), e_, #call);   \
    } while (0)

// Grows a device buffer (contents are not kept).  Waits for the stream first: the old buffer may be in use.
ppd_status grow_device(ppd_ctx* ctx, void** ptr, size_t* have, size_t need, hipStream_t st) {
    if (need <= *have) return PPD_OK;
    PPD_HIP(ctx, hipStreamSynchronize(st));
    if (*ptr) PPD_HIP(ctx, hipFree(*ptr));
    *ptr = nullptr;
    *have = 0;
    size_t want = need + need / 4 + 4096;
    if (hipMalloc(ptr, want) != hipSuccess) {
        (void)hipGetLastError();
        *ptr = nullptr;
        return fail(ctx, PPD_ERR_WORKSPACE, "workspace allocation of " + std::to_string(want) + " bytes failed");
    }
    *have = want;
    return PPD_OK;
}

// The kernels move 16 bytes per lane: tensors and pools must start on a 16-byte boundary.
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- the static scratch array of the entry point that allocates nothing -------------------------------------
// One array per GPU the library runs on, held until the process ends: queue counters, the uploaded plan and the
// split partials of ppd_mixed_attention_static.  Host code never passes the array's name to a kernel (on the host
// it is only a stand-in): the device address is asked for once per device and kept in g_scratch_ptr.
constexpr size_t kStaticCounterBytes = 4096;
constexpr size_t kStaticPlanBytes = (size_t(2) << 20) - kStaticCounterBytes;
constexpr size_t kStaticPartialBytes = PPD_STATIC_SCRATCH_BYTES - (size_t(2) << 20);
static_assert(ppd::kCounterWords * sizeof(uint32_t) <= kStaticCounterBytes, "counters fit their slot");
static __device__ __align__(256) unsigned char scratch[PPD_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {nullptr};
// which context's plan the array of a device holds (nullptr: none), and that plan's serial number
const ppd_ctx* g_scratch_owner[kMaxDevices] = {nullptr};

// Device address of this device's copy of the array; the device must be current.
hipError_t static_scratch_address(int device, unsigned char** out) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

// Zeroes the queue cursors and the finished-workgroup counts of a counter block (not the sticky error flags).  A
// kernel rather than a memset: a memset node recorded into a captured graph has replayed wrongly on this platform.
__global__ void ppd_clear_counters_kernel(uint32_t* counters) {
    for (int i = threadIdx.x; i < ppd::kCounterWords; i += blockDim.x)
        if (i == 10 || i == 11 || i >= ppd::kCursorBase) counters[i] = 0u;
}

// Debugging aid (PPD_DEBUG_SLOTS=1): marks every slot of an append in a bitmap; a bit found set already is a
// duplicate slot within the call (error flag bit 2).  The second pass clears the bits again.
__global__ void ppd_mark_slots_kernel(const int64_t* slots, int64_t T, int64_t pool_slots, uint32_t* seen, uint32_t* flags,
                                      int clear) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const int64_t s = slots[t];
    if (s < 0 || s >= pool_slots) return;
    const uint32_t bit = 1u << (s & 31);
    if (clear) {
        atomicAnd(&seen[s >> 5], ~bit);
    } else if (atomicOr(&seen[s >> 5], bit) & bit) {
        atomicOr(flags, 4u);
    }
}

// PPD_DEBUG_SLOTS=1: looks for duplicate slots among the T slots of an append (error flag bit 2), on `stream`.
void check_duplicate_slots(ppd_ctx* ctx, const int64_t* slot_mapping, int64_t T, hipStream_t hs) {
    if (!ctx->d_slot_seen || T <= 0) return;
    const int64_t pool_slots = ctx->shape.num_pages * ppd::kPage;
    const unsigned blocks = (unsigned)((T + 255) / 256);
    for (int clear = 0; clear < 2; ++clear)
        hipLaunchKernelGGL(ppd_mark_slots_kernel, dim3(blocks), dim3(256), 0, hs, slot_mapping, T, pool_slots, ctx->d_slot_seen,
                           ctx->d_counters + 9, clear);
}

ppd_status mixed_attention_impl(ppd_ctx* ctx, const void* q, const void* kv_pages, const int32_t* page_tables,
                                int32_t max_pages, const int32_t* L, const int32_t* n, int32_t B, float scale,
                                void* out, void* stream, bool use_static) {
    if (!ctx) return PPD_ERR_NULL;
    if (B < 0) return fail(ctx, PPD_ERR_RANGE, "B < 0");
    if (B == 0) {
        ctx->plan.items.clear();
        ctx->plan.groups.clear();
        ctx->plan.units.clear();
        ctx->plan_on_device = false;
        std::memset(&ctx->plan.stats, 0, sizeof ctx->plan.stats);
        return PPD_OK;
    }
    if (!q || !kv_pages || !page_tables || !L || !n || !out)
        return fail(ctx, PPD_ERR_NULL, "q / kv_pages / page_tables / L / n / out is NULL");
    if (!(scale >= 0.f) || !std::isfinite(scale)) return fail(ctx, PPD_ERR_RANGE, "scale must be finite and >= 0");
    if (!aligned16(q) || !aligned16(out) || !aligned16(kv_pages) || (reinterpret_cast<uintptr_t>(page_tables) & 3u))
        return fail(ctx, PPD_ERR_RANGE, "q / out / kv_pages must be 16-byte aligned, page_tables 4-byte aligned");
    for (int i = 0; i < B; ++i) {
        if (n[i] < 1 || L[i] < 0) return fail(ctx, PPD_ERR_RANGE, "n_i must be >= 1 and L_i >= 0");
        const int64_t need = ((int64_t)L[i] + n[i] + ppd::kPage - 1) / ppd::kPage;
        if (need > max_pages)
            return fail(ctx, PPD_ERR_PAGETABLE, "sequence " + std::to_string(i) + " needs " + std::to_string(need) +
                                                    " pages, max_pages is " + std::to_string(max_pages));
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
    PPD_HIP(ctx, hipSetDevice(ctx->device));
    const char* msg = "";
    ppd_status st = PPD_OK;
    const int where = use_static ? 2 : 1;
    if (ctx->fp8_pages && ctx->launch_mode != 0)
        return fail(ctx, PPD_ERR_RANGE, "FP8 pages are read by the one-launch kernel only: set launch_mode to 0");
    ppd::PlanOptions opts = ctx->opts;
    if (ctx->launch_mode != 0) opts.wave_tiles = 0;  // the specialised kernels run every narrow tile on four waves
    opts.kv_elem_bytes = ctx->fp8_pages ? 1 : 2;
    const bool same_opts = std::memcmp(&ctx->plan_opts, &opts, sizeof(ppd::PlanOptions)) == 0;
    const bool reuse = ctx->plan_on_device && ctx->plan_where == where && same_opts &&
                       (!use_static || g_scratch_owner[ctx->device] == ctx) && (int32_t)ctx->plan_L.size() == B &&
                       std::memcmp(ctx->plan_L.data(), L, sizeof(int32_t) * B) == 0 &&
                       std::memcmp(ctx->plan_n.data(), n, sizeof(int32_t) * B) == 0;
    // A context serves one stream at a time.  When the caller moves to another stream, the work enqueued on the
    // previous one (the plan upload, kernels that share the queue counters) has to finish first.  Under capture
    // nothing runs yet and no synchronisation is allowed: there the caller answers for the order.
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    PPD_HIP(ctx, hipStreamIsCapturing(hs, &capturing));
    const bool in_capture = capturing != hipStreamCaptureStatusNone;
    if (!in_capture && ctx->have_plan_stream && ctx->plan_stream != hs) PPD_HIP(ctx, hipStreamSynchronize(ctx->plan_stream));
    if (!reuse && in_capture)
        return fail(ctx, PPD_ERR_RANGE, "plan changed under capture: run the step once eagerly with these L, n and "
                                        "options first, then capture it");
    const auto t_plan0 = std::chrono::steady_clock::now();
    if (!reuse) {
        ctx->plan_on_device = false;
        st = ppd::build_plan(ctx->shape, L, n, B, opts, &ctx->plan, &msg);
        if (st != PPD_OK) return fail(ctx, st, msg);
    }

    const ppd::Plan& plan = ctx->plan;
    const size_t items_bytes = plan.items.size() * sizeof(ppd_work_item);
    const size_t groups_bytes = plan.groups.size() * sizeof(ppd::MergeGroup);
    const size_t units_bytes = plan.units.size() * sizeof(ppd::MergeUnit);
    const size_t bounds_bytes = sizeof plan.queue_begin;  // the queues' bounds travel behind the tables
    const size_t total = items_bytes + groups_bytes + units_bytes + bounds_bytes;
    unsigned char* sbase = nullptr;
    if (use_static) {
        PPD_HIP(ctx, static_scratch_address(ctx->device, &sbase));
        if (total > kStaticPlanBytes || (size_t)plan.stats.partial_floats * sizeof(float) > kStaticPartialBytes)
            return fail(ctx, PPD_ERR_WORKSPACE,
                        "batch too large for the static scratch array: plan " + std::to_string(total) + " of " +
                            std::to_string(kStaticPlanBytes) + " bytes, split partials " +
                            std::to_string((size_t)plan.stats.partial_floats * sizeof(float)) + " of " +
                            std::to_string(kStaticPartialBytes) + " bytes; use ppd_mixed_attention");
    }
    void* d_plan = use_static ? static_cast<void*>(sbase + kStaticCounterBytes) : nullptr;
    if (!reuse) {
        // upload: [items][groups][units] through pinned staging
        void* host = nullptr;
        hipEvent_t done = nullptr;
        if (use_static) {
            if (ctx->static_staging_in_flight) {
                PPD_HIP(ctx, hipEventSynchronize(ctx->static_staging_done));
                ctx->static_staging_in_flight = false;
            }
            host = ctx->static_staging;
            done = ctx->static_staging_done;
        } else {
            Staging& sg = ctx->staging[ctx->next_slot];
            ctx->next_slot = (ctx->next_slot + 1) % kStagingSlots;
            if (sg.in_flight) {
                PPD_HIP(ctx, hipEventSynchronize(sg.done));
                sg.in_flight = false;
            }
            if (sg.bytes < total) {
                if (sg.host) PPD_HIP(ctx, hipHostFree(sg.host));
                sg.host = nullptr;
                sg.bytes = 0;
                const size_t want = total + total / 4 + 4096;
                if (hipHostMalloc(&sg.host, want, hipHostMallocDefault) != hipSuccess) {
                    (void)hipGetLastError();
                    sg.host = nullptr;
                    return fail(ctx, PPD_ERR_WORKSPACE, "pinned staging allocation failed");
                }
                sg.bytes = want;
            }
            st = grow_device(ctx, &ctx->d_items, &ctx->d_items_bytes, total, hs);
            if (st != PPD_OK) return st;
            {
                void* p = ctx->d_partials;
                size_t have = ctx->d_partials_floats * sizeof(float);
                st = grow_device(ctx, &p, &have, (size_t)plan.stats.partial_floats * sizeof(float), hs);
                ctx->d_partials = static_cast<float*>(p);
                ctx->d_partials_floats = have / sizeof(float);
                if (st != PPD_OK) return st;
            }
            host = sg.host;
            done = sg.done;
            sg.in_flight = true;
        }
        std::memcpy(host, plan.items.data(), items_bytes);
        if (groups_bytes) {
            std::memcpy(static_cast<char*>(host) + items_bytes, plan.groups.data(), groups_bytes);
            std::memcpy(static_cast<char*>(host) + items_bytes + groups_bytes, plan.units.data(), units_bytes);
        }
        std::memcpy(static_cast<char*>(host) + total - bounds_bytes, plan.queue_begin, bounds_bytes);
        PPD_HIP(ctx, hipMemcpyAsync(use_static ? d_plan : ctx->d_items, host, total, hipMemcpyHostToDevice, hs));
        PPD_HIP(ctx, hipEventRecord(done, hs));
        if (use_static) {
            ctx->static_staging_in_flight = true;
            g_scratch_owner[ctx->device] = ctx;
        }
        ctx->plan_L.assign(L, L + B);
        ctx->plan_n.assign(n, n + B);
        ctx->plan_opts = opts;
        ctx->plan_on_device = true;
        ctx->plan_where = where;
        ctx->plan.stats.plan_host_us = (int32_t)std::chrono::duration_cast<std::chrono::microseconds>(
                                           std::chrono::steady_clock::now() - t_plan0).count();
    }
    if (!use_static) d_plan = ctx->d_items;
    if (!in_capture) {
        ctx->plan_stream = hs;
        ctx->have_plan_stream = true;
    }

    const int G = ctx->shape.num_q_heads / ctx->shape.num_kv_heads;
    // Masked scores are -inf and enter the exponent as s*c: keep c strictly positive so that scale = 0 gives
    // 2^(-inf) = 0 for masked keys and 2^(~0) = 1 for visible ones (identical to the exact result in fp32).
    float scale_log2e = scale * 1.4426950408889634f;
    if (ctx->fp8_pages) scale_log2e = (float)((double)scale * (double)ctx->k_scale * 1.4426950408889634);
    if (scale_log2e < 1e-30f) scale_log2e = 1e-30f;
    ppd::KParams kp;
    kp.q = static_cast<const uint16_t*>(q);
    kp.out = static_cast<uint16_t*>(out);
    kp.pool = static_cast<const uint16_t*>(kv_pages);
    kp.page_tables = page_tables;
    kp.items = static_cast<const ppd_work_item*>(d_plan);
    kp.partials = use_static ? reinterpret_cast<float*>(sbase + (size_t(2) << 20)) : ctx->d_partials;
    kp.counters = use_static ? reinterpret_cast<uint32_t*>(sbase) : ctx->d_counters;
    kp.num_pages = ctx->shape.num_pages;
    kp.page_stride = 2LL * ctx->shape.num_kv_heads * ppd::kPage * ctx->shape.head_dim;
    kp.n_items = (int32_t)plan.items.size();
    kp.queue_begin = reinterpret_cast<const int32_t*>(static_cast<const char*>(d_plan) + total - bounds_bytes);
    kp.pref_mode = ctx->opts.pref_mode;
    kp.narrow_cus = plan.narrow_cus;
    kp.max_pages = max_pages;
    kp.Hq = ctx->shape.num_q_heads;
    kp.Hkv = ctx->shape.num_kv_heads;
    kp.G = G;
    kp.invG = 65536 / G + 1;
    kp.scale_log2e = scale_log2e;
    kp.v_scale = ctx->fp8_pages ? ctx->v_scale : 1.f;
    // The static array is shared by every context of the process on this GPU and keeps the last call's contents:
    // the cursors and finished counts must start at zero whoever ran before.
    if (use_static)
        hipLaunchKernelGGL(ppd_clear_counters_kernel, dim3(1), dim3(512), 0, hs, kp.counters);
    const bool timed = !use_static && ctx->timing && ctx->ev_used < kMaxTimedLaunches;
    if (timed) {
        if (ctx->ev_used == ctx->ev_pairs.size()) {
            std::pair<hipEvent_t, hipEvent_t> p{nullptr, nullptr};
            PPD_HIP(ctx, hipEventCreate(&p.first));
            ctx->ev_pairs.push_back(p);  // owned by the context from here on, also if the second create fails
            PPD_HIP(ctx, hipEventCreate(&ctx->ev_pairs.back().second));
        }
        if (!ctx->ev_pairs[ctx->ev_used].second) PPD_HIP(ctx, hipEventCreate(&ctx->ev_pairs[ctx->ev_used].second));
        PPD_HIP(ctx, hipEventRecord(ctx->ev_pairs[ctx->ev_used].first, hs));
    }
    const int D = ctx->shape.head_dim;
    const bool has_narrow = plan.stats.n_narrow > 0, has_mfma = plan.stats.n_mfma > 0;
    const int mode = ctx->launch_mode;
    int rc = 0;
    if (mode == 0 && has_narrow && !has_mfma && ctx->narrow_kernel) {
        // a decode-only step: the first tiles are handed out by workgroup index, no more workgroups than there are slots
        const int64_t n_wave = plan.queue_begin[ppd::kQueues] - plan.queue_begin[ppd::kWaveQueue];
        constexpr int NW = ppd::kNarrowKernelWaves;
        const int64_t slots = (plan.queue_begin[ppd::kWaveQueue] - plan.queue_begin[ppd::kNarrowQueue]) + (n_wave + NW - 1) / NW;
        const int64_t wgs = (int64_t)plan.stats.grid * (ppd::kWaves / NW);  // as many waves on a unit as the planned grid has
        rc = ppd::launch_narrow(kp, D, (int)std::max<int64_t>(1, std::min<int64_t>(wgs, slots)), stream, ctx->fp8_pages);
        if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch narrow-tile kernel");
    } else if (mode == 0 || (mode == 1 && !(has_narrow && has_mfma))) {
        rc = ppd::launch_mixed(kp, D, plan.stats.grid, stream, ctx->fp8_pages);
        if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch mixed attention");
    } else {
        // The co-resident pair: the row-block kernel on the caller's stream, the stream kernel beside it on the
        // context's own stream, forked from and joined to the caller's stream.
        const int cus = ctx->num_cus;
        const int grid_m = has_mfma ? (int)std::min<int64_t>(cus, plan.stats.n_mfma) : 0;
        const int grid_n = has_narrow ? (int)std::min<int64_t>(has_mfma ? cus + 2 * (cus - grid_m) : 3 * cus,
                                                               plan.stats.n_narrow) : 0;
        const bool fork = grid_m > 0 && grid_n > 0;
        if (fork) {
            PPD_HIP(ctx, hipEventRecord(ctx->ev_fork, hs));
            PPD_HIP(ctx, hipStreamWaitEvent(ctx->side_stream, ctx->ev_fork, 0));
        }
        if (grid_m > 0) {
            rc = ppd::launch_mfma_only(kp, D, grid_m, stream);
            if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch row-block kernel");
        }
        if (grid_n > 0) {
            rc = ppd::launch_stream_only(kp, D, grid_n, fork ? ctx->side_stream : stream);
            if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch stream kernel");
        }
        if (fork) {
            PPD_HIP(ctx, hipEventRecord(ctx->ev_join, ctx->side_stream));
            PPD_HIP(ctx, hipStreamWaitEvent(hs, ctx->ev_join, 0));
        }
    }
    if (timed) {
        PPD_HIP(ctx, hipEventRecord(ctx->ev_pairs[ctx->ev_used].second, hs));
        ctx->ev_used += 1;
    }
    if (!plan.groups.empty()) {
        ppd::MergeParams mp;
        mp.groups = reinterpret_cast<const ppd::MergeGroup*>(static_cast<const char*>(d_plan) + items_bytes);
        mp.partials = kp.partials;
        mp.out = static_cast<uint16_t*>(out);
        mp.n_groups = (int32_t)plan.groups.size();
        mp.units = reinterpret_cast<const ppd::MergeUnit*>(static_cast<const char*>(d_plan) + items_bytes +
                                                          groups_bytes);
        mp.n_units = (int32_t)plan.units.size();
        mp.Hq = kp.Hq;
        mp.G = G;
        mp.invG = kp.invG;
        mp.D = D;
        mp.scale_log2e = scale_log2e;
        mp.v_scale = kp.v_scale;
        rc = ppd::launch_merge(mp, stream);
        if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch merge");
    }
    if (ctx->log_calls)
        std::fprintf(stderr, "ppd: mixed_attention%s%s B=%d tiles=%lld (narrow %lld of which one-wave %d, row-block %lld) merge groups=%lld "
                             "chunks=%d/%d grid=%d launch_mode=%d plan=%s (%d us)\n",
                     use_static ? "_static" : "", ctx->fp8_pages ? " (FP8 pages)" : "", (int)B, (long long)plan.stats.n_items, (long long)plan.stats.n_narrow,
                     (int)(plan.queue_begin[ppd::kQueues] - plan.queue_begin[ppd::kWaveQueue]), (long long)plan.stats.n_mfma,
                     (long long)plan.stats.n_groups, (int)plan.stats.narrow_chunk, (int)plan.stats.mfma_chunk, (int)plan.stats.grid,
                     mode, reuse ? "reused" : "built", (int)plan.stats.plan_host_us);
    return PPD_OK;
}

}  // namespace

extern "C" {

const char* ppd_version(void) { return "0.2"; }

const char* ppd_last_error(const ppd_ctx* ctx) { return ctx ? ctx->error.c_str() : g_create_error.c_str(); }

ppd_status ppd_create(const ppd_shape* shape, int32_t device, ppd_ctx** out) {
    if (!out) return fail(nullptr, PPD_ERR_NULL, "out is NULL");
    *out = nullptr;
    const char* msg = "";
    ppd_status st = ppd::validate_shape(shape, &msg);
    if (st != PPD_OK) return fail(nullptr, st, msg);
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess || count <= 0) {
        (void)hipGetLastError();
        return fail(nullptr, PPD_ERR_HIP, "no HIP device available: this library has no CPU path");
    }
    if (device < 0 || device >= count || device >= kMaxDevices)
        return fail(nullptr, PPD_ERR_RANGE, "device index out of range");
    ppd_ctx* ctx = new ppd_ctx();
    ctx->shape = *shape;
    ctx->device = device;
    auto bail = [&](hipError_t err, const char* what) {
        g_create_error = std::string(what) + ": " + hipGetErrorString(err);
        ppd_destroy(ctx);
        return PPD_ERR_HIP;
    };
    if ((e = hipSetDevice(device)) != hipSuccess) return bail(e, "hipSetDevice");
    hipDeviceProp_t prop;
    if ((e = hipGetDeviceProperties(&prop, device)) != hipSuccess) return bail(e, "hipGetDeviceProperties");
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
        g_create_error = std::string("device is ") + prop.gcnArchName + ", this library is built for gfx950 only";
        ppd_destroy(ctx);
        return PPD_ERR_HIP;
    }
    ctx->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    ctx->opts.num_cus = ctx->num_cus;
    if ((e = (hipError_t)ppd::prepare_mixed_kernels()) != hipSuccess) return bail(e, "hipFuncSetAttribute");
    const size_t counter_bytes = ppd::kCounterWords * sizeof(uint32_t);
    if ((e = hipMalloc((void**)&ctx->d_counters, counter_bytes)) != hipSuccess) return bail(e, "hipMalloc(counters)");
    if ((e = hipMemset(ctx->d_counters, 0, counter_bytes)) != hipSuccess) return bail(e, "hipMemset(counters)");
    for (auto& s : ctx->staging)
        if ((e = hipEventCreateWithFlags(&s.done, hipEventDisableTiming)) != hipSuccess) return bail(e, "hipEventCreate");
    // the stream kernel of the co-resident pair runs on a stream of the context's own (default priority)
    if ((e = hipStreamCreateWithFlags(&ctx->side_stream, hipStreamNonBlocking)) != hipSuccess) return bail(e, "hipStreamCreate");
    if ((e = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming)) != hipSuccess) return bail(e, "hipEventCreate");
    if ((e = hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming)) != hipSuccess) return bail(e, "hipEventCreate");
    // everything ppd_mixed_attention_static needs is set up here, so that the call itself allocates nothing: the
    // device address of this GPU's scratch array and a pinned staging buffer for the plan upload
    {
        unsigned char* sp = nullptr;
        if ((e = static_scratch_address(device, &sp)) != hipSuccess) return bail(e, "hipGetSymbolAddress(scratch)");
    }
    if ((e = hipHostMalloc(&ctx->static_staging, kStaticPlanBytes, hipHostMallocDefault)) != hipSuccess)
        return bail(e, "hipHostMalloc(static staging)");
    if ((e = hipEventCreateWithFlags(&ctx->static_staging_done, hipEventDisableTiming)) != hipSuccess)
        return bail(e, "hipEventCreate");
    const char* env = std::getenv("PPD_LOG");
    ctx->log_calls = env && env[0] == '1';
    env = std::getenv("PPD_DEBUG_SLOTS");
    if (env && env[0] == '1') {
        const size_t words = (size_t)((shape->num_pages * ppd::kPage + 31) / 32);
        if ((e = hipMalloc((void**)&ctx->d_slot_seen, words * sizeof(uint32_t))) != hipSuccess) return bail(e, "hipMalloc(slot bitmap)");
        if ((e = hipMemset(ctx->d_slot_seen, 0, words * sizeof(uint32_t))) != hipSuccess) return bail(e, "hipMemset(slot bitmap)");
    }
    *out = ctx;
    return PPD_OK;
}

ppd_status ppd_destroy(ppd_ctx* ctx) {
    if (!ctx) return PPD_OK;
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
    if (ctx->d_items) (void)hipFree(ctx->d_items);
    if (ctx->d_partials) (void)hipFree(ctx->d_partials);
    if (ctx->d_counters) (void)hipFree(ctx->d_counters);
    if (ctx->d_slot_seen) (void)hipFree(ctx->d_slot_seen);
    for (auto& s : ctx->staging) {
        if (s.host) (void)hipHostFree(s.host);
        if (s.done) (void)hipEventDestroy(s.done);
    }
    for (auto& p : ctx->ev_pairs) {
        if (p.first) (void)hipEventDestroy(p.first);
        if (p.second) (void)hipEventDestroy(p.second);
    }
    if (ctx->side_stream) (void)hipStreamDestroy(ctx->side_stream);
    if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
    if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
    if (ctx->static_staging) (void)hipHostFree(ctx->static_staging);
    if (ctx->static_staging_done) (void)hipEventDestroy(ctx->static_staging_done);
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (ctx->device >= 0 && ctx->device < kMaxDevices && g_scratch_owner[ctx->device] == ctx)
            g_scratch_owner[ctx->device] = nullptr;
    }
    delete ctx;
    return PPD_OK;
}

ppd_status ppd_set_option(ppd_ctx* ctx, const char* key, int64_t value) {
    if (!ctx || !key) return fail(ctx, PPD_ERR_NULL, "ctx / key is NULL");
    std::string k(key);
    if (k == "narrow_chunk" || k == "mfma_chunk") {
        if (value < 0 || value % ppd::kTileTokens || value > (1 << 30) ||
            (k == "mfma_chunk" && value > ppd::kMaxMfmaChunk))
            return fail(ctx, PPD_ERR_RANGE, k + " must be 0 or a positive multiple of 64 (mfma_chunk at most 32768)");
        (k == "narrow_chunk" ? ctx->opts.narrow_chunk : ctx->opts.mfma_chunk) = (int32_t)value;
    } else if (k == "grid") {
        if (value < 0 || value > 65536) return fail(ctx, PPD_ERR_RANGE, "grid must be in [0, 65536]");
        ctx->opts.grid = (int32_t)value;
    } else if (k == "force_kind") {
        if (value != -1 && value != 1) return fail(ctx, PPD_ERR_RANGE, "force_kind must be -1 or 1");
        ctx->opts.force_kind = (int32_t)value;
    } else if (k == "pref_mode") {
        if (value < 0 || value > 3) return fail(ctx, PPD_ERR_RANGE, "pref_mode must be in [0, 3]");
        ctx->opts.pref_mode = (int32_t)value;
    } else if (k == "narrow_cus") {
        if (value < -1 || value > 32) return fail(ctx, PPD_ERR_RANGE, "narrow_cus must be in [-1, 32]");
        ctx->opts.narrow_cus = (int32_t)value;
    } else if (k == "wave_tiles") {
        if (value < -1 || value > 1) return fail(ctx, PPD_ERR_RANGE, "wave_tiles must be -1, 0 or 1");
        ctx->opts.wave_tiles = (int32_t)value;
    } else if (k == "launch_mode") {
        if (value < 0 || value > 2) return fail(ctx, PPD_ERR_RANGE, "launch_mode must be in [0, 2]");
        ctx->launch_mode = (int)value;
    } else if (k == "narrow_kernel") {
        if (value < 0 || value > 1) return fail(ctx, PPD_ERR_RANGE, "narrow_kernel must be 0 or 1");
        ctx->narrow_kernel = value != 0;
    } else if (k == "timing") {
        ctx->timing = value != 0;
        ctx->ev_used = 0;
    } else {
        return fail(ctx, PPD_ERR_RANGE, "unknown option " + k);
    }
    return PPD_OK;
}

ppd_status ppd_set_kv_format(ppd_ctx* ctx, int32_t format, float k_scale, float v_scale) {
    if (!ctx) return PPD_ERR_NULL;
    if (format != PPD_KV_BF16 && format != PPD_KV_FP8_E4M3)
        return fail(ctx, PPD_ERR_RANGE, "format must be PPD_KV_BF16 or PPD_KV_FP8_E4M3");
    if (format == PPD_KV_FP8_E4M3) {
        if (!(k_scale > 0.f) || !(v_scale > 0.f) || !std::isfinite(k_scale) || !std::isfinite(v_scale) ||
            !std::isfinite(1.0f / k_scale) || !std::isfinite(1.0f / v_scale))
            return fail(ctx, PPD_ERR_RANGE, "k_scale and v_scale must be finite and > 0, and so must their reciprocals");
        ctx->fp8_pages = true;
        ctx->k_scale = k_scale;
        ctx->v_scale = v_scale;
    } else {
        ctx->fp8_pages = false;
        ctx->k_scale = ctx->v_scale = 1.f;
    }
    return PPD_OK;
}

ppd_status ppd_kv_append(ppd_ctx* ctx, const void* k, const void* v, void* kv_pages, const int64_t* slot_mapping,
                         int64_t T, void* stream) {
    if (!ctx) return PPD_ERR_NULL;
    if (T < 0 || T >= (int64_t(1) << 31)) return fail(ctx, PPD_ERR_RANGE, "T out of range");
    if (T == 0) return PPD_OK;
    if (!k || !v || !kv_pages || !slot_mapping) return fail(ctx, PPD_ERR_NULL, "k / v / kv_pages / slot_mapping is NULL");
    if (!aligned16(k) || !aligned16(v) || !aligned16(kv_pages) || (reinterpret_cast<uintptr_t>(slot_mapping) & 7u))
        return fail(ctx, PPD_ERR_RANGE, "k / v / kv_pages must be 16-byte aligned, slot_mapping 8-byte aligned");
    PPD_HIP(ctx, hipSetDevice(ctx->device));
    int rc = ppd::launch_kv_append(static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v), kv_pages,
                                   slot_mapping, T, ctx->shape.num_kv_heads, ctx->shape.head_dim, ctx->shape.num_pages,
                                   1, 0, ctx->d_counters + 9, stream, ctx->fp8_pages, 1.0f / ctx->k_scale,
                                   1.0f / ctx->v_scale);
    if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch kv_append");
    check_duplicate_slots(ctx, slot_mapping, T, static_cast<hipStream_t>(stream));
    if (ctx->log_calls) std::fprintf(stderr, "ppd: kv_append T=%lld\n", (long long)T);
    return PPD_OK;
}

ppd_status ppd_kv_land(ppd_ctx* ctx, const void* k, const void* v, void* kv_pages, int64_t layer_stride_elems,
                       int32_t num_layers, const int64_t* slot_mapping, int64_t T, void* stream) {
    if (!ctx) return PPD_ERR_NULL;
    if (T < 0 || T >= (int64_t(1) << 31)) return fail(ctx, PPD_ERR_RANGE, "T out of range");
    if (num_layers < 0 || num_layers > 65535) return fail(ctx, PPD_ERR_RANGE, "num_layers must be in [0, 65535]");
    if (T == 0 || num_layers == 0) return PPD_OK;
    if (!k || !v || !kv_pages || !slot_mapping) return fail(ctx, PPD_ERR_NULL, "k / v / kv_pages / slot_mapping is NULL");
    const int64_t pool_elems = 2LL * ctx->shape.num_kv_heads * ppd::kPage * ctx->shape.head_dim * ctx->shape.num_pages;
    if (num_layers > 1 && layer_stride_elems < pool_elems)
        return fail(ctx, PPD_ERR_RANGE, "layer_stride_elems is smaller than one pool: layers would overlap");
    if (!aligned16(k) || !aligned16(v) || !aligned16(kv_pages) || (reinterpret_cast<uintptr_t>(slot_mapping) & 7u) ||
        (num_layers > 1 && layer_stride_elems % (ctx->fp8_pages ? 16 : 8) != 0))
        return fail(ctx, PPD_ERR_RANGE,
                    "k / v / kv_pages must be 16-byte aligned (layer_stride_elems a multiple of 8, of 16 for FP8 pages), "
                    "slot_mapping 8-byte aligned");
    PPD_HIP(ctx, hipSetDevice(ctx->device));
    int rc = ppd::launch_kv_append(static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v), kv_pages,
                                   slot_mapping, T, ctx->shape.num_kv_heads, ctx->shape.head_dim, ctx->shape.num_pages,
                                   num_layers, layer_stride_elems, ctx->d_counters + 9, stream, ctx->fp8_pages,
                                   1.0f / ctx->k_scale, 1.0f / ctx->v_scale);
    if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch kv_land");
    check_duplicate_slots(ctx, slot_mapping, T, static_cast<hipStream_t>(stream));
    if (ctx->log_calls) std::fprintf(stderr, "ppd: kv_land T=%lld layers=%d\n", (long long)T, (int)num_layers);
    return PPD_OK;
}

ppd_status ppd_mixed_attention(ppd_ctx* ctx, const void* q, const void* kv_pages, const int32_t* page_tables,
                               int32_t max_pages, const int32_t* L, const int32_t* n, int32_t B, float scale,
                               void* out, void* stream) {
    return mixed_attention_impl(ctx, q, kv_pages, page_tables, max_pages, L, n, B, scale, out, stream, false);
}

ppd_status ppd_mixed_attention_static(ppd_ctx* ctx, const void* q, const void* kv_pages, const int32_t* page_tables,
                                      int32_t max_pages, const int32_t* L, const int32_t* n, int32_t B, float scale,
                                      void* out, void* stream) {
    return mixed_attention_impl(ctx, q, kv_pages, page_tables, max_pages, L, n, B, scale, out, stream, true);
}

ppd_status ppd_get_plan_stats(const ppd_ctx* ctx, ppd_plan_stats* stats) {
    if (!ctx || !stats) return PPD_ERR_NULL;
    *stats = ctx->plan.stats;
    return PPD_OK;
}

ppd_status ppd_last_kernel_ms(ppd_ctx* ctx, float* ms) {
    if (!ctx || !ms) return fail(ctx, PPD_ERR_NULL, "ctx / ms is NULL");
    if (ctx->ev_used == 0) return fail(ctx, PPD_ERR_RANGE, "no timed launch: set option \"timing\" to 1 and run a step");
    PPD_HIP(ctx, hipSetDevice(ctx->device));
    const auto& p = ctx->ev_pairs[ctx->ev_used - 1];
    PPD_HIP(ctx, hipEventSynchronize(p.second));
    PPD_HIP(ctx, hipEventElapsedTime(ms, p.first, p.second));
    return PPD_OK;
}

ppd_status ppd_timed_kernels_ms(ppd_ctx* ctx, double* total_ms, int32_t* launches) {
    if (!ctx || !total_ms || !launches) return fail(ctx, PPD_ERR_NULL, "ctx / total_ms / launches is NULL");
    *total_ms = 0.0;
    *launches = 0;
    PPD_HIP(ctx, hipSetDevice(ctx->device));
    double sum = 0.0;
    for (size_t i = 0; i < ctx->ev_used; ++i) {
        float ms = 0.f;
        PPD_HIP(ctx, hipEventSynchronize(ctx->ev_pairs[i].second));
        PPD_HIP(ctx, hipEventElapsedTime(&ms, ctx->ev_pairs[i].first, ctx->ev_pairs[i].second));
        sum += ms;
    }
    *total_ms = sum;
    *launches = (int32_t)ctx->ev_used;
    ctx->ev_used = 0;
    return PPD_OK;
}

ppd_status ppd_device_error_flags(ppd_ctx* ctx, void* stream, uint32_t* flags) {
    if (!ctx || !flags) return fail(ctx, PPD_ERR_NULL, "ctx / flags is NULL");
    hipStream_t hs = static_cast<hipStream_t>(stream);
    PPD_HIP(ctx, hipSetDevice(ctx->device));
    PPD_HIP(ctx, hipStreamSynchronize(hs));
    uint32_t v = 0, vs = 0;
    PPD_HIP(ctx, hipMemcpy(&v, ctx->d_counters + 9, sizeof v, hipMemcpyDeviceToHost));
    PPD_HIP(ctx, hipMemset(ctx->d_counters + 9, 0, sizeof v));
    // calls of ppd_mixed_attention_static raise their flags in the static array of this GPU
    unsigned char* sp = nullptr;
    PPD_HIP(ctx, static_scratch_address(ctx->device, &sp));
    PPD_HIP(ctx, hipMemcpy(&vs, reinterpret_cast<uint32_t*>(sp) + 9, sizeof vs, hipMemcpyDeviceToHost));
    if (vs) PPD_HIP(ctx, hipMemset(reinterpret_cast<uint32_t*>(sp) + 9, 0, sizeof vs));
    *flags = v | vs;
    return PPD_OK;
}

}  // extern "C"
