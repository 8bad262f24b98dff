// Host side of libppd: context, argument checks, plan upload and kernel launches behind the C ABI.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
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
    uint32_t* d_counters = nullptr;  // kCounterWords words: error flags, finished count, timing sums; queue cursors
    Staging staging[kStagingSlots];
    int next_slot = 0;
    // the plan on the device stays valid while L, n and the planner options do not change (the layers of one
    // engine step call with the same lengths): such calls skip planning and upload
    std::vector<int32_t> plan_L, plan_n;
    ppd::PlanOptions plan_opts;
    bool plan_on_device = false;
    // optional timing of the mixed kernel alone (option "timing"): one pair of events per launch since the option
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

}  // namespace

extern "C" {

const char* ppd_version(void) { return "0.1"; }

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
    if (device < 0 || device >= count) return fail(nullptr, PPD_ERR_RANGE, "device index out of range");
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
    for (auto& s : ctx->staging) {
        if (s.host) (void)hipHostFree(s.host);
        if (s.done) (void)hipEventDestroy(s.done);
    }
    for (auto& p : ctx->ev_pairs) {
        if (p.first) (void)hipEventDestroy(p.first);
        if (p.second) (void)hipEventDestroy(p.second);
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
    } else if (k == "timing") {
        ctx->timing = value != 0;
        ctx->ev_used = 0;
    } else {
        return fail(ctx, PPD_ERR_RANGE, "unknown option " + k);
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
    int rc = ppd::launch_kv_append(static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                                   static_cast<uint16_t*>(kv_pages), slot_mapping, T, ctx->shape.num_kv_heads,
                                   ctx->shape.head_dim, ctx->shape.num_pages, 1, 0, ctx->d_counters + 9, stream);
    if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch kv_append");
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
        (num_layers > 1 && layer_stride_elems % 8 != 0))
        return fail(ctx, PPD_ERR_RANGE,
                    "k / v / kv_pages must be 16-byte aligned (layer_stride_elems a multiple of 8), slot_mapping 8-byte aligned");
    PPD_HIP(ctx, hipSetDevice(ctx->device));
    int rc = ppd::launch_kv_append(static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                                   static_cast<uint16_t*>(kv_pages), slot_mapping, T, ctx->shape.num_kv_heads,
                                   ctx->shape.head_dim, ctx->shape.num_pages, num_layers, layer_stride_elems,
                                   ctx->d_counters + 9, stream);
    if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch kv_land");
    return PPD_OK;
}

double ppd_transfer_delay_s(int64_t n_tokens, int64_t kv_bytes_per_token, double beta_target_bytes_per_s,
                            double t_fast_s) {
    if (n_tokens < 0 || kv_bytes_per_token < 0 || !(beta_target_bytes_per_s > 0.0)) return -1.0;
    const double d = (double)n_tokens * (double)kv_bytes_per_token / beta_target_bytes_per_s - t_fast_s;
    return d > 0.0 ? d : 0.0;
}

ppd_status ppd_mixed_attention(ppd_ctx* ctx, const void* q, const void* kv_pages, const int32_t* page_tables,
                               int32_t max_pages, const int32_t* L, const int32_t* n, int32_t B, float scale,
                               void* out, void* stream) {
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
    const char* msg = "";
    ppd_status st = PPD_OK;
    const bool same_opts = std::memcmp(&ctx->plan_opts, &ctx->opts, sizeof(ppd::PlanOptions)) == 0;
    const bool reuse = ctx->plan_on_device && same_opts && (int32_t)ctx->plan_L.size() == B &&
                       std::memcmp(ctx->plan_L.data(), L, sizeof(int32_t) * B) == 0 &&
                       std::memcmp(ctx->plan_n.data(), n, sizeof(int32_t) * B) == 0;
    const auto t_plan0 = std::chrono::steady_clock::now();
    if (!reuse) {
        ctx->plan_on_device = false;
        st = ppd::build_plan(ctx->shape, L, n, B, ctx->opts, &ctx->plan, &msg);
        if (st != PPD_OK) return fail(ctx, st, msg);
    }
    for (int i = 0; i < B; ++i) {
        const int64_t need = ((int64_t)L[i] + n[i] + ppd::kPage - 1) / ppd::kPage;
        if (need > max_pages)
            return fail(ctx, PPD_ERR_PAGETABLE, "sequence " + std::to_string(i) + " needs " + std::to_string(need) +
                                                    " pages, max_pages is " + std::to_string(max_pages));
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
    PPD_HIP(ctx, hipSetDevice(ctx->device));

    const ppd::Plan& plan = ctx->plan;
    const size_t items_bytes = plan.items.size() * sizeof(ppd_work_item);
    const size_t groups_bytes = plan.groups.size() * sizeof(ppd::MergeGroup);
    const size_t units_bytes = plan.units.size() * sizeof(ppd::MergeUnit);
    const size_t total = items_bytes + groups_bytes + units_bytes;
    if (!reuse) {
        // upload: [items][groups][units] through one pinned staging slot
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
        std::memcpy(sg.host, plan.items.data(), items_bytes);
        if (groups_bytes) {
            std::memcpy(static_cast<char*>(sg.host) + items_bytes, plan.groups.data(), groups_bytes);
            std::memcpy(static_cast<char*>(sg.host) + items_bytes + groups_bytes, plan.units.data(), units_bytes);
        }
        PPD_HIP(ctx, hipMemcpyAsync(ctx->d_items, sg.host, total, hipMemcpyHostToDevice, hs));
        PPD_HIP(ctx, hipEventRecord(sg.done, hs));
        sg.in_flight = true;
        ctx->plan_L.assign(L, L + B);
        ctx->plan_n.assign(n, n + B);
        ctx->plan_opts = ctx->opts;
        ctx->plan_on_device = true;
        ctx->plan.stats.plan_host_us = (int32_t)std::chrono::duration_cast<std::chrono::microseconds>(
                                           std::chrono::steady_clock::now() - t_plan0).count();
    }

    const int G = ctx->shape.num_q_heads / ctx->shape.num_kv_heads;
    // Masked scores are -inf and enter the exponent as s*c: keep c strictly positive so that scale = 0 gives
    // 2^(-inf) = 0 for masked keys and 2^(~0) = 1 for visible ones (identical to the exact result in fp32).
    float scale_log2e = scale * 1.4426950408889634f;
    if (scale_log2e < 1e-30f) scale_log2e = 1e-30f;
    ppd::KParams kp;
    kp.q = static_cast<const uint16_t*>(q);
    kp.out = static_cast<uint16_t*>(out);
    kp.pool = static_cast<const uint16_t*>(kv_pages);
    kp.page_tables = page_tables;
    kp.items = static_cast<const ppd_work_item*>(ctx->d_items);
    kp.partials = ctx->d_partials;
    kp.counters = ctx->d_counters;
    kp.num_pages = ctx->shape.num_pages;
    kp.page_stride = 2LL * ctx->shape.num_kv_heads * ppd::kPage * ctx->shape.head_dim;
    kp.n_items = (int32_t)plan.items.size();
    std::memcpy(kp.queue_begin, plan.queue_begin, sizeof kp.queue_begin);
    kp.pref_mode = ctx->opts.pref_mode;
    kp.narrow_cus = plan.narrow_cus;
    kp.max_pages = max_pages;
    kp.Hq = ctx->shape.num_q_heads;
    kp.Hkv = ctx->shape.num_kv_heads;
    kp.G = G;
    kp.invG = 65536 / G + 1;
    kp.scale_log2e = scale_log2e;
    const bool timed = ctx->timing && ctx->ev_used < kMaxTimedLaunches;
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
    int rc = ppd::launch_mixed(kp, ctx->shape.head_dim, plan.stats.grid, stream);
    if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch mixed attention");
    if (timed) {
        PPD_HIP(ctx, hipEventRecord(ctx->ev_pairs[ctx->ev_used].second, hs));
        ctx->ev_used += 1;
    }
    if (!plan.groups.empty()) {
        ppd::MergeParams mp;
        mp.groups = reinterpret_cast<const ppd::MergeGroup*>(static_cast<const char*>(ctx->d_items) + items_bytes);
        mp.partials = ctx->d_partials;
        mp.out = static_cast<uint16_t*>(out);
        mp.n_groups = (int32_t)plan.groups.size();
        mp.units = reinterpret_cast<const ppd::MergeUnit*>(static_cast<const char*>(ctx->d_items) + items_bytes +
                                                          groups_bytes);
        mp.n_units = (int32_t)plan.units.size();
        mp.Hq = kp.Hq;
        mp.G = G;
        mp.invG = kp.invG;
        mp.D = ctx->shape.head_dim;
        mp.scale_log2e = scale_log2e;
        rc = ppd::launch_merge(mp, stream);
        if (rc != 0) return hip_fail(ctx, (hipError_t)rc, "launch merge");
    }
    return PPD_OK;
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

ppd_status ppd_debug_counters(ppd_ctx* ctx, void* stream, uint32_t* out64, int32_t clear) {
    if (!ctx || !out64) return fail(ctx, PPD_ERR_NULL, "ctx / out64 is NULL");
    hipStream_t hs = static_cast<hipStream_t>(stream);
    PPD_HIP(ctx, hipSetDevice(ctx->device));
    PPD_HIP(ctx, hipStreamSynchronize(hs));
    PPD_HIP(ctx, hipMemcpy(out64, ctx->d_counters, 256, hipMemcpyDeviceToHost));
    if (clear) PPD_HIP(ctx, hipMemset(ctx->d_counters + 16, 0, 192));
    return PPD_OK;
}

ppd_status ppd_device_error_flags(ppd_ctx* ctx, void* stream, uint32_t* flags) {
    if (!ctx || !flags) return fail(ctx, PPD_ERR_NULL, "ctx / flags is NULL");
    hipStream_t hs = static_cast<hipStream_t>(stream);
    PPD_HIP(ctx, hipSetDevice(ctx->device));
    PPD_HIP(ctx, hipStreamSynchronize(hs));
    uint32_t v = 0;
    PPD_HIP(ctx, hipMemcpy(&v, ctx->d_counters + 9, sizeof v, hipMemcpyDeviceToHost));
    PPD_HIP(ctx, hipMemset(ctx->d_counters + 9, 0, sizeof v));
    *flags = v;
    return PPD_OK;
}

}  // extern "C"
