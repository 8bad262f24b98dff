// Stand-alone probe: how fast can MI355X stream reads when nothing is computed?  Two access patterns, both with
// eight waves per compute unit and a fixed number of 16-byte loads per lane in flight:
//   stream: every workgroup reads contiguous 128 KiB blocks of one large buffer;
//   paged : the decode path's pattern -- a wave reads, per step, the 4 KiB K block and the 4 KiB V block (32 KiB
//           apart) of one (page, KV head) of a 64 KiB page, pages visited in random order (a paged KV cache
//           with 8 KV heads and head_dim 128).
// Prints one JSON line per pattern.  The paged figure is the practical ceiling of the narrow (decode) tiles of
// the mixed kernel: they issue exactly these loads.  Not part of the library; bench.py --read-probe runs it.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CHECK(call)                                                                  \
    do {                                                                             \
        hipError_t e_ = (call);                                                      \
        if (e_ != hipSuccess) {                                                      \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));        \
            exit(1);                                                                 \
        }                                                                            \
    } while (0)

constexpr int kThreads = 512;
constexpr int kInFlight = 8;  // 16-byte loads per lane issued before the first is used

template <bool NT>
__device__ __forceinline__ u32x4 load16(const u32x4* p) {
    return NT ? __builtin_nontemporal_load(p) : *p;
}

template <bool NT>
__global__ __launch_bounds__(kThreads) void stream_read(const u32x4* __restrict__ p, size_t nblocks, uint32_t* sink) {
    uint32_t acc = 0;
    for (size_t b = blockIdx.x; b < nblocks; b += gridDim.x) {
        const u32x4* q = p + b * (kThreads * kInFlight) + threadIdx.x;
        u32x4 v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) v[u] = load16<NT>(q + u * kThreads);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) acc ^= v[u][0] ^ v[u][3];
    }
    if (acc == 0x12345678u) sink[0] = acc;  // keeps the loads alive
}

// wave w (global index) owns steps [w * per_wave, (w + 1) * per_wave) of `pages` and KV head w & 7
template <bool NT>
__global__ __launch_bounds__(kThreads) void paged_read(const char* __restrict__ pool, const int* __restrict__ pages,
                                                       int per_wave, int nwaves, uint32_t* sink) {
    const int lane = threadIdx.x & 63;
    uint32_t acc = 0;
    for (int w = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6); w < nwaves; w += gridDim.x * (kThreads / 64)) {
        const int* list = pages + (size_t)w * per_wave;
        const int head = w & 7;
        for (int s = 0; s < per_wave; ++s) {
            const char* base = pool + (size_t)list[s] * 65536 + head * 4096 + lane * 16;
            u32x4 v[kInFlight];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[j] = load16<NT>(reinterpret_cast<const u32x4*>(base + j * 1024));
                v[4 + j] = load16<NT>(reinterpret_cast<const u32x4*>(base + 32768 + j * 1024));
            }
#pragma unroll
            for (int j = 0; j < kInFlight; ++j) acc ^= v[j][0] ^ v[j][3];
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

template <typename Launch>
static double time_ms(Launch launch, int reps) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    launch();
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i) launch();
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    return ms / reps;
}

int main() {
    const int npages = 131072;  // 8 GiB
    const size_t bytes = (size_t)npages * 65536;
    char* pool = nullptr;
    uint32_t* sink = nullptr;
    CHECK(hipMalloc(&pool, bytes));
    CHECK(hipMalloc(&sink, 4));
    CHECK(hipMemset(pool, 1, bytes));
    const int grid = 256;

    const size_t nblocks = bytes / (kThreads * kInFlight * 16);
    const double ms_stream = time_ms([&] { stream_read<false><<<grid, kThreads>>>((const u32x4*)pool, nblocks, sink); }, 3);
    printf("{\"pattern\": \"stream\", \"bytes\": %zu, \"us\": %.1f, \"GBs\": %.1f}\n", bytes, ms_stream * 1e3,
           bytes / ms_stream / 1e6);
    const double ms_stream_nt = time_ms([&] { stream_read<true><<<grid, kThreads>>>((const u32x4*)pool, nblocks, sink); }, 3);
    printf("{\"pattern\": \"stream, non-temporal loads\", \"bytes\": %zu, \"us\": %.1f, \"GBs\": %.1f}\n", bytes,
           ms_stream_nt * 1e3, bytes / ms_stream_nt / 1e6);

    // every (page, head) once: head h's pages in an order of their own, cut into runs of per_wave steps
    const int per_wave = 256;
    const int nwaves = npages * 8 / per_wave;
    std::vector<int> list((size_t)nwaves * per_wave);
    std::vector<int> perm(npages);
    std::mt19937 rng(1);
    for (int h = 0; h < 8; ++h) {
        for (int i = 0; i < npages; ++i) perm[i] = i;
        std::shuffle(perm.begin(), perm.end(), rng);
        int idx = 0;
        for (int w = h; w < nwaves; w += 8)
            for (int s = 0; s < per_wave; ++s) list[(size_t)w * per_wave + s] = perm[idx++];
    }
    int* dlist = nullptr;
    CHECK(hipMalloc(&dlist, list.size() * sizeof(int)));
    CHECK(hipMemcpy(dlist, list.data(), list.size() * sizeof(int), hipMemcpyHostToDevice));
    const double ms_paged = time_ms([&] { paged_read<false><<<grid, kThreads>>>(pool, dlist, per_wave, nwaves, sink); }, 3);
    printf("{\"pattern\": \"paged\", \"bytes\": %zu, \"us\": %.1f, \"GBs\": %.1f}\n", bytes, ms_paged * 1e3,
           bytes / ms_paged / 1e6);
    const double ms_paged_nt = time_ms([&] { paged_read<true><<<grid, kThreads>>>(pool, dlist, per_wave, nwaves, sink); }, 3);
    printf("{\"pattern\": \"paged, non-temporal loads\", \"bytes\": %zu, \"us\": %.1f, \"GBs\": %.1f}\n", bytes,
           ms_paged_nt * 1e3, bytes / ms_paged_nt / 1e6);
    CHECK(hipFree(dlist));
    CHECK(hipFree(sink));
    CHECK(hipFree(pool));
    return 0;
}
