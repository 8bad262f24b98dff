// Host planner of the one-launch mixed step: classifies sequences, splits key ranges, orders tiles.
//
// Per sequence (L cached, n new; paper section 4.1 with L = the paper's n and n = its m): n*G <= 16 query
// columns -> narrow tiles (decode is n = 1), else row blocks of 256/G rows on the MFMA path.  A tile is
// (sequence, KV head, row block, key range); key ranges are split only as far as filling and balancing the
// workgroups needs, and tiles run longest-first from nine queues (one of narrow tiles, eight of row-block tiles,
// one per XCD) so that HBM-bound narrow tiles and MFMA-bound row-block tiles run side by side on the chip.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <unordered_map>

#include "ppd_internal.h"

namespace ppd {

ppd_status validate_shape(const ppd_shape* s, const char** err) {
    static const char* kNull = "shape is NULL";
    static const char* kDim = "head_dim must be 64 or 128";
    static const char* kPageSz = "page_size must be 16";
    static const char* kHeads = "num_q_heads must be G * num_kv_heads with 1 <= G <= 8, num_kv_heads >= 1";
    static const char* kPages = "num_pages must be >= 1 and the pool below 2^40 elements";
    const char* dummy;
    if (!err) err = &dummy;
    if (!s) { *err = kNull; return PPD_ERR_NULL; }
    if (s->head_dim != 64 && s->head_dim != 128) { *err = kDim; return PPD_ERR_SHAPE; }
    if (s->page_size != kPage) { *err = kPageSz; return PPD_ERR_SHAPE; }
    if (s->num_kv_heads < 1 || s->num_q_heads < 1 || s->num_q_heads % s->num_kv_heads != 0) {
        *err = kHeads; return PPD_ERR_SHAPE;
    }
    int G = s->num_q_heads / s->num_kv_heads;
    if (G < 1 || G > 8) { *err = kHeads; return PPD_ERR_SHAPE; }
    if (s->num_kv_heads > 1024) { *err = kHeads; return PPD_ERR_SHAPE; }
    if (s->num_pages < 1 || s->num_pages > (int64_t(1) << 40) / (2LL * s->num_kv_heads * kPage * s->head_dim)) {
        *err = kPages; return PPD_ERR_SHAPE;
    }
    return PPD_OK;
}

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Splits [0, len) into pieces of at most ~chunk tokens with boundaries on multiples of kTileTokens.
static void split_range(int64_t len, int64_t chunk, std::vector<int32_t>* bounds) {
    bounds->clear();
    int64_t nsplit = std::max<int64_t>(1, (len + chunk - 1) / chunk);
    int64_t per = round_up((len + nsplit - 1) / nsplit, kTileTokens);
    for (int64_t b = 0; b < len; b += per) bounds->push_back((int32_t)b);
    bounds->push_back((int32_t)len);
}

// Split size of the MFMA row-block tiles.  Every split costs a partial (fp32 o, m, l per column) that the tile
// writes and a separate merge launch reads back; not splitting leaves few, long tiles that may not fill or balance
// the workgroups.  The choice is made by estimate: for each candidate size the row blocks are cut (all KV heads
// alike), their tiles list-scheduled longest-first, at kTileStartUs + kTileIterUs per 64 keys, onto the
// workgroups that will take MFMA tiles first in the launch; the launch then takes the longer of that schedule and
// of all work spread evenly over all workgroups (narrow tiles included: a compute unit streams ~45 GB/s, HBM
// delivers ~6.5 TB/s to all of them together), plus the cost of the partials.  Candidates run from whole key ranges
// downwards and stop once there are far more tiles than workgroups.  Constants fitted to measured launches
// (append-prefill batches of 2..16 sequences, 256 workgroups): the estimate is within ~8 % of the kernel time and
// ranks the candidates of one batch correctly.
struct RowBlock { int64_t vis_end; int32_t nrows; };

// Compute units (of the 32 of an XCD) whose workgroups take narrow tiles first.  A workgroup of the mixed kernel
// fills a compute unit (8 waves of up to 256 registers), so the two kinds are split by physical unit.  Narrow tiles are bound by the bytes a unit keeps in flight (about 45 GB/s each), MFMA tiles
// by compute (about 2.3 us per 64 keys of a row block): the split is sized so that both kinds finish together;
// whoever finishes first steals from the other anyway.
// A unit streams FP8 pages at about 38 GB/s: its loads are 8 bytes per lane instead of 16 and 8, and a unit's memory
// pipeline moves fewer bytes per second with narrower loads (about 58 GB/s at best, with contiguous 16-byte loads).
static double unit_bytes_per_us(int elem_bytes) { return elem_bytes == 1 ? 38e3 : 45e3; }

static int narrow_units(double narrow_bytes, double mfma_iters, int elem_bytes) {
    if (narrow_bytes == 0) return 0;
    if (mfma_iters == 0) return 32;
    const double narrow_cu_us = narrow_bytes / unit_bytes_per_us(elem_bytes);  // CU-microseconds
    const double mfma_us = mfma_iters * 2.3 / kWgPerCu;
    const int cus = (int)std::lround(32.0 * narrow_cu_us / (narrow_cu_us + mfma_us));
    return std::min(std::max(cus, 2), 20);            // HBM saturates well before all units stream
}

static int64_t choose_mfma_chunk(const std::vector<RowBlock>& blocks, int G, int Hkv, int D, int slots,
                                 double narrow_bytes, int elem_bytes) {
    constexpr double kTileStartUs = 16.0;
    // 1.7 us per 64 keys at D = 128; at D = 64 the two products halve and the softmax stays (measured ~0.65x)
    const double kTileIterUs = 1.7 * (0.3 + 0.7 * D / 128.0);
    constexpr double kMergeLaunchUs = 12.0, kPartialBytesPerUs = 2.5e6;
    constexpr double kHbmBytesPerUs = 6.5e6;
    const double kUnitBytesPerUs = unit_bytes_per_us(elem_bytes);
    static const int64_t kCandidates[] = {32768, 24576, 16384, 12288, 8192, 6144, 4096, 3072, 2048, 1024, 512};
    const double narrow_work = narrow_bytes / kUnitBytesPerUs;  // unit-microseconds
    const double narrow_floor = narrow_bytes / kHbmBytesPerUs;  // however many units stream
    int64_t best_chunk = kCandidates[0];
    double best = -1.0, even_first = -1.0;
    std::vector<double> tiles, load;
    std::vector<int32_t> bounds;
    for (int64_t c : kCandidates) {
        tiles.clear();
        double partial_bytes = 0, mfma_work = 0, iters = 0;
        for (const RowBlock& rb : blocks) {
            split_range(rb.vis_end, c, &bounds);
            const int nsplit = (int)bounds.size() - 1;
            for (int k = 0; k < nsplit; ++k) {
                const double it = (double)((bounds[k + 1] - bounds[k] + kTileTokens - 1) / kTileTokens);
                tiles.push_back(kTileStartUs + kTileIterUs * it);
                mfma_work += tiles.back() * Hkv;
                iters += it * Hkv;
            }
            if (nsplit > 1) partial_bytes += (double)rb.nrows * G * (D + 2) * 4.0 * nsplit * Hkv;
        }
        // the workgroups that take MFMA tiles first, as the launch will split them
        const int S = std::max(1, slots - narrow_units(narrow_bytes, iters, elem_bytes) * slots / 32);
        std::sort(tiles.begin(), tiles.end(), std::greater<double>());
        load.assign((size_t)S, 0.0);  // min-heap of workgroup finish times; the earliest workgroup takes the next tile
        for (double t : tiles)
            for (int h = 0; h < Hkv; ++h) {
                load[0] += t;
                for (size_t at = 0;;) {  // sift the grown root down
                    size_t kid = 2 * at + 1;
                    if (kid >= (size_t)S) break;
                    if (kid + 1 < (size_t)S && load[kid + 1] < load[kid]) ++kid;
                    if (load[at] <= load[kid]) break;
                    std::swap(load[at], load[kid]);
                    at = kid;
                }
            }
        const double makespan = *std::max_element(load.begin(), load.end());
        const double even = std::max((mfma_work + narrow_work) / slots, narrow_floor);
        const double est = std::max(makespan, even) +
                           (partial_bytes > 0 ? kMergeLaunchUs + partial_bytes / kPartialBytesPerUs : 0.0);
        if (best < 0 || est < 0.99 * best) {  // a smaller chunk has to win clearly
            best = est;
            best_chunk = c;
        }
        if ((int64_t)tiles.size() * Hkv > 16LL * S) break;  // plenty of tiles already: smaller pieces only add partials
        // Smaller pieces only add tiles, so `even` never falls below what the first candidate gives, and no later
        // estimate can be below it: once the best estimate is within 1 % of that bound nothing can still win.
        if (even_first < 0) even_first = even;
        if (0.99 * best <= even_first) break;
    }
    return best_chunk;
}

// Split size of the narrow tiles of a launch that has nothing else and fewer (sequence, KV head) pairs than twice the
// workgroups: the few-sequences, long-context corner, where the fixed rule below leaves compute units idle or
// the last round of tiles nearly empty.  Estimate per candidate: tiles longest-first in rounds of `slots`; a round
// takes kStartUs plus its longest tile at what a unit streams (kUnitBytesPerUs, or its share of kHbmBytesPerUs
// when more units stream than HBM can feed); a split range costs a merge launch plus kMergeSplitUs per split
// (the merge walks the splits of a column one after the other).  Constants fitted to 114 measured launches
// (1..16 sequences x 4K..256K context x six split sizes; log-error 11 % rms, the pick within 3 % of the best
// measured size in all 19 batches).
static int64_t choose_narrow_chunk(const std::vector<int64_t>& lengths, int Hkv, int D, int slots, int elem_bytes) {
    constexpr double kStartUs = 7.0, kHbmBytesPerUs = 7.0e6;
    const double kUnitBytesPerUs = elem_bytes == 1 ? 44e3 : 55e3;
    constexpr double kMergeUs = 4.0, kMergeSplitUs = 0.3;
    static const int64_t kCandidates[] = {8192, 6144, 4096, 3072, 2048, 1536, 1024, 768, 512};
    const double bytes_per_key = 2.0 * D * elem_bytes;
    int64_t best_chunk = kCandidates[0];
    double best = -1.0;
    std::vector<int32_t> tiles, bounds;
    for (int64_t c : kCandidates) {
        tiles.clear();
        int max_split = 1;
        for (int64_t len : lengths) {
            split_range(len, c, &bounds);
            const int nsplit = (int)bounds.size() - 1;
            max_split = std::max(max_split, nsplit);
            for (int k = 0; k < nsplit; ++k)
                for (int h = 0; h < Hkv; ++h) tiles.push_back(bounds[k + 1] - bounds[k]);
        }
        if ((int64_t)tiles.size() > 8LL * slots && best >= 0) break;  // more than enough tiles: stop refining
        std::sort(tiles.begin(), tiles.end(), std::greater<int32_t>());
        double est = max_split > 1 ? kMergeUs + kMergeSplitUs * max_split : 0.0;
        for (size_t j = 0; j < tiles.size(); j += (size_t)slots) {
            const double streaming = (double)std::min<size_t>((size_t)slots, tiles.size() - j);
            const double rate = std::min(kUnitBytesPerUs, kHbmBytesPerUs / streaming);
            est += kStartUs + tiles[j] * bytes_per_key / rate;
        }
        if (best < 0 || est < 0.99 * best) {  // a smaller chunk has to win clearly
            best = est;
            best_chunk = c;
        }
    }
    return best_chunk;
}

ppd_status build_plan(const ppd_shape& s, const int32_t* L, const int32_t* n, int32_t B, const PlanOptions& o,
                      Plan* plan, const char** err) {
    static const char* kNull = "L / n is NULL";
    static const char* kNeg = "n_i must be >= 1 and L_i >= 0";
    static const char* kBig = "L_i + n_i and the total row count must stay below 2^30";
    static const char* kTiles = "the batch needs more than 2^22 tiles: too large for one launch";
    static const char* kChunk = "chunk options must be 0 or a positive multiple of 64 (mfma_chunk <= 32768); grid >= 0";
    const char* dummy;
    if (!err) err = &dummy;
    plan->items.clear();
    plan->groups.clear();
    plan->units.clear();
    std::memset(&plan->stats, 0, sizeof plan->stats);
    std::memset(plan->queue_begin, 0, sizeof plan->queue_begin);
    if (B < 0) { *err = kNeg; return PPD_ERR_RANGE; }
    if (B > 0 && (!L || !n)) { *err = kNull; return PPD_ERR_NULL; }
    if (o.narrow_chunk < 0 || o.narrow_chunk % kTileTokens || o.mfma_chunk < 0 || o.mfma_chunk % kTileTokens ||
        o.mfma_chunk > kMaxMfmaChunk || o.grid < 0 || o.num_cus < 1) {
        *err = kChunk; return PPD_ERR_RANGE;
    }
    const int D = s.head_dim, Hq = s.num_q_heads, Hkv = s.num_kv_heads, G = Hq / Hkv;
    const int64_t kv_tok_bytes_head = 2LL * D * (o.kv_elem_bytes == 1 ? 1 : 2);  // K and V of one token of one KV head
    int64_t rows = 0;
    double flops = 0;
    int64_t kv_tokens = 0;
    for (int i = 0; i < B; ++i) {
        if (n[i] < 1 || L[i] < 0) { *err = kNeg; return PPD_ERR_RANGE; }
        if ((int64_t)L[i] + n[i] >= (1 << 30)) { *err = kBig; return PPD_ERR_RANGE; }
        rows += n[i];
        kv_tokens += (int64_t)L[i] + n[i];
        flops += 4.0 * Hq * D * ((double)n[i] * L[i] + (double)n[i] * ((double)n[i] + 1) / 2);
    }
    if (rows >= (1 << 30)) { *err = kBig; return PPD_ERR_RANGE; }

    auto is_narrow = [&](int i) { return o.force_kind != 1 && (int64_t)n[i] * G <= kNarrowCols; };
    const int rows_per_block = kMfmaCols / G;

    double narrow_tokens = 0;          // keys of the narrow tiles, counted once per KV head
    std::vector<int64_t> narrow_lengths;
    std::vector<RowBlock> row_blocks;  // of one KV head
    for (int i = 0; i < B; ++i) {
        if (is_narrow(i)) {
            narrow_tokens += (double)Hkv * (L[i] + n[i]);
            narrow_lengths.push_back((int64_t)L[i] + n[i]);
        } else {
            const int64_t blocks = ((int64_t)n[i] + rows_per_block - 1) / rows_per_block;
            if (((int64_t)row_blocks.size() + blocks) * Hkv > kMaxTiles) { *err = kTiles; return PPD_ERR_RANGE; }
            for (int r0 = 0; r0 < n[i]; r0 += rows_per_block) {
                const int nrows = std::min(rows_per_block, n[i] - r0);
                const int64_t vis_end = (int64_t)L[i] + r0 + nrows;
                row_blocks.push_back(RowBlock{vis_end, nrows});
            }
        }
    }
    if ((int64_t)(row_blocks.size() + narrow_lengths.size()) * Hkv > kMaxTiles) { *err = kTiles; return PPD_ERR_RANGE; }
    const int slots = o.grid > 0 ? o.grid : kWgPerCu * o.num_cus;  // resident workgroups
    // Narrow tiles: every split costs a partial and, above all, a gap in the workgroup's stream of loads (claim,
    // page ids, first loads: ~8 us), so key ranges stay whole unless the batch is too small to occupy the chip:
    // measured over batch sizes 1..512 and contexts 4K..32K, ~100 tiles or more per launch and no tile shorter
    // than 512 keys is within a few percent of the best split everywhere.
    int64_t narrow_chunk = o.narrow_chunk > 0
                               ? o.narrow_chunk
                               : std::min<int64_t>(8192, std::max<int64_t>(512, round_up((int64_t)(narrow_tokens / 96), kTileTokens)));
    if (o.narrow_chunk == 0 && row_blocks.empty() && (int64_t)narrow_lengths.size() * Hkv < 2LL * slots)
        narrow_chunk = choose_narrow_chunk(narrow_lengths, Hkv, D, slots, o.kv_elem_bytes == 1 ? 1 : 2);
    int64_t mfma_chunk = o.mfma_chunk;
    if (mfma_chunk == 0 && !row_blocks.empty())
        mfma_chunk = choose_mfma_chunk(row_blocks, G, Hkv, D, slots, narrow_tokens * kv_tok_bytes_head, o.kv_elem_bytes == 1 ? 1 : 2);
    if (mfma_chunk == 0) mfma_chunk = kMaxMfmaChunk;

    struct Keyed { double cost; ppd_work_item it; };
    std::vector<Keyed> keyed;
    keyed.reserve((row_blocks.size() + narrow_lengths.size()) * (size_t)Hkv);
    std::vector<int32_t> bounds;
    int64_t part_floats = 0;
    int64_t grow = 0;
    int64_t n_narrow = 0, n_mfma = 0, bytes_tiles = 0;
    for (int i = 0; i < B; ++i) {
        const bool narrow = is_narrow(i);
        const int blk = narrow ? n[i] : rows_per_block;
        for (int r0 = 0; r0 < n[i]; r0 += blk) {
            const int nrows = std::min(blk, n[i] - r0);
            const int64_t vis_end = (int64_t)L[i] + r0 + nrows;  // keys 0 .. L + last row of the block
            split_range(vis_end, narrow ? narrow_chunk : mfma_chunk, &bounds);
            const int nsplit = (int)bounds.size() - 1;
            if ((int64_t)keyed.size() + (int64_t)nsplit * Hkv > kMaxTiles) { *err = kTiles; return PPD_ERR_RANGE; }
            const int64_t stride = (int64_t)nrows * G * (D + 2);
            for (int h = 0; h < Hkv; ++h) {
                int group = -1;
                int64_t base = -1;
                if (nsplit > 1) {
                    group = (int)plan->groups.size();
                    base = part_floats;
                    plan->groups.push_back(MergeGroup{(int32_t)(grow + r0), nrows, h, nsplit, base, stride});
                    for (int c0 = 0; c0 < nrows * G; c0 += kMergeCols) plan->units.push_back(MergeUnit{group, c0});
                    part_floats += stride * nsplit;
                }
                for (int sp = 0; sp < nsplit; ++sp) {
                    ppd_work_item it;
                    std::memset(&it, 0, sizeof it);
                    it.kind = narrow ? 0 : 1;
                    it.seq = i;
                    it.kvh = h;
                    it.row0 = r0;
                    it.nrows = nrows;
                    it.grow0 = (int32_t)(grow + r0);
                    it.L = L[i];
                    it.kv_total = L[i] + n[i];
                    it.kv_begin = bounds[sp];
                    it.kv_end = bounds[sp + 1];
                    it.group = group;
                    it.part_off = nsplit > 1 ? base + stride * sp : -1;
                    const int64_t toks = it.kv_end - it.kv_begin;
                    keyed.push_back(Keyed{(narrow ? 1.0 : 2.0) * toks, it});
                    (narrow ? n_narrow : n_mfma) += 1;
                    bytes_tiles += toks * kv_tok_bytes_head;
                }
            }

        }
        grow += n[i];
    }
    // Queues.  Narrow tiles read every key once: one queue, longest first.  MFMA row-block tiles of one
    // (sequence, KV head, key range) read the same K/V: they form a sharing group that is kept together in
    // one of eight per-XCD queues (the workgroups of an XCD share its L2), groups spread over the queues
    // longest-first onto the least loaded queue; inside a queue the tiles of a group stay adjacent so that they
    // run at about the same time.
    std::vector<Keyed> narrow_items;
    struct Share { double cost; std::vector<ppd_work_item> items; };
    std::vector<Share> shares;
    {
        std::unordered_map<uint64_t, size_t> index;
        for (auto& k : keyed) {
            if (k.it.kind == 0) { narrow_items.push_back(k); continue; }
            const uint64_t key = ((uint64_t)k.it.seq * (uint64_t)Hkv + (uint64_t)k.it.kvh) * (1ull << 24) +
                                 (uint64_t)(k.it.kv_begin / kTileTokens);
            auto f = index.find(key);
            if (f == index.end()) {
                index.emplace(key, shares.size());
                shares.push_back(Share{0.0, {}});
                f = index.find(key);
            }
            shares[f->second].cost += k.cost;
            shares[f->second].items.push_back(k.it);
        }
    }
    std::stable_sort(shares.begin(), shares.end(), [](const Share& a, const Share& b) { return a.cost > b.cost; });
    std::vector<size_t> members[kXcds];
    double load[kXcds] = {0};
    for (size_t k = 0; k < shares.size(); ++k) {
        int q = 0;
        for (int x = 1; x < kXcds; ++x)
            if (load[x] < load[q]) q = x;
        load[q] += shares[k].cost;
        members[q].push_back(k);
    }
    // Inside a queue the groups run longest TILE first (a group's tiles run side by side on different workgroups,
    // so it is the length of one tile, not the sum over the group, that decides how late it may start): a single
    // long tile of a short append-prefill must not wait behind groups of many short ones.
    std::vector<ppd_work_item> queues[kXcds];
    for (int q = 0; q < kXcds; ++q) {
        auto longest = [&](size_t k) {
            int32_t m = 0;
            for (auto& it : shares[k].items) m = std::max(m, it.kv_end - it.kv_begin);
            return m;
        };
        std::vector<std::pair<int32_t, size_t>> order;
        for (size_t k : members[q]) order.emplace_back(longest(k), k);
        std::stable_sort(order.begin(), order.end(), [](const std::pair<int32_t, size_t>& a, const std::pair<int32_t, size_t>& b) { return a.first > b.first; });
        for (auto& o2 : order)
            for (auto& it : shares[o2.second].items) {
                it.queue = q;
                queues[q].push_back(it);
            }
    }
    std::stable_sort(narrow_items.begin(), narrow_items.end(), [](const Keyed& a, const Keyed& b) { return a.cost > b.cost; });
    plan->items.reserve(keyed.size());
    for (int q = 0; q < kXcds; ++q) {
        plan->queue_begin[q] = (int32_t)plan->items.size();
        for (auto& it : queues[q]) plan->items.push_back(it);
    }
    // Narrow tiles, longest first.  The short ones at the end of the list form the wave-tile queue when there are
    // enough of them to keep the waves of every workgroup busy (then eight tiles share the fixed cost of one); with
    // fewer, eight waves per tile keep more compute units streaming.
    size_t wave_from = narrow_items.size();
    if (o.wave_tiles != 0 && o.force_kind != 1) {
        size_t first_short = 0;
        while (first_short < narrow_items.size() &&
               narrow_items[first_short].it.kv_end - narrow_items[first_short].it.kv_begin > kWaveTileKeys)
            ++first_short;
        const size_t n_short = narrow_items.size() - first_short;
        // (by the chip's workgroup slots, not by a grid override: that option must stay scheduling only)
        if (n_short > 0 && (o.wave_tiles == 1 || n_short >= (size_t)6 * (size_t)(kWgPerCu * o.num_cus))) wave_from = first_short;
    }
    plan->queue_begin[kNarrowQueue] = (int32_t)plan->items.size();
    for (size_t k = 0; k < narrow_items.size(); ++k) {
        if (k == wave_from) plan->queue_begin[kWaveQueue] = (int32_t)plan->items.size();
        narrow_items[k].it.queue = k < wave_from ? kNarrowQueue : kWaveQueue;
        plan->items.push_back(narrow_items[k].it);
    }
    if (wave_from == narrow_items.size()) plan->queue_begin[kWaveQueue] = (int32_t)plan->items.size();
    plan->queue_begin[kQueues] = (int32_t)plan->items.size();

    // Split of the compute units between the two kinds when both are present (see narrow_units).
    {
        double narrow_bytes = 0, mfma_iters = 0;
        for (auto& k : keyed) {
            const double toks = (double)(k.it.kv_end - k.it.kv_begin);
            if (k.it.kind == 0) narrow_bytes += toks * kv_tok_bytes_head;
            else mfma_iters += std::ceil(toks / kTileTokens);
        }
        plan->narrow_cus = o.narrow_cus >= 0 ? std::min(o.narrow_cus, 32) : narrow_units(narrow_bytes, mfma_iters, o.kv_elem_bytes == 1 ? 1 : 2);
    }

    ppd_plan_stats& st = plan->stats;
    st.n_items = (int64_t)plan->items.size();
    st.n_narrow = n_narrow;
    st.n_mfma = n_mfma;
    st.n_groups = (int64_t)plan->groups.size();
    st.partial_floats = part_floats;
    st.kv_bytes = kv_tokens * kv_tok_bytes_head * Hkv;
    st.kv_bytes_tiles = bytes_tiles;
    st.flops = flops;
    st.narrow_chunk = (int32_t)narrow_chunk;
    st.mfma_chunk = (int32_t)mfma_chunk;
    // a workgroup's eight waves take eight wave tiles at a time
    const int64_t wave_groups = (plan->queue_begin[kQueues] - plan->queue_begin[kWaveQueue] + kWaves - 1) / kWaves;
    st.grid = (int32_t)std::max<int64_t>(1, std::min<int64_t>(slots, plan->queue_begin[kWaveQueue] + wave_groups));
    return PPD_OK;
}

}  // namespace ppd

extern "C" ppd_status ppd_plan_build(const ppd_shape* shape, const int32_t* L, const int32_t* n, int32_t B,
                                     int32_t narrow_chunk, int32_t mfma_chunk, int32_t grid, int32_t force_kind,
                                     int32_t num_cus, ppd_work_item* items, int64_t capacity, ppd_plan_stats* stats) {
    ppd_status st = ppd::validate_shape(shape, nullptr);
    if (st != PPD_OK) return st;
    ppd::PlanOptions o;
    o.narrow_chunk = narrow_chunk;
    o.mfma_chunk = mfma_chunk;
    o.grid = grid;
    o.force_kind = force_kind;
    o.num_cus = num_cus > 0 ? num_cus : 256;
    ppd::Plan plan;
    st = ppd::build_plan(*shape, L, n, B, o, &plan, nullptr);
    if (st != PPD_OK) return st;
    if (items)
        for (int64_t i = 0; i < std::min<int64_t>(capacity, (int64_t)plan.items.size()); ++i) items[i] = plan.items[i];
    if (stats) *stats = plan.stats;
    return PPD_OK;
}
