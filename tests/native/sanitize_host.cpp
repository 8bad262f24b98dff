// Host-only check under AddressSanitizer + UndefinedBehaviorSanitizer (built and run by tests/test_sanitizers.py):
// the planner and the routing functions of the library on random and edge-case inputs, and the oracle's C code on a
// tiny batch.  No GPU code is compiled in; nothing here computes a reference value.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <random>
#include <vector>

#include "../../include/ppd.h"

extern "C" {
int ppd_oracle_kv_append(const uint16_t*, const uint16_t*, uint16_t*, const int64_t*, int64_t, int, int, int, int64_t);
int ppd_oracle_mixed_attention(const uint16_t*, const uint16_t*, const int32_t*, int, const int32_t*, const int32_t*, int, int,
                               int, int, int, int64_t, float, const uint8_t*, float*);
}

static int plan_fuzz() {
    std::mt19937_64 rng(7);
    long tiles = 0;
    for (int trial = 0; trial < 150; ++trial) {
        ppd_shape s;
        const int hk[] = {1, 2, 4, 8, 16};
        s.num_kv_heads = hk[rng() % 5];
        const int G = 1 + (int)(rng() % 8);
        s.num_q_heads = G * s.num_kv_heads;
        s.head_dim = (rng() & 1) ? 64 : 128;
        s.page_size = 16;
        s.num_pages = 1 << 24;
        const int Bs[] = {0, 1, 2, 5, 30, 100, 300};
        const int B = Bs[rng() % 7];
        const int Lmax[] = {100, 5000, 70000, 1000000};
        const int lm = Lmax[rng() % 4];
        const int nmax[] = {2, 70, 700, 3000, 20000};
        const int nm = nmax[rng() % 5];
        std::vector<int32_t> L(B), n(B);
        for (int i = 0; i < B; ++i) {
            const int k = (int)(rng() % 4);
            L[i] = k == 3 ? 0 : (int)(rng() % lm);
            n[i] = k == 0 ? 1 : 1 + (int)(rng() % nm);
        }
        const int nc[] = {0, 0, 64, 1024, 8192}, mc[] = {0, 0, 64, 512, 32768}, gr[] = {0, 0, 1, 7, 300};
        ppd_plan_stats st;
        const int o_nc = nc[rng() % 5], o_mc = mc[rng() % 5], o_gr = gr[rng() % 5], o_fk = (rng() % 5 == 0) ? 1 : -1;
        ppd_status rc = ppd_plan_build(&s, L.data(), n.data(), B, o_nc, o_mc, o_gr, o_fk, 256, nullptr, 0, &st);
        if (rc == PPD_ERR_RANGE) continue;  // more than 2^22 tiles: refused, as documented
        if (rc != PPD_OK) { std::printf("plan: rc %d at trial %d\n", (int)rc, trial); return 1; }
        if (st.n_items < 50000) {
            std::vector<ppd_work_item> items((size_t)st.n_items + 1);
            const int64_t counted = st.n_items;
            rc = ppd_plan_build(&s, L.data(), n.data(), B, o_nc, o_mc, o_gr, o_fk, 256, items.data(), counted, &st);
            if (rc != PPD_OK || st.n_items != counted) { std::printf("plan: second call rc %d\n", (int)rc); return 2; }
            for (int64_t i = 0; i < st.n_items; ++i)
                if (items[i].kv_begin < 0 || items[i].kv_end > items[i].kv_total || items[i].kv_begin >= items[i].kv_end ||
                    items[i].seq < 0 || items[i].seq >= B) { std::printf("plan: bad item\n"); return 3; }
        }
        tiles += st.n_items;
    }
    // argument errors
    ppd_shape bad = {32, 8, 96, 16, 10};
    ppd_plan_stats st;
    int32_t one = 1, zero = 0, neg = -1;
    if (ppd_plan_build(&bad, &one, &one, 1, 0, 0, 0, -1, 256, nullptr, 0, &st) != PPD_ERR_SHAPE) return 4;
    ppd_shape ok = {32, 8, 128, 16, 10};
    if (ppd_plan_build(&ok, &neg, &one, 1, 0, 0, 0, -1, 256, nullptr, 0, &st) != PPD_ERR_RANGE) return 5;
    if (ppd_plan_build(&ok, &one, &zero, 1, 0, 0, 0, -1, 256, nullptr, 0, &st) != PPD_ERR_RANGE) return 6;
    if (ppd_plan_build(nullptr, &one, &one, 1, 0, 0, 0, -1, 256, nullptr, 0, &st) != PPD_ERR_NULL) return 7;
    std::printf("planner ok, %ld tiles\n", tiles);
    return 0;
}

static int route_fuzz() {
    std::mt19937_64 rng(11);
    std::uniform_real_distribution<double> u(-1.0, 1.0);
    double dt[PPD_ROUTE_CELLS], dp[PPD_ROUTE_CELLS];
    uint8_t table[PPD_ROUTE_CELLS];
    for (int i = 0; i < PPD_ROUTE_CELLS; ++i) { dt[i] = u(rng); dp[i] = u(rng); }
    if (ppd_route_table_build(dt, dp, 1.0, 2.0, table) != PPD_OK) return 1;
    if (ppd_route_table_build(dt, dp, -1.0, 2.0, table) != PPD_ERR_RANGE) return 2;
    if (ppd_route_table_build(dt, dp, NAN, 2.0, table) != PPD_ERR_RANGE) return 3;
    const double centers[9] = {0.0625, 0.125, 0.25, 0.5, 1, 2, 8, 16, 32};
    const int count = 20000;
    std::vector<int32_t> turn(count);
    std::vector<int64_t> a(count), b(count), c(count);
    std::vector<double> q(count);
    std::vector<int8_t> x(count);
    for (int i = 0; i < count; ++i) {
        turn[i] = (int32_t)(rng() % 7) - 1;                        // -1 and 0 are invalid
        a[i] = (int64_t)(rng() % 5000) - 3;                        // <= 0 is invalid
        b[i] = (int64_t)(rng() % 5000) - 3;
        c[i] = (int64_t)(rng() % (1ll << 40)) - 5;
        q[i] = (rng() % 50 == 0) ? NAN : u(rng) * 40.0;            // NaN, negative and 0 are invalid
    }
    if (ppd_route_decide_batch(table, centers, count, turn.data(), a.data(), b.data(), c.data(), q.data(), x.data()) != PPD_OK) return 4;
    for (int i = 0; i < count; ++i) {
        const bool valid_turn = turn[i] >= 1;
        const bool valid = valid_turn && (turn[i] == 1 || (a[i] >= 1 && b[i] >= 1 && c[i] >= 0 && q[i] > 0.0));
        if ((x[i] < 0) == valid) { std::printf("route: validity mismatch at %d\n", i); return 5; }
        const int32_t cell = ppd_route_cell(centers, a[i], b[i], c[i], q[i]);
        if (cell >= PPD_ROUTE_CELLS) return 6;
    }
    if (ppd_route_decide_batch(table, centers, count, nullptr, a.data(), b.data(), c.data(), q.data(), x.data()) != PPD_ERR_NULL) return 7;
    if (ppd_transfer_delay_s(-1, 10, 1e9, 0) != -1.0 || ppd_transfer_delay_s(5115, 131072, 25e9, 4.5e-3) <= 0) return 8;
    std::printf("routing ok\n");
    return 0;
}

static int oracle_tiny() {
    const int Hq = 4, Hkv = 2, D = 64, P = 16, B = 2;
    const int64_t num_pages = 5;
    const int32_t L[B] = {17, 0}, n[B] = {3, 20};
    const int T = 23, tok = 17 + 3 + 20;
    std::vector<uint16_t> k((size_t)tok * Hkv * D, 0x3F80), v((size_t)tok * Hkv * D, 0x4000), q((size_t)T * Hq * D, 0x3F00);
    std::vector<uint16_t> pool((size_t)num_pages * 2 * Hkv * P * D, 0x7FC1);
    const int32_t pt[B][2] = {{3, 1}, {4, 0}};
    std::vector<int64_t> slots;
    for (int i = 0; i < B; ++i)
        for (int t = 0; t < L[i] + n[i]; ++t) slots.push_back((int64_t)pt[i][t / P] * P + t % P);
    slots.push_back(-1);                                           // a skipped token
    k.resize(k.size() + (size_t)Hkv * D, 0);
    v.resize(v.size() + (size_t)Hkv * D, 0);
    if (ppd_oracle_kv_append(k.data(), v.data(), pool.data(), slots.data(), (int64_t)slots.size(), Hkv, D, P, num_pages) != 0) return 1;
    std::vector<float> out((size_t)T * Hq * D, 0.f);
    if (ppd_oracle_mixed_attention(q.data(), pool.data(), &pt[0][0], 2, L, n, B, Hq, Hkv, D, P, num_pages, 0.125f, nullptr,
                                   out.data()) != 0) return 2;
    for (float o : out)
        if (std::fabs(o - 2.0f) > 1e-6f) { std::printf("oracle: all V rows are 2.0, got %g\n", o); return 3; }
    int64_t far = num_pages * P;                                   // one slot past the pool: must be refused, not written
    if (ppd_oracle_kv_append(k.data(), v.data(), pool.data(), &far, 1, Hkv, D, P, num_pages) == 0) return 4;
    std::printf("oracle ok\n");
    return 0;
}

int main() {
    int rc = plan_fuzz();
    if (rc) return 10 + rc;
    rc = route_fuzz();
    if (rc) return 30 + rc;
    rc = oracle_tiny();
    if (rc) return 50 + rc;
    return 0;
}
