/*
 * CPU oracle for the mixed append-prefill + decode paged-attention step and the paged KV append.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and the cpu_baseline leg
 * of the benchmark may build, load or call it.  It shares no code with the HIP library: the page-pool
 * index functions below are written from the layout sentence alone.
 *
 * What it computes (paper section 4.1, paragraph "Full Prefill vs. Append Prefill", with the renaming
 * L = cached tokens (paper: n), n = new tokens (paper: m)):  each of the n new tokens of a sequence
 * attends over the L cached keys and, causally, over the new tokens up to and including itself, so new
 * row j sees keys 0 .. L+j.  Decode is n = 1 (section 2.1); full prefill is L = 0.  The method is exact:
 * cached KV is reused with no recomputation, so the result has the plain softmax-attention definition and
 * this file is that definition written out, in double precision, with no blocking, fusion or reordering.
 *
 * Declared page-pool layout (bf16 elements, P tokens per page, D a multiple of 8, P a multiple of 8):
 *   page stride           S = 2 * Hkv * P * D
 *   K(page,h,tok,d)   at  page*S +             h*P*D + (d/8)*(P*8) + tok*8 + d%8
 *   V(page,h,tok,d)   at  page*S + Hkv*P*D  +  h*P*D + (tok/8)*(D*8) + d*8 + tok%8
 * i.e. inside a (page, head) block K keeps 8 consecutive d of one token together and is token-minor over
 * those 16-byte granules; V keeps 8 consecutive tokens of one d together.
 *
 * FP8 pages (an extension beyond the paper, which keeps KV in 16-bit precision; nothing in the method changes):
 * the same two layouts with one-byte elements holding OCP FP8 E4M3 codes (1 sign, 4 exponent bits of bias 7, 3
 * mantissa bits; no infinities; S.1111.111 is NaN; largest finite value 448).  The append stores
 * code = e4m3(x * (1 / scale)) -- product and reciprocal in binary32, rounded to the nearest code, ties to the
 * even code, magnitudes beyond 448 saturating to 448 -- with one scale for K and one for V; attention reads
 * K = value(code) * k_scale, V = value(code) * v_scale and is the definition above on those values.
 *
 * Pins (tests/test_oracle_*.py): dense brute force from the un-paged token arrays, recompute-prefill
 * equivalence, n=1 == decode, page relabelling, chunking, closed forms, GQA replication, a library
 * softmax-attention routine on a contiguous case, sentinel check of the append; for the FP8 codes: the format's
 * landmark values, round trips of all codes, a library float8 conversion, and attention on a 16-bit pool that
 * holds the decoded values.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_to_double(uint16_t bits) {
    uint32_t u = ((uint32_t)bits) << 16; /* bf16 is the top half of an IEEE binary32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static int64_t k_index(int64_t page, int h, int tok, int d, int Hkv, int D, int P) {
    int64_t S = 2LL * Hkv * P * D;
    return page * S + (int64_t)h * P * D + (int64_t)(d / 8) * (P * 8) + (int64_t)tok * 8 + d % 8;
}

static int64_t v_index(int64_t page, int h, int tok, int d, int Hkv, int D, int P) {
    int64_t S = 2LL * Hkv * P * D;
    return page * S + (int64_t)Hkv * P * D + (int64_t)h * P * D + (int64_t)(tok / 8) * (D * 8) + (int64_t)d * 8 +
           tok % 8;
}

/* Paged KV append: token t goes to slot = page*P + offset; a negative slot skips the token.
 * Raw 16-bit copies.  Returns 0, or -1 if a slot lies outside the pool (nothing is checked beyond that). */
int ppd_oracle_kv_append(const uint16_t *k, const uint16_t *v, uint16_t *pool, const int64_t *slot_mapping,
                         int64_t T, int Hkv, int D, int P, int64_t num_pages) {
    for (int64_t t = 0; t < T; ++t) {
        int64_t slot = slot_mapping[t];
        if (slot < 0) continue;
        int64_t page = slot / P;
        int tok = (int)(slot % P);
        if (page >= num_pages) return -1;
        for (int h = 0; h < Hkv; ++h)
            for (int d = 0; d < D; ++d) {
                int64_t src = (t * Hkv + h) * D + d;
                pool[k_index(page, h, tok, d, Hkv, D, P)] = k[src];
                pool[v_index(page, h, tok, d, Hkv, D, P)] = v[src];
            }
    }
    return 0;
}

/* KV landing: the same append for every layer of a transferred request (paper section 4.2: KV moves to the
 * decode node on turn 1; appendix "Bandwidth Simulation": the footprint is tokens x bytes-per-token over all
 * layers).  k, v: [layers][T][Hkv][D]; pool of layer l starts layer_stride elements after that of layer l-1. */
int ppd_oracle_kv_land(const uint16_t *k, const uint16_t *v, uint16_t *pools, int64_t layer_stride, int layers,
                       const int64_t *slot_mapping, int64_t T, int Hkv, int D, int P, int64_t num_pages) {
    for (int l = 0; l < layers; ++l) {
        int rc = ppd_oracle_kv_append(k + (int64_t)l * T * Hkv * D, v + (int64_t)l * T * Hkv * D,
                                      pools + (int64_t)l * layer_stride, slot_mapping, T, Hkv, D, P, num_pages);
        if (rc != 0) return rc;
    }
    return 0;
}

/* Injected delay that emulates a slower interconnect (paper appendix "Bandwidth Simulation", the equation for
 * the simulated delay): max(0, B / beta_target - t_fast) with B = n_tokens * s_kv. */
double ppd_oracle_transfer_delay(double n_tokens, double s_kv_bytes, double beta_target, double t_fast) {
    double d = n_tokens * s_kv_bytes / beta_target - t_fast;
    return d > 0.0 ? d : 0.0;
}

/* Value of an E4M3 code: (-1)^s * 2^(e-7) * (1 + m/8) for e > 0, (-1)^s * 2^-6 * (m/8) for e = 0. */
double ppd_oracle_e4m3_value(uint8_t code) {
    int sgn = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double mag;
    if (e == 15 && m == 7) return NAN;
    if (e == 0)
        mag = ldexp((double)m / 8.0, -6);
    else
        mag = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sgn ? -mag : mag;
}

/* Code of a binary32 value: the finite code whose value is nearest, the even code on a tie, 448 for anything
 * larger in magnitude (infinities included), the NaN code for NaN.  Plain search over the 127 magnitudes. */
uint8_t ppd_oracle_e4m3_code(float y) {
    uint8_t sgn = signbit(y) ? 0x80 : 0x00;
    if (isnan(y)) return (uint8_t)(sgn | 0x7F);
    double a = fabs((double)y);
    int best = 0;
    double best_err = INFINITY;
    for (int c = 0; c <= 0x7E; ++c) {
        double err = fabs(ppd_oracle_e4m3_value((uint8_t)c) - a);
        if (err < best_err || (err == best_err && (c & 1) == 0)) {
            best = c;
            best_err = err;
        }
    }
    return (uint8_t)(sgn | best);
}

static uint8_t quantise(uint16_t bf16_bits, float scale) {
    uint32_t u = ((uint32_t)bf16_bits) << 16;
    float x;
    memcpy(&x, &u, sizeof x);
    volatile float inv = 1.0f / scale; /* binary32 reciprocal, then one binary32 product */
    volatile float y = x * inv;
    return ppd_oracle_e4m3_code(y);
}

/* The append into FP8 pages: as ppd_oracle_kv_append, each element stored as its E4M3 code. */
int ppd_oracle_kv_append_fp8(const uint16_t *k, const uint16_t *v, uint8_t *pool, const int64_t *slot_mapping,
                             int64_t T, int Hkv, int D, int P, int64_t num_pages, float k_scale, float v_scale) {
    for (int64_t t = 0; t < T; ++t) {
        int64_t slot = slot_mapping[t];
        if (slot < 0) continue;
        int64_t page = slot / P;
        int tok = (int)(slot % P);
        if (page >= num_pages) return -1;
        for (int h = 0; h < Hkv; ++h)
            for (int d = 0; d < D; ++d) {
                int64_t src = (t * Hkv + h) * D + d;
                pool[k_index(page, h, tok, d, Hkv, D, P)] = quantise(k[src], k_scale);
                pool[v_index(page, h, tok, d, Hkv, D, P)] = quantise(v[src], v_scale);
            }
    }
    return 0;
}

int ppd_oracle_kv_land_fp8(const uint16_t *k, const uint16_t *v, uint8_t *pools, int64_t layer_stride, int layers,
                           const int64_t *slot_mapping, int64_t T, int Hkv, int D, int P, int64_t num_pages,
                           float k_scale, float v_scale) {
    for (int l = 0; l < layers; ++l) {
        int rc = ppd_oracle_kv_append_fp8(k + (int64_t)l * T * Hkv * D, v + (int64_t)l * T * Hkv * D,
                                          pools + (int64_t)l * layer_stride, slot_mapping, T, Hkv, D, P, num_pages,
                                          k_scale, v_scale);
        if (rc != 0) return rc;
    }
    return 0;
}

/* Element `index` of a pool: a bf16 value, or for FP8 pages the code's value times the tensor's scale. */
static double kv_value(const void *pool, int64_t index, int fp8, double scale) {
    if (fp8) return ppd_oracle_e4m3_value(((const uint8_t *)pool)[index]) * scale;
    return bf16_to_double(((const uint16_t *)pool)[index]);
}

/* Mixed-batch attention.  q, out: [T][Hq][D] with the rows of sequence i starting at sum_{j<i} n_j.
 * row_mask (may be NULL): compute only rows with row_mask[r] != 0, leave the others untouched.
 * out is fp32 (rounded once from the double result).  Returns 0, or a negative code for an invalid
 * page-table entry. */
static int attention(const uint16_t *q, const void *pool, int fp8, double k_scale, double v_scale,
                     const int32_t *page_tables, int max_pages, const int32_t *L, const int32_t *n, int B, int Hq,
                     int Hkv, int D, int P, int64_t num_pages, float scale, const uint8_t *row_mask, float *out) {
    int G = Hq / Hkv;
    int64_t T = 0;
    for (int i = 0; i < B; ++i) T += n[i];
    /* flat list of (sequence, row) so that the parallel loop below is a plain loop over output rows */
    int32_t *row_seq = (int32_t *)malloc((size_t)(T > 0 ? T : 1) * sizeof(int32_t));
    int32_t *row_j = (int32_t *)malloc((size_t)(T > 0 ? T : 1) * sizeof(int32_t));
    int64_t r = 0;
    for (int i = 0; i < B; ++i)
        for (int j = 0; j < n[i]; ++j) {
            row_seq[r] = i;
            row_j[r] = j;
            ++r;
        }
    int status = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t row = 0; row < T; ++row)
        for (int h = 0; h < Hq; ++h) {
            if (row_mask && !row_mask[row]) continue;
            int i = row_seq[row];
            int j = row_j[row];
            int g = h / G;             /* KV head shared by this query head */
            int64_t visible = (int64_t)L[i] + j + 1; /* keys 0 .. L+j */
            const uint16_t *qv = q + (row * Hq + h) * D;
            double *s = (double *)malloc((size_t)visible * sizeof(double));
            double m = -INFINITY;
            int bad = 0;
            for (int64_t t = 0; t < visible; ++t) {
                int32_t page = page_tables[(int64_t)i * max_pages + t / P];
                if (page < 0 || page >= num_pages) { bad = 1; break; }
                double dot = 0.0;
                for (int d = 0; d < D; ++d)
                    dot += bf16_to_double(qv[d]) * kv_value(pool, k_index(page, g, (int)(t % P), d, Hkv, D, P), fp8, k_scale);
                s[t] = (double)scale * dot;
                if (s[t] > m) m = s[t];
            }
            if (bad) {
#pragma omp atomic write
                status = -2;
                free(s);
                continue;
            }
            double l = 0.0;
            for (int64_t t = 0; t < visible; ++t) {
                s[t] = exp(s[t] - m);
                l += s[t];
            }
            for (int d = 0; d < D; ++d) {
                double acc = 0.0;
                for (int64_t t = 0; t < visible; ++t) {
                    int32_t page = page_tables[(int64_t)i * max_pages + t / P];
                    acc += s[t] * kv_value(pool, v_index(page, g, (int)(t % P), d, Hkv, D, P), fp8, v_scale);
                }
                out[(row * Hq + h) * D + d] = (float)(acc / l);
            }
            free(s);
        }
    free(row_seq);
    free(row_j);
    return status;
}

int ppd_oracle_mixed_attention(const uint16_t *q, const uint16_t *pool, const int32_t *page_tables,
                               int max_pages, const int32_t *L, const int32_t *n, int B, int Hq, int Hkv, int D,
                               int P, int64_t num_pages, float scale, const uint8_t *row_mask, float *out) {
    return attention(q, pool, 0, 1.0, 1.0, page_tables, max_pages, L, n, B, Hq, Hkv, D, P, num_pages, scale, row_mask,
                     out);
}

/* The same on FP8 pages: K = value(code) * k_scale, V = value(code) * v_scale. */
int ppd_oracle_mixed_attention_fp8(const uint16_t *q, const uint8_t *pool, float k_scale, float v_scale,
                                   const int32_t *page_tables, int max_pages, const int32_t *L, const int32_t *n,
                                   int B, int Hq, int Hkv, int D, int P, int64_t num_pages, float scale,
                                   const uint8_t *row_mask, float *out) {
    return attention(q, pool, 1, (double)k_scale, (double)v_scale, page_tables, max_pages, L, n, B, Hq, Hkv, D, P,
                     num_pages, scale, row_mask, out);
}
