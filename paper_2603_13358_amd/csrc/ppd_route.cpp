// Host-only arithmetic of the library: the KV-transfer delay model and the PPD routing decision: the score of local append-prefill versus the prefill-node path, the offline
// table of its sign over a discretised workload grid, and the per-request lookup (paper section 3, the score
// equation; section 5, algorithm "PPD Dynamic Routing"; appendix "Decision-Engine Discretization").
#include <cmath>
#include <cstring>

#include "../../include/ppd.h"

namespace {

// benchmark QPS levels of the offline phase (section 4.2, experimental setup)
const double kQpsLevels[PPD_ROUTE_QPS_LEVELS] = {0.5, 1, 2, 4, 6, 8, 10, 12, 16, 20};

int context_class(int64_t n_ctx) {  // small <= 512 < large <= 4096 < huge
    return n_ctx <= 512 ? 0 : (n_ctx <= 4096 ? 1 : 2);
}

int nearest_qps(double qps) {
    int best = 0;
    for (int i = 1; i < PPD_ROUTE_QPS_LEVELS; ++i)
        if (std::fabs(kQpsLevels[i] - qps) < std::fabs(kQpsLevels[best] - qps)) best = i;
    return best;
}

// The nine workload types are input/output token ratios; a request goes to the type whose ratio is nearest on
// a logarithmic scale (ratios span 1/16 .. 32, a linear distance would fold all decode-heavy types together).
int nearest_ratio(const double* centers, double ratio) {
    int best = 0;
    double bd = INFINITY;
    for (int i = 0; i < PPD_ROUTE_RATIO_CLASSES; ++i) {
        const double d = std::fabs(std::log(ratio) - std::log(centers[i]));
        if (d < bd) { bd = d; best = i; }
    }
    return best;
}

}  // namespace

extern "C" {

// Injected-delay equation of the appendix "Bandwidth Simulation" (host arithmetic).
double ppd_transfer_delay_s(int64_t n_tokens, int64_t kv_bytes_per_token, double beta_target_bytes_per_s,
                            double t_fast_s) {
    if (n_tokens < 0 || kv_bytes_per_token < 0 || !(beta_target_bytes_per_s > 0.0)) return -1.0;
    const double d = (double)n_tokens * (double)kv_bytes_per_token / beta_target_bytes_per_s - t_fast_s;
    return d > 0.0 ? d : 0.0;
}

double ppd_route_score(double w_ttft, double w_tpot, double delta_ttft, double delta_tpot) {
    return w_ttft * delta_ttft - w_tpot * delta_tpot;
}

ppd_status ppd_route_table_build(const double* delta_ttft, const double* delta_tpot, double w_ttft, double w_tpot,
                                 uint8_t* x_table) {
    if (!delta_ttft || !delta_tpot || !x_table) return PPD_ERR_NULL;
    if (!(w_ttft >= 0.0) || !(w_tpot >= 0.0)) return PPD_ERR_RANGE;
    for (int i = 0; i < PPD_ROUTE_CELLS; ++i)
        x_table[i] = ppd_route_score(w_ttft, w_tpot, delta_ttft[i], delta_tpot[i]) > 0.0 ? 1 : 0;
    return PPD_OK;
}

int32_t ppd_route_cell(const double* ratio_centers, int64_t n_in, int64_t n_out, int64_t n_ctx, double qps) {
    if (!ratio_centers || n_in < 1 || n_out < 1 || n_ctx < 0 || !(qps > 0.0)) return -1;
    for (int i = 0; i < PPD_ROUTE_RATIO_CLASSES; ++i)
        if (!(ratio_centers[i] > 0.0)) return -1;
    const int c = context_class(n_ctx);
    const int r = nearest_ratio(ratio_centers, (double)n_in / (double)n_out);
    const int q = nearest_qps(qps);
    return (c * PPD_ROUTE_RATIO_CLASSES + r) * PPD_ROUTE_QPS_LEVELS + q;
}

int32_t ppd_route_decide(const uint8_t* x_table, const double* ratio_centers, int32_t turn, int64_t n_in,
                         int64_t n_out, int64_t n_ctx, double qps) {
    if (!x_table || turn < 1) return -1;
    if (turn == 1) return 0;  // no cached KV yet: the prefill-node path
    const int32_t cell = ppd_route_cell(ratio_centers, n_in, n_out, n_ctx, qps);
    if (cell < 0) return -1;
    return x_table[cell] ? 1 : 0;
}

ppd_status ppd_route_decide_batch(const uint8_t* x_table, const double* ratio_centers, int64_t count,
                                  const int32_t* turn, const int64_t* n_in, const int64_t* n_out, const int64_t* n_ctx,
                                  const double* qps, int8_t* x_out) {
    if (count < 0) return PPD_ERR_RANGE;
    if (count == 0) return PPD_OK;
    if (!x_table || !ratio_centers || !turn || !n_in || !n_out || !n_ctx || !qps || !x_out) return PPD_ERR_NULL;
    for (int64_t i = 0; i < count; ++i)
        x_out[i] = (int8_t)ppd_route_decide(x_table, ratio_centers, turn[i], n_in[i], n_out[i], n_ctx[i], qps[i]);
    return PPD_OK;
}

}  // extern "C"
