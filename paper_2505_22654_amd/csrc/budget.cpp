// Host-side budget arithmetic of the C ABI: stage budgets from retention rates and the
// theoretical FLOPs count (Sec. 5.1 "Implementation Details", Eq. 6).  No GPU code here.
#include <cmath>
#include <cstdint>

#include "../../include/vscan.h"

namespace {

bool rate_ok(double r) { return std::isfinite(r) && r >= 0.0 && r <= 1.0; }

bool layers_ok(int32_t n_layers, int32_t prune_layer) {
    return n_layers > 0 && prune_layer >= 0 && prune_layer <= n_layers;
}

int32_t nearest(double v) { return (int32_t)std::floor(v + 0.5); }

}  // namespace

extern "C" int vscan_budget(int32_t n_visual, int32_t n_layers, int32_t prune_layer, double r1,
                            double r2, int32_t *keep_encoder, int32_t *keep_llm,
                            double *avg_tokens) {
    if (n_visual < 0 || !layers_ok(n_layers, prune_layer)) return VSCAN_ERR_SHAPE;
    if (!rate_ok(r1) || !rate_ok(r2)) return VSCAN_ERR_BUDGET;
    const int32_t n1 = nearest(r1 * (double)n_visual);
    const int32_t n2 = nearest(r2 * (double)n1);
    if (keep_encoder) *keep_encoder = n1;
    if (keep_llm) *keep_llm = n2;
    if (avg_tokens)
        *avg_tokens = ((double)prune_layer * n1 + (double)(n_layers - prune_layer) * n2) /
                      (double)n_layers;
    return VSCAN_OK;
}

extern "C" int vscan_budget_solve_r1(int32_t n_layers, int32_t prune_layer, double avg_rate,
                                     double r2, double *r1) {
    if (!r1) return VSCAN_ERR_NULL;
    if (!layers_ok(n_layers, prune_layer)) return VSCAN_ERR_SHAPE;
    if (!rate_ok(avg_rate) || !rate_ok(r2)) return VSCAN_ERR_BUDGET;
    const double denom = (double)prune_layer + (double)(n_layers - prune_layer) * r2;
    if (!(denom > 0.0)) return VSCAN_ERR_BUDGET;
    const double r = avg_rate * (double)n_layers / denom;
    if (r > 1.0) return VSCAN_ERR_BUDGET;
    *r1 = r;
    return VSCAN_OK;
}

extern "C" int vscan_flops(const int32_t *n_per_layer, int32_t n_layers, int64_t d, int64_t m,
                           double *flops) {
    if (!n_per_layer || !flops) return VSCAN_ERR_NULL;
    if (n_layers <= 0 || d <= 0 || m <= 0) return VSCAN_ERR_SHAPE;
    double total = 0.0;
    const double dd = (double)d, mm = (double)m;
    for (int32_t l = 0; l < n_layers; ++l) {
        if (n_per_layer[l] < 0) return VSCAN_ERR_SHAPE;
        const double n = (double)n_per_layer[l];
        total += 4.0 * n * dd * dd + 2.0 * n * n * dd + 3.0 * n * dd * mm;
    }
    *flops = total;
    return VSCAN_OK;
}
