// Host-only helpers of libbnn: the layer-to-implementation mapping of the paper's Alg. 1 over
// a profiled latency table, and batch-norm folding into (threshold, flip).  No GPU code.
#include <cmath>
#include <limits>

#include "bnn_internal.h"

extern "C" {

bnn_status bnn_map_layers(const double *cpu_us, const double *gpu_us, int n_batch, int n_layers, int n_impl,
                          int *best_batch, int *mapping, double *total_us)
{
    if (!cpu_us || !gpu_us || !best_batch || !mapping) return BNN_ERR_NULL;
    if (n_batch < 1 || n_layers < 1 || n_impl < 1) return BNN_ERR_SHAPE;
    const int64_t count = (int64_t)n_batch * n_layers * n_impl;
    for (int64_t i = 0; i < count; ++i) {
        if (!std::isfinite(cpu_us[i]) || !std::isfinite(gpu_us[i]) || cpu_us[i] < 0 || gpu_us[i] < 0)
            return BNN_ERR_SHAPE;
    }
    double result_time = std::numeric_limits<double>::infinity();
    int proper = 0;
    for (int b = 0; b < n_batch; ++b) {
        double sum_min = 0.0;
        for (int l = 0; l < n_layers; ++l) {
            double min_time = std::numeric_limits<double>::infinity();
            for (int j = 0; j < n_impl; ++j) {
                const int64_t at = ((int64_t)b * n_layers + l) * n_impl + j;
                const double t = cpu_us[at] + gpu_us[at];
                if (t < min_time) min_time = t;
            }
            sum_min += min_time;
        }
        if (sum_min < result_time) { result_time = sum_min; proper = b; }
    }
    for (int l = 0; l < n_layers; ++l) {
        double min_time = std::numeric_limits<double>::infinity();
        int pick = 0;
        for (int j = 0; j < n_impl; ++j) {
            const int64_t at = ((int64_t)proper * n_layers + l) * n_impl + j;
            const double t = cpu_us[at] + gpu_us[at];
            if (t < min_time) { min_time = t; pick = j; }
        }
        mapping[l] = pick;
    }
    *best_batch = proper;
    if (total_us) *total_us = result_time;
    return BNN_OK;
}

bnn_status bnn_fold_batchnorm(const double *gamma, const double *beta, const double *mean, const double *var,
                              double eps, int n, int32_t *thr, uint8_t *flip)
{
    if (!gamma || !beta || !mean || !var || !thr || !flip) return BNN_ERR_NULL;
    if (n < 1 || !std::isfinite(eps)) return BNN_ERR_SHAPE;
    for (int i = 0; i < n; ++i) {
        if (!std::isfinite(gamma[i]) || !std::isfinite(beta[i]) || !std::isfinite(mean[i]) ||
            !std::isfinite(var[i]) || var[i] + eps <= 0.0)
            return BNN_ERR_SHAPE;
    }
    const double lo = (double)std::numeric_limits<int32_t>::min(), hi = (double)std::numeric_limits<int32_t>::max();
    auto clamp32 = [&](double v) { return (int32_t)(v < lo ? lo : (v > hi ? hi : v)); };
    for (int i = 0; i < n; ++i) {
        if (gamma[i] == 0.0) {
            // constant output: +1 iff beta > 0.  x > INT32_MIN holds for every sum this library makes.
            thr[i] = std::numeric_limits<int32_t>::min();
            flip[i] = beta[i] > 0.0 ? 0 : 1;
            continue;
        }
        const double tau = mean[i] - beta[i] * std::sqrt(var[i] + eps) / gamma[i];
        if (gamma[i] > 0.0) {
            thr[i] = clamp32(std::floor(tau));          // x > tau  <=>  x > floor(tau)
            flip[i] = 0;
        } else {
            thr[i] = clamp32(std::ceil(tau) - 1.0);     // x < tau  <=>  not (x > ceil(tau) - 1)
            flip[i] = 1;
        }
    }
    return BNN_OK;
}

}  // extern "C"
