// Host-only helpers of libbnn: the layer-to-implementation mapping of the paper's Alg. 1 over
// a profiled latency table, and batch-norm folding into (threshold, flip).  No GPU code.
#include <algorithm>
#include <cmath>
#include <functional>
#include <limits>
#include <new>
#include <vector>

#include "bnn_internal.h"

extern "C" {

bnn_status bnn_map_layers(const double *cpu_us, const double *gpu_us, int n_batch, int n_layers, int n_impl,
                          int *best_batch, int *mapping, double *total_us)
{
    if (!cpu_us || !gpu_us || !best_batch || !mapping) return BNN_ERR_NULL;
    if (n_batch < 1 || n_layers < 1 || n_impl < 1) return BNN_ERR_SHAPE;
    const size_t cells = (size_t)n_batch * n_layers;
    for (size_t i = 0; i < cells * n_impl; ++i) {
        if (!std::isfinite(cpu_us[i]) || !std::isfinite(gpu_us[i]) || cpu_us[i] < 0 || gpu_us[i] < 0)
            return BNN_ERR_SHAPE;
    }
    // The search of Alg. 1 separates: the cheapest implementation of a (batch size, layer) cell
    // does not depend on any other cell, and a batch size's cost is the sum over its row of cells.
    // So: one argmin per cell into a table, one sum per row, the cheapest row, and that row of the
    // table is the answer.  std::min_element returns the first of equal minima, which is the
    // tie rule of a strict "smaller than" scan.
    std::vector<int> choice;
    std::vector<double> row_cost, latency;
    try {
        choice.resize(cells);
        row_cost.assign(n_batch, 0.0);
        latency.resize(n_impl);
    } catch (const std::bad_alloc &) {
        return BNN_ERR_UNSUPPORTED;      // no exception crosses the C boundary
    }
    for (size_t cell = 0; cell < cells; ++cell) {
        const double *c = cpu_us + cell * n_impl, *g = gpu_us + cell * n_impl;
        std::transform(c, c + n_impl, g, latency.begin(), std::plus<double>());
        const auto cheapest = std::min_element(latency.begin(), latency.end());
        choice[cell] = (int)(cheapest - latency.begin());
        row_cost[cell / n_layers] += *cheapest;
    }
    const int winner = (int)(std::min_element(row_cost.begin(), row_cost.end()) - row_cost.begin());
    std::copy_n(choice.begin() + (size_t)winner * n_layers, n_layers, mapping);
    *best_batch = winner;
    if (total_us) *total_us = row_cost[winner];
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
