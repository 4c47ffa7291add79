// Host-side planning of the expert offload runtime (Section III.C): the break-even batch size of
// the cost model (Eq. 7-8) and the two-stage expert placement (Algorithm 2).  No device work.
#include "haq_common.h"

#include <algorithm>
#include <cmath>
#include <new>
#include <numeric>
#include <vector>

using namespace haq;

extern "C" {

int32_t haq_offload_n_critical(double t_e, double latency_cpu, double latency_gpu, int64_t* n_critical) {
    if (!n_critical) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_offload_n_critical: null output");
    if (!(t_e >= 0.0) || !(latency_cpu > 0.0) || !(latency_gpu >= 0.0) || !std::isfinite(t_e) || !std::isfinite(latency_cpu) ||
        !std::isfinite(latency_gpu))
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_offload_n_critical: t_e=%g latency_cpu=%g latency_gpu=%g", t_e, latency_cpu, latency_gpu);
    if (!(latency_cpu > latency_gpu)) {  // the CPU is never slower: never transfer
        *n_critical = -1;
        return HAQ_OK;
    }
    // largest n with n * latency_cpu <= t_e + n * latency_gpu: start from the real-valued
    // break-even point and settle the boundary with the inequality itself
    const double x = t_e / (latency_cpu - latency_gpu);
    if (x > 9.0e18) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_offload_n_critical: break-even batch beyond the integer range");
    int64_t n = (int64_t)std::floor(x);
    auto cpu_not_slower = [&](int64_t m) { return (double)m * latency_cpu <= t_e + (double)m * latency_gpu; };
    while (n > 0 && !cpu_not_slower(n)) --n;
    while (cpu_not_slower(n + 1)) ++n;
    *n_critical = n;
    return HAQ_OK;
}

int32_t haq_select_experts(int32_t num_layers, int32_t experts_per_layer, int32_t top_k, int32_t supplement_k,
                           const int32_t* path_offsets, const int32_t* path_experts, int32_t path_len,
                           const double* path_freq, const double* expert_freq, int32_t* selected, int32_t* n_selected) {
    if (num_layers <= 0 || experts_per_layer <= 0 || top_k < 1 || supplement_k < 0 || path_len < 1)
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_select_experts: layers=%d experts=%d top_k=%d supplement_k=%d path_len=%d", num_layers,
                 experts_per_layer, top_k, supplement_k, path_len);
    if (!path_offsets || !path_experts || !path_freq || !expert_freq || !selected || !n_selected)
        HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_select_experts: null buffer");
    const int cap = top_k + supplement_k;
    for (int l = 0; l < num_layers; ++l) {
        const int p0 = path_offsets[l], p1 = path_offsets[l + 1];
        if (p0 < 0 || p1 < p0) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_select_experts: path_offsets of layer %d", l);
        for (int p = p0; p < p1; ++p)
            for (int j = 0; j < path_len; ++j) {
                const int e = path_experts[(size_t)p * path_len + j];
                if (e < 0 || e >= experts_per_layer) HAQ_FAIL(HAQ_ERR_INVALID_ARG, "haq_select_experts: expert %d in a path of layer %d", e, l);
            }
    }
    // Algorithm 2, per layer.  Stage I: lay the layer's paths end to end, most frequent path first
    // (equal frequencies in input order); the first top_k distinct experts of that sequence are
    // placed.  Stage II: of the experts not placed yet, the most frequently activated ones (ties
    // by index) fill the remaining top_k + supplement_k - (placed) positions.
    try {
    std::vector<int> paths, rest;
    std::vector<char> placed((size_t)experts_per_layer);
    for (int l = 0; l < num_layers; ++l) {
        int32_t* sel = selected + (size_t)l * cap;
        const double* f = expert_freq + (size_t)l * experts_per_layer;
        std::fill(placed.begin(), placed.end(), 0);
        paths.resize((size_t)(path_offsets[l + 1] - path_offsets[l]));
        std::iota(paths.begin(), paths.end(), path_offsets[l]);
        std::stable_sort(paths.begin(), paths.end(), [&](int a, int b) { return path_freq[a] > path_freq[b]; });
        int n = 0;
        for (size_t i = 0; i < paths.size() * (size_t)path_len && n < top_k; ++i) {
            const int e = path_experts[(size_t)paths[i / path_len] * path_len + i % path_len];
            if (!placed[e]) {
                placed[e] = 1;
                sel[n++] = e;
            }
        }
        rest.clear();
        for (int e = 0; e < experts_per_layer; ++e)
            if (!placed[e]) rest.push_back(e);
        std::stable_sort(rest.begin(), rest.end(), [&](int a, int b) { return f[a] > f[b]; });
        for (size_t i = 0; i < rest.size() && n < cap; ++i) sel[n++] = rest[i];
        n_selected[l] = n;
        std::fill(sel + n, sel + cap, -1);
    }
    } catch (const std::bad_alloc&) {
        HAQ_FAIL(HAQ_ERR_HIP, "haq_select_experts: out of host memory");
    }
    return HAQ_OK;
}

}  // extern "C"
