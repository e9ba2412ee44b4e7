// Arithmetic of the offline profiler (host only, no HIP): the latency model of paper Section 4.2 fitted from
// microbenchmarks (Section 4.5 "Expert performance metrics"), the maximum batch size (Section 4.5), the arranging
// window's thresholds derived from that model, and the decay-window search for the number of experts to keep on the
// device (Section 4.4, Eq. 1-3).  The measurements themselves are taken by the caller through the library's other calls.
#include <cmath>
#include <vector>
#include <cstdint>

#include "../../include/coe.h"

extern "C" {

int coe_profiler_fit_latency(int32_t n, const int32_t* batch, const double* latency_us, double* k_us, double* b_us)
{
    if (n < 2 || !batch || !latency_us || !k_us || !b_us) return COE_EINVAL;
    double mx = 0.0, my = 0.0;
    for (int32_t i = 0; i < n; ++i) { mx += batch[i]; my += latency_us[i]; }
    mx /= n; my /= n;
    double sxx = 0.0, sxy = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        const double dx = batch[i] - mx;
        sxx += dx * dx;
        sxy += dx * (latency_us[i] - my);
    }
    if (!(sxx > 0.0)) return COE_EINVAL;                  // all batch sizes equal: no line
    *k_us = sxy / sxx;
    *b_us = my - *k_us * mx;
    return COE_OK;
}

int coe_profiler_max_batch(int32_t n, const int32_t* batch, const double* latency_us, double tol, int32_t* max_batch)
{
    if (n < 1 || !batch || !latency_us || !max_batch || !(tol >= 0.0)) return COE_EINVAL;
    double best = INFINITY;
    for (int32_t i = 0; i < n; ++i) {
        if (batch[i] <= 0 || !(latency_us[i] > 0.0)) return COE_EINVAL;
        best = std::fmin(best, latency_us[i] / batch[i]);
    }
    int32_t pick = -1;
    for (int32_t i = 0; i < n; ++i)
        if (latency_us[i] / batch[i] <= best * (1.0 + tol) && (pick < 0 || batch[i] < pick)) pick = batch[i];
    *max_batch = pick;
    return COE_OK;
}

int coe_profiler_arranging_window(double k_us, double b_us, double load_us, double efficiency, int32_t* min_group_resident,
                                  int32_t* min_group_missing)
{
    if (!(k_us > 0.0) || !(b_us >= 0.0) || !(load_us >= 0.0) || !(efficiency >= 0.0) || !(efficiency < 1.0) ||
        !min_group_resident || !min_group_missing)
        return COE_EINVAL;
    const double r = efficiency / (1.0 - efficiency);
    const double a = std::ceil(r * b_us / k_us), b = std::ceil(r * (b_us + load_us) / k_us);
    if (b > 2147483647.0) return COE_ERANGE;
    *min_group_resident = (int32_t)a;
    *min_group_missing = (int32_t)b;
    return COE_OK;
}

int coe_profiler_usage_probabilities(int32_t n_requests, int32_t max_stages, const int32_t* path, int32_t n_experts, float* prob)
{
    if (n_requests <= 0 || max_stages <= 0 || n_experts <= 0 || !path || !prob) return COE_EINVAL;
    std::vector<int64_t> visits((size_t)n_experts, 0);
    std::vector<int32_t> seen((size_t)n_experts, -1);          // last request that counted the expert (a path visits it once)
    for (int32_t r = 0; r < n_requests; ++r)
        for (int32_t s = 0; s < max_stages; ++s) {
            const int32_t e = path[(size_t)r * max_stages + s];
            if (e == -1) continue;
            if (e < 0 || e >= n_experts) return COE_EINVAL;
            if (seen[e] != r) { seen[e] = r; ++visits[e]; }
        }
    for (int32_t e = 0; e < n_experts; ++e) prob[e] = (float)((double)visits[e] / (double)n_requests);
    return COE_OK;
}

int coe_profiler_memory_scores(int32_t n, const int64_t* nbytes, double* score, int64_t* unit_bytes)
{
    if (n <= 0 || !nbytes || !score || !unit_bytes) return COE_EINVAL;
    int64_t unit = nbytes[0];
    for (int32_t e = 0; e < n; ++e) {
        if (nbytes[e] <= 0) return COE_EINVAL;
        if (nbytes[e] < unit) unit = nbytes[e];
    }
    for (int32_t e = 0; e < n; ++e) score[e] = (double)nbytes[e] / (double)unit;
    *unit_bytes = unit;
    return COE_OK;
}

int coe_profiler_executable_batch(int64_t free_bytes, int64_t bytes_per_request, int32_t profiled_max_batch, int32_t* batch)
{
    if (free_bytes < 0 || bytes_per_request <= 0 || profiled_max_batch < 0 || !batch) return COE_EINVAL;
    const int64_t fits = free_bytes / bytes_per_request;
    *batch = (int32_t)(fits < (int64_t)profiled_max_batch ? fits : (int64_t)profiled_max_batch);
    return COE_OK;
}

int coe_profiler_expert_budget(int64_t total_bytes, int64_t reserve_bytes, int64_t bytes_per_request, int32_t max_batch,
                               int64_t unit_bytes, int64_t* budget_bytes, double* budget_scores)
{
    if (total_bytes < 0 || reserve_bytes < 0 || bytes_per_request < 0 || max_batch < 0 || unit_bytes <= 0 || !budget_bytes)
        return COE_EINVAL;
    // (compared before subtracting: the workspace of a large batch may exceed any memory)
    const long double need = (long double)reserve_bytes + (long double)bytes_per_request * (long double)max_batch;
    const int64_t left = need >= (long double)total_bytes ? 0 : total_bytes - reserve_bytes - bytes_per_request * (int64_t)max_batch;
    *budget_bytes = left;
    if (budget_scores) *budget_scores = (double)left / (double)unit_bytes;
    return COE_OK;
}

int coe_profiler_window_step(int32_t n_experts_total, double initial_window, double error_margin, int32_t fit_points,
                             int32_t n_measured, const double* throughput, coe_window_state* out)
{
    if (n_experts_total <= 0 || !(initial_window > 0.0) || !(initial_window < 100.0) || !(error_margin >= 0.0) || fit_points < 2 ||
        n_measured < 0 || (n_measured > 0 && !throughput) || !out)
        return COE_EINVAL;
    const double decay = 1.0 - initial_window / 100.0;                                   // Eq. 1
    // window k: [low_k, high_k) on the expert axis, size_k = initial_window * decay^k
    double low = 0.0, size = initial_window;
    for (int32_t k = 0; k + 1 < n_measured; ++k) { low += size; size *= decay; }
    auto count = [&](double bound) {
        const double c = std::ceil(bound - 1e-9);
        return (int32_t)(c < 1.0 ? 1.0 : c > n_experts_total ? (double)n_experts_total : c);
    };
    out->window_low = low;
    out->window_high = low + size;
    out->n_low = count(low);
    out->n_high = count(low + size);
    out->linear_error = 0.0;
    out->status = COE_WINDOW_MEASURE;
    out->n_next = out->n_high;
    if (n_measured == 0) return COE_OK;                                                   // measure at the first window's upper bound
    // the window just measured is window n_measured - 1 = [low, low + size)
    const int32_t N = n_measured - 1;                                                     // values before the newest one
    if (N >= fit_points) {
        // Eq. 2: least-squares line through (1, t_1) ... (N, t_N); Eq. 3: relative shortfall of value N + 1
        double mx = 0.0, my = 0.0;
        for (int32_t i = 0; i < N; ++i) { mx += i + 1; my += throughput[i]; }
        mx /= N; my /= N;
        double sxx = 0.0, sxy = 0.0;
        for (int32_t i = 0; i < N; ++i) { sxx += (i + 1 - mx) * (i + 1 - mx); sxy += (i + 1 - mx) * (throughput[i] - my); }
        const double k = sxy / sxx, b = my - k * mx;
        const double predicted = k * (N + 1) + b;
        if (predicted > 0.0) {
            out->linear_error = (predicted - throughput[N]) / predicted;
            if (out->linear_error > error_margin) {
                out->status = COE_WINDOW_SHORTFALL;
                out->n_next = 0;
                return COE_OK;
            }
        }
    }
    if (out->n_high >= n_experts_total) {               // every expert was loaded for this measurement: nothing left to slide to
        out->status = COE_WINDOW_END;
        out->n_next = 0;
        return COE_OK;
    }
    out->n_next = count(low + size + size * decay);      // upper bound of the next window
    return COE_OK;
}

}  // extern "C"
