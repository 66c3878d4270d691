// Burst-parallel planner for a chain of layers (paper section 4.2, algorithm "Search Linear") and the
// closed-form communication costs of section 4.1.  Host code only: the tables are a few kilobytes.
#include "../../include/dp.h"
#include <cmath>
#include <vector>

void dp_set_error(const char *fmt, ...);   // dp_api.hip

namespace {

// One admission scan of the algorithm: candidates come in GPU-count order with their amplification and
// their cost; a candidate is taken when its amplification is within max(best admitted so far, limit)
// and its cost does not exceed the best so far.  Used for every predecessor choice and for the choice
// of the last layer's GPU count.
struct Scan {
    double limit;
    double best_amp = INFINITY, best_cost = INFINITY;
    int pick = -1;
    explicit Scan(double lim) : limit(lim) {}
    bool offer(int idx, double amp, double cost)
    {
        const double bound = best_amp > limit ? best_amp : limit;
        if (!(amp <= bound) || !(cost <= best_cost)) return false;
        best_cost = cost;
        best_amp = amp < best_amp ? amp : best_amp;
        pick = idx;
        return true;
    }
};

bool finite_nonneg(double v) { return std::isfinite(v) && v >= 0.0; }

}  // namespace

extern "C" dp_status dp_plan_chain(const dp_plan_desc *d, int32_t *gpus_per_layer, double *iteration_time, double *S_out,
                                   double *T_out)
{
    if (d == nullptr || gpus_per_layer == nullptr || iteration_time == nullptr || d->gpu_counts == nullptr || d->comp == nullptr) {
        dp_set_error("dp_plan_chain: null argument");
        return DP_ERR_NULL;
    }
    const int L = d->n_layers, G = d->n_gpu_counts;
    if (L < 1 || G < 1 || d->gpu_counts[0] != 1 || std::isnan(d->amp_limit)) {
        dp_set_error("dp_plan_chain: need n_layers >= 1, n_gpu_counts >= 1, gpu_counts[0] == 1 and a limit that is a number");
        return DP_ERR_BAD_DESC;
    }
    for (int a = 1; a < G; ++a)
        if (d->gpu_counts[a] <= d->gpu_counts[a - 1]) {
            dp_set_error("dp_plan_chain: gpu_counts must ascend strictly");
            return DP_ERR_BAD_DESC;
        }
    for (long long k = 0; k < (long long)L * G; ++k) {
        if (!std::isfinite(d->comp[k]) || d->comp[k] <= 0.0) { dp_set_error("dp_plan_chain: comp[%lld] is not a positive finite time", k); return DP_ERR_BAD_DESC; }
        if (d->sync != nullptr && !finite_nonneg(d->sync[k])) { dp_set_error("dp_plan_chain: sync[%lld] is negative or not finite", k); return DP_ERR_BAD_DESC; }
    }
    if (d->comm != nullptr)
        for (long long k = 0; k < (long long)L * G * G; ++k)
            if (!finite_nonneg(d->comm[k])) { dp_set_error("dp_plan_chain: comm[%lld] is negative or not finite", k); return DP_ERR_BAD_DESC; }

    // rows 0..L; row i describes layer i of the paper's 1-based numbering (inputs are 0-based: layer i is row i-1 there)
    std::vector<double> S((size_t)(L + 1) * G, 0.0), T((size_t)(L + 1) * G, 0.0), amp((size_t)G, 0.0);
    std::vector<int> from((size_t)(L + 1) * G, -1);
    for (int i = 1; i <= L; ++i) {
        const double *comp_i = d->comp + (size_t)(i - 1) * G;
        const double *sync_i = d->sync != nullptr ? d->sync + (size_t)(i - 1) * G : nullptr;
        const double *comm_i = d->comm != nullptr ? d->comm + (size_t)(i - 1) * G * G : nullptr;
        const double *S_prev = &S[(size_t)(i - 1) * G];
        for (int a = 0; a < G; ++a) {
            Scan scan(d->amp_limit);
            double best_t = INFINITY;
            for (int b = 0; b < G; ++b) {
                const double c = comm_i != nullptr ? comm_i[(size_t)b * G + a] : 0.0;
                if (scan.offer(b, amp[b], S_prev[b] + c)) best_t = c;
            }
            const double sy = sync_i != nullptr ? sync_i[a] : 0.0;
            S[(size_t)i * G + a] = scan.best_cost + comp_i[a] + sy;
            T[(size_t)i * G + a] = best_t + comp_i[a] + sy;
            from[(size_t)i * G + a] = scan.pick;
        }
        for (int a = 0; a < G; ++a) amp[a] = T[(size_t)i * G + a] * d->gpu_counts[a] / comp_i[0];   // Amp(i, g) for the next layer's scans
    }
    Scan last(d->amp_limit);
    for (int a = 0; a < G; ++a) last.offer(a, amp[a], S[(size_t)L * G + a]);
    int a = last.pick;
    for (int i = L; i >= 1; --i) {
        gpus_per_layer[i - 1] = d->gpu_counts[a];
        a = from[(size_t)i * G + a];
    }
    *iteration_time = last.best_cost;
    if (S_out != nullptr) std::copy(S.begin(), S.end(), S_out);
    if (T_out != nullptr) std::copy(T.begin(), T.end(), T_out);
    return DP_OK;
}

extern "C" dp_status dp_plan_cost_tables(int32_t L, int32_t G, const int32_t *gpu_counts, const double *act_bytes, const double *param_bytes,
                                         double bandwidth, double delay, double *comm_out, double *sync_out)
{
    if (gpu_counts == nullptr || act_bytes == nullptr || param_bytes == nullptr || comm_out == nullptr || sync_out == nullptr) {
        dp_set_error("dp_plan_cost_tables: null argument");
        return DP_ERR_NULL;
    }
    if (L < 1 || G < 1 || !(bandwidth > 0.0) || !finite_nonneg(delay)) {
        dp_set_error("dp_plan_cost_tables: need n_layers >= 1, n_gpu_counts >= 1, bandwidth > 0, delay >= 0");
        return DP_ERR_BAD_DESC;
    }
    for (int a = 0; a < G; ++a)
        if (gpu_counts[a] < 1) { dp_set_error("dp_plan_cost_tables: gpu_counts[%d] < 1", a); return DP_ERR_BAD_DESC; }
    for (int i = 0; i < L; ++i) {
        if (!finite_nonneg(act_bytes[i]) || !finite_nonneg(param_bytes[i])) { dp_set_error("dp_plan_cost_tables: byte counts of layer %d are negative or not finite", i); return DP_ERR_BAD_DESC; }
        for (int b = 0; b < G; ++b)
            for (int a = 0; a < G; ++a) {
                double t = 0.0;
                const int g = gpu_counts[b], h = gpu_counts[a];
                if (i > 0 && g != h) {
                    const int lo = g < h ? g : h, hi = g < h ? h : g;
                    const double payload = act_bytes[i] * (1.0 / lo - 1.0 / hi);
                    t = 2.0 * (payload / bandwidth + delay);
                }
                comm_out[((size_t)i * G + b) * G + a] = t;
            }
        for (int a = 0; a < G; ++a) {
            const int g = gpu_counts[a];
            sync_out[(size_t)i * G + a] = g == 1 ? 0.0 : 2.0 * (param_bytes[i] * (g - 1.0) / g / bandwidth + delay);
        }
    }
    return DP_OK;
}
