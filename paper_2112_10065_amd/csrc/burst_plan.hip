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

// ---- Branch/join blocks (section 4.2, paragraph "Multi-chain graph reduction") ----------------------
namespace {

struct BranchView {
    int L;
    const double *comp, *comm, *sync, *join, *move;
    double comm_at(int l, int b, int a, int G) const { return comm != nullptr ? comm[((size_t)l * G + b) * G + a] : 0.0; }
    double sync_at(int l, int a, int G) const { return sync != nullptr ? sync[(size_t)l * G + a] : 0.0; }
    double join_at(int b, int a, int G) const { return join != nullptr ? join[(size_t)b * G + a] : 0.0; }
    double move_at(int g, int h, int G) const { return move != nullptr ? move[(size_t)g * G + h] : INFINITY; }
};

// Result of searching one branch from a pinned start: per joining-layer count h the time, the plan and its widest count.
struct BranchReach {
    std::vector<double> time;       // [G]
    std::vector<int> plan;          // [G][L] GPU-count indices
    std::vector<int> widest;        // [G] largest GPU count on the plan, 0 for an empty branch
};

void search_branch(const BranchView &br, const int32_t *gpus, int G, double limit, int start, BranchReach *out)
{
    const int L = br.L;
    out->time.assign(G, 0.0);
    out->plan.assign((size_t)G * (L > 0 ? L : 1), 0);
    out->widest.assign(G, 0);
    if (L == 0) {
        for (int h = 0; h < G; ++h) out->time[h] = br.join_at(start, h, G);
        return;
    }
    std::vector<double> S((size_t)(L + 1) * G, INFINITY), T((size_t)(L + 1) * G, INFINITY);
    std::vector<int> from((size_t)(L + 1) * G, -1);
    for (int a = 0; a < G; ++a) {      // layer 1 has the pinned branching layer as its only predecessor
        const double t1 = br.comm_at(0, start, a, G) + br.comp[a] + br.sync_at(0, a, G);
        S[(size_t)G + a] = t1;
        T[(size_t)G + a] = t1;
        from[(size_t)G + a] = start;
    }
    for (int i = 2; i <= L; ++i)
        for (int a = 0; a < G; ++a) {
            Scan scan(limit);
            double best_t = INFINITY;
            for (int b = 0; b < G; ++b) {
                const double amp = T[(size_t)(i - 1) * G + b] * gpus[b] / br.comp[(size_t)(i - 2) * G];
                const double c = br.comm_at(i - 1, b, a, G);
                if (scan.offer(b, amp, S[(size_t)(i - 1) * G + b] + c)) best_t = c;
            }
            S[(size_t)i * G + a] = scan.best_cost + br.comp[(size_t)(i - 1) * G + a] + br.sync_at(i - 1, a, G);
            T[(size_t)i * G + a] = best_t + br.comp[(size_t)(i - 1) * G + a] + br.sync_at(i - 1, a, G);
            from[(size_t)i * G + a] = scan.pick;
        }
    for (int h = 0; h < G; ++h) {
        Scan scan(limit);
        for (int b = 0; b < G; ++b)
            scan.offer(b, T[(size_t)L * G + b] * gpus[b] / br.comp[(size_t)(L - 1) * G], S[(size_t)L * G + b] + br.join_at(b, h, G));
        out->time[h] = scan.best_cost;
        int b = scan.pick, widest = 0;
        for (int i = L; i >= 1; --i) {
            out->plan[(size_t)h * L + i - 1] = b;
            widest = gpus[b] > widest ? gpus[b] : widest;
            b = from[(size_t)i * G + b];
        }
        out->widest[h] = widest;
    }
}

// Decisions of one block for one (g, h).
struct BlockCell {
    double tr = 0.0;
    int critical = 0, extra = 0;
    std::vector<unsigned char> parallel;
    std::vector<int> plan;          // branch plans concatenated
};

bool check_table(const char *what, const double *t, long long n, bool positive, bool allow_inf)
{
    if (t == nullptr) return true;
    for (long long k = 0; k < n; ++k) {
        const double v = t[k];
        const bool ok = positive ? (std::isfinite(v) && v > 0.0) : (v >= 0.0 && (allow_inf || std::isfinite(v)));
        if (!ok) { dp_set_error("dp_plan_graph: %s[%lld] is out of range", what, k); return false; }
    }
    return true;
}

}  // namespace

extern "C" dp_status dp_plan_graph(const dp_plan_graph_desc *gd, int32_t *gpus_per_layer, int32_t *branch_gpus, uint8_t *branch_parallel,
                                   int32_t *critical_branch, double *iteration_time, double *S_out, double *T_out)
{
    if (gd == nullptr || gpus_per_layer == nullptr || iteration_time == nullptr || gd->chain.gpu_counts == nullptr || gd->chain.comp == nullptr ||
        gd->n_branches == nullptr) {
        dp_set_error("dp_plan_graph: null argument");
        return DP_ERR_NULL;
    }
    const dp_plan_desc *d = &gd->chain;
    const int L = d->n_layers, G = d->n_gpu_counts;
    if (L < 1 || G < 1 || d->gpu_counts[0] != 1 || std::isnan(d->amp_limit)) {
        dp_set_error("dp_plan_graph: need n_layers >= 1, n_gpu_counts >= 1, gpu_counts[0] == 1 and a limit that is a number");
        return DP_ERR_BAD_DESC;
    }
    for (int a = 1; a < G; ++a)
        if (d->gpu_counts[a] <= d->gpu_counts[a - 1]) { dp_set_error("dp_plan_graph: gpu_counts must ascend strictly"); return DP_ERR_BAD_DESC; }
    if (gd->n_branches[0] != 0) { dp_set_error("dp_plan_graph: the first layer has no branching layer before it"); return DP_ERR_BAD_DESC; }
    long long total_branches = 0, total_branch_layers = 0;
    for (int i = 0; i < L; ++i) {
        if (gd->n_branches[i] < 0) { dp_set_error("dp_plan_graph: n_branches[%d] < 0", i); return DP_ERR_BAD_DESC; }
        total_branches += gd->n_branches[i];
    }
    if (total_branches > 0 && gd->branches == nullptr) { dp_set_error("dp_plan_graph: branches is null"); return DP_ERR_NULL; }
    if (!check_table("comp", d->comp, (long long)L * G, true, false) || !check_table("sync", d->sync, (long long)L * G, false, false) ||
        !check_table("comm", d->comm, (long long)L * G * G, false, false))
        return DP_ERR_BAD_DESC;
    for (long long k = 0; k < total_branches; ++k) {
        const dp_plan_branch &b = gd->branches[k];
        if (b.n_layers < 0) { dp_set_error("dp_plan_graph: branch %lld has n_layers < 0", k); return DP_ERR_BAD_DESC; }
        if (b.n_layers > 0 && b.comp == nullptr) { dp_set_error("dp_plan_graph: branch %lld has no comp table", k); return DP_ERR_NULL; }
        if (!check_table("branch comp", b.comp, (long long)b.n_layers * G, true, false) ||
            !check_table("branch sync", b.sync, (long long)b.n_layers * G, false, false) ||
            !check_table("branch comm", b.comm, (long long)b.n_layers * G * G, false, false) ||
            !check_table("branch join", b.join, (long long)G * G, false, false) || !check_table("branch move", b.move, (long long)G * G, false, true))
            return DP_ERR_BAD_DESC;
        total_branch_layers += b.n_layers;
    }

    const int32_t *gpus = d->gpu_counts;
    std::vector<double> S((size_t)(L + 1) * G, 0.0), T((size_t)(L + 1) * G, 0.0), amp((size_t)G, 0.0), amp_next((size_t)G, 0.0);
    std::vector<int> from((size_t)(L + 1) * G, -1);
    std::vector<std::vector<BlockCell>> blocks((size_t)L);   // [layer][g * G + h], empty for a direct edge
    std::vector<long long> first_branch((size_t)L, 0);
    long long seen = 0;
    for (int i = 0; i < L; ++i) { first_branch[i] = seen; seen += gd->n_branches[i]; }

    for (int i = 1; i <= L; ++i) {
        const double *comp_i = d->comp + (size_t)(i - 1) * G;
        const double *sync_i = d->sync != nullptr ? d->sync + (size_t)(i - 1) * G : nullptr;
        const double *comm_i = d->comm != nullptr ? d->comm + (size_t)(i - 1) * G * G : nullptr;
        const int nb = gd->n_branches[i - 1];
        double one_gpu = comp_i[0], branch_one_gpu = 0.0;
        std::vector<BlockCell> &cells = blocks[i - 1];
        if (nb > 0) {
            std::vector<BranchView> view((size_t)nb);
            int plan_len = 0;
            for (int k = 0; k < nb; ++k) {
                const dp_plan_branch &b = gd->branches[first_branch[i - 1] + k];
                view[k] = BranchView{b.n_layers, b.comp, b.comm, b.sync, b.join, b.move};
                for (int l = 0; l < b.n_layers; ++l) branch_one_gpu += b.comp[(size_t)l * G];
                plan_len += b.n_layers;
            }
            one_gpu += branch_one_gpu;
            cells.assign((size_t)G * G, BlockCell());
            std::vector<BranchReach> reach((size_t)nb);
            for (int g = 0; g < G; ++g) {
                for (int k = 0; k < nb; ++k) search_branch(view[k], gpus, G, d->amp_limit, g, &reach[k]);
                for (int h = 0; h < G; ++h) {
                    BlockCell &cell = cells[(size_t)g * G + h];
                    cell.parallel.assign((size_t)nb, 0);
                    cell.plan.reserve((size_t)plan_len);
                    double t = 0.0;
                    for (int k = 0; k < nb; ++k) {
                        t += reach[k].time[h];
                        if (reach[k].time[h] > reach[cell.critical].time[h]) cell.critical = k;
                        for (int l = 0; l < view[k].L; ++l) cell.plan.push_back(reach[k].plan[(size_t)h * view[k].L + l]);
                    }
                    const double longest = reach[cell.critical].time[h];
                    const double sync_h = sync_i != nullptr ? sync_i[h] : 0.0;
                    for (int k = 0; k < nb; ++k) {
                        const double tk = reach[k].time[h];
                        if (k == cell.critical || view[k].L == 0 || !(tk + view[k].move_at(g, h, G) <= longest)) continue;
                        const double a_moved = (t - tk + comp_i[h] + sync_h) * (gpus[h] + cell.extra + reach[k].widest[h]) / one_gpu;
                        if (a_moved <= d->amp_limit) {
                            t -= tk;
                            cell.extra += reach[k].widest[h];
                            cell.parallel[k] = 1;
                        }
                    }
                    cell.tr = t;
                }
            }
        }
        for (int a = 0; a < G; ++a) {
            Scan scan(d->amp_limit);
            double best_t = INFINITY;
            for (int b = 0; b < G; ++b) {
                const double c = nb > 0 ? cells[(size_t)b * G + a].tr : (comm_i != nullptr ? comm_i[(size_t)b * G + a] : 0.0);
                if (scan.offer(b, amp[b], S[(size_t)(i - 1) * G + b] + c)) best_t = c;
            }
            const double sy = sync_i != nullptr ? sync_i[a] : 0.0;
            S[(size_t)i * G + a] = scan.best_cost + comp_i[a] + sy;
            T[(size_t)i * G + a] = best_t + comp_i[a] + sy;
            from[(size_t)i * G + a] = scan.pick;
            const int extra = nb > 0 ? cells[(size_t)scan.pick * G + a].extra : 0;
            amp_next[a] = T[(size_t)i * G + a] * (gpus[a] + extra) / one_gpu;
        }
        amp.swap(amp_next);
    }
    Scan last(d->amp_limit);
    for (int a = 0; a < G; ++a) last.offer(a, amp[a], S[(size_t)L * G + a]);
    std::vector<int> plan((size_t)L, 0);
    int a = last.pick;
    for (int i = L; i >= 1; --i) {
        plan[i - 1] = a;
        gpus_per_layer[i - 1] = gpus[a];
        a = from[(size_t)i * G + a];
    }
    long long layer_at = 0;
    for (int i = 0; i < L; ++i) {
        const int nb = gd->n_branches[i];
        if (critical_branch != nullptr) critical_branch[i] = -1;
        if (nb == 0) continue;
        const BlockCell &cell = blocks[i][(size_t)plan[i - 1] * G + plan[i]];
        if (critical_branch != nullptr) critical_branch[i] = cell.critical;
        for (int k = 0; k < nb; ++k)
            if (branch_parallel != nullptr) branch_parallel[first_branch[i] + k] = cell.parallel[k];
        for (size_t l = 0; l < cell.plan.size(); ++l, ++layer_at)
            if (branch_gpus != nullptr) branch_gpus[layer_at] = gpus[cell.plan[l]];
    }
    *iteration_time = last.best_cost;
    if (S_out != nullptr) std::copy(S.begin(), S.end(), S_out);
    if (T_out != nullptr) std::copy(T.begin(), T.end(), T_out);
    return DP_OK;
}
