// Host-side performance predictor: one training iteration of a pipeline of stages in 1F1B order
// (workload simulator, Section 3.2 of the paper), the metrics of Section 4.1 (Eq. 1-3) and the layer
// split of the automatic parallel planner (Section 3.3).  No GPU code.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <vector>

#include "../../include/hh_predict.h"

namespace hh {
int set_error(int code, const char* msg);
}

namespace {

int fail(int code, const char* msg) { return hh::set_error(code, msg); }

struct Op {
    bool fwd;
    int m;
};

// Stage p of P: forwards of the first w = min(M, P - p) micro-batches, then backward m / forward m + w.
std::vector<Op> stage_program(int p, int P, int M) {
    const int w = std::min(M, P - p);
    std::vector<Op> ops;
    ops.reserve(2 * (size_t)M);
    for (int m = 0; m < w; m++) ops.push_back({true, m});
    for (int m = 0; m < M; m++) {
        ops.push_back({false, m});
        if (m + w < M) ops.push_back({true, m + w});
    }
    return ops;
}

struct Timeline {
    double iter_ms;
    std::vector<double> finish;   // per stage
};

// tf[p], tb[p]: one micro-batch through all layers of stage p; link[p]: boundary tensor p <-> p+1.
// Returns false if the programs cannot all complete (cannot happen for the 1F1B programs above).
bool run_pipeline(const std::vector<double>& tf, const std::vector<double>& tb, const std::vector<double>& link, int M,
                  Timeline& out) {
    const int P = (int)tf.size();
    std::vector<std::vector<Op>> prog(P);
    for (int p = 0; p < P; p++) prog[p] = stage_program(p, P, M);
    const double NOT_DONE = -1.0;
    std::vector<double> f_done((size_t)P * M, NOT_DONE), b_done((size_t)P * M, NOT_DONE);
    std::vector<size_t> pc(P, 0);
    std::vector<double> free_at(P, 0.0);
    size_t left = 0;
    for (int p = 0; p < P; p++) left += prog[p].size();
    while (left > 0) {
        bool moved = false;
        for (int p = 0; p < P; p++) {
            while (pc[p] < prog[p].size()) {
                const Op op = prog[p][pc[p]];
                double ready = 0.0;
                if (op.fwd && p > 0) {
                    const double d = f_done[(size_t)(p - 1) * M + op.m];
                    if (d == NOT_DONE) break;
                    ready = d + link[p - 1];
                } else if (!op.fwd && p < P - 1) {
                    const double d = b_done[(size_t)(p + 1) * M + op.m];
                    if (d == NOT_DONE) break;
                    ready = d + link[p];
                }
                const double start = std::max(free_at[p], ready);
                free_at[p] = start + (op.fwd ? tf[p] : tb[p]);
                (op.fwd ? f_done : b_done)[(size_t)p * M + op.m] = free_at[p];
                pc[p]++;
                left--;
                moved = true;
            }
        }
        if (!moved) return false;
    }
    out.finish = free_at;
    out.iter_ms = *std::max_element(free_at.begin(), free_at.end());
    return true;
}

int check_stages(const hh_sim_stage* st, int n, bool need_layers) {
    if (!st) return fail(HH_ERR_INVALID_ARG, "stages is NULL");
    if (n <= 0) return fail(HH_ERR_INVALID_ARG, "n_stages must be positive");
    for (int p = 0; p < n; p++) {
        if (need_layers && st[p].n_layers <= 0) return fail(HH_ERR_INVALID_ARG, "every stage needs at least one layer");
        if (st[p].n_devices <= 0) return fail(HH_ERR_INVALID_ARG, "every stage needs at least one device");
        if (!(st[p].fwd_ms > 0.0) || !(st[p].bwd_ms > 0.0)) return fail(HH_ERR_INVALID_ARG, "fwd_ms and bwd_ms must be positive");
        if (!(st[p].peak_tflops > 0.0)) return fail(HH_ERR_INVALID_ARG, "peak_tflops must be positive");
    }
    return HH_OK;
}

int simulate(const hh_sim_stage* st, const int32_t* layers, int P, int M, int micro_batch, int seq, int hidden, int dp,
             double flop_per_layer, hh_sim_result* out, double* finish, uint64_t* peak) {
    std::vector<double> tf(P), tb(P), link(P > 1 ? P - 1 : 0);
    const double msg_bytes = (double)micro_batch * seq * hidden * 2.0;   // Eq. (3)
    for (int p = 0; p < P; p++) {
        tf[p] = layers[p] * st[p].fwd_ms;
        tb[p] = layers[p] * st[p].bwd_ms;
        if (p < P - 1) link[p] = st[p].link_gbytes_per_s > 0.0 ? msg_bytes / (st[p].link_gbytes_per_s * 1e9) * 1e3 : 0.0;
    }
    Timeline tl;
    if (!run_pipeline(tf, tb, link, M, tl)) return fail(HH_ERR_INVALID_ARG, "pipeline programs deadlocked");
    double busiest = 0.0, peak_sum = 0.0, layer_count = 0.0;
    int64_t devices = 0;
    for (int p = 0; p < P; p++) {
        busiest = std::max(busiest, M * (tf[p] + tb[p]));
        devices += st[p].n_devices;
        peak_sum += st[p].peak_tflops * st[p].n_devices;
        layer_count += layers[p];
        if (finish) finish[p] = tl.finish[p];
        if (peak) {
            const uint64_t live = (uint64_t)std::min(M, P - p);
            peak[p] = (uint64_t)layers[p] * (st[p].weight_bytes + st[p].grad_bytes + st[p].optimizer_bytes) +
                      live * (uint64_t)layers[p] * st[p].saved_act_bytes;
        }
    }
    const double iter_s = tl.iter_ms * 1e-3;
    out->iter_ms = tl.iter_ms;
    out->bubble_fraction = 1.0 - busiest / tl.iter_ms;
    out->n_devices = devices;
    out->tokens_per_s_per_device = (double)seq * ((double)M * micro_batch * dp) / ((double)devices * iter_s);   // Eq. (1)
    out->tflops_per_device = flop_per_layer * layer_count * M * dp / iter_s / (double)devices / 1e12;
    out->mean_peak_tflops = peak_sum / (double)devices;
    out->mfu = out->tflops_per_device / out->mean_peak_tflops;                                                  // Eq. (2)
    return HH_OK;
}

int check_run(int M, int micro_batch, int seq, int hidden, int dp, double flop) {
    if (M <= 0 || micro_batch <= 0 || seq <= 0 || hidden <= 0 || dp <= 0)
        return fail(HH_ERR_INVALID_ARG, "n_micro, micro_batch, seq, hidden and data_parallel must be positive");
    if (!(flop >= 0.0)) return fail(HH_ERR_INVALID_ARG, "flop_per_layer must not be negative");
    return HH_OK;
}

}  // namespace

extern "C" int hh_sim_pipeline(const hh_sim_stage* stages, int n_stages, int n_micro, int micro_batch, int seq, int hidden,
                               int data_parallel, double flop_per_layer, hh_sim_result* out, double* stage_finish_ms,
                               uint64_t* stage_peak_bytes) {
    int rc = check_stages(stages, n_stages, true);
    if (rc != HH_OK) return rc;
    rc = check_run(n_micro, micro_batch, seq, hidden, data_parallel, flop_per_layer);
    if (rc != HH_OK) return rc;
    if (!out) return fail(HH_ERR_INVALID_ARG, "out is NULL");
    std::vector<int32_t> layers(n_stages);
    for (int p = 0; p < n_stages; p++) layers[p] = stages[p].n_layers;
    return simulate(stages, layers.data(), n_stages, n_micro, micro_batch, seq, hidden, data_parallel, flop_per_layer, out,
                    stage_finish_ms, stage_peak_bytes);
}

extern "C" int hh_sim_weighted_mean(const double* values, const int64_t* counts, int n, double* out) {
    if (!values || !counts || !out) return fail(HH_ERR_INVALID_ARG, "values / counts / out is NULL");
    if (n <= 0) return fail(HH_ERR_INVALID_ARG, "n must be positive");
    double num = 0.0, den = 0.0;
    for (int i = 0; i < n; i++) {
        if (counts[i] < 0) return fail(HH_ERR_INVALID_ARG, "counts must not be negative");
        num += values[i] * (double)counts[i];
        den += (double)counts[i];
    }
    if (den <= 0.0) return fail(HH_ERR_INVALID_ARG, "counts sum to zero");
    *out = num / den;
    return HH_OK;
}

extern "C" int hh_plan_layers(const hh_sim_stage* stages, int n_stages, int total_layers, int n_micro, int micro_batch, int seq,
                              int hidden, int data_parallel, double flop_per_layer, int slack, int32_t* layers_out,
                              hh_sim_result* best) {
    int rc = check_stages(stages, n_stages, false);
    if (rc != HH_OK) return rc;
    rc = check_run(n_micro, micro_batch, seq, hidden, data_parallel, flop_per_layer);
    if (rc != HH_OK) return rc;
    if (!layers_out || !best) return fail(HH_ERR_INVALID_ARG, "layers_out / best is NULL");
    if (total_layers < n_stages) return fail(HH_ERR_INVALID_ARG, "fewer layers than stages");
    if (slack < 0) return fail(HH_ERR_INVALID_ARG, "slack must not be negative");
    const int P = n_stages;
    // load balance (rule 1): layers in proportion to the stage's speed, 1 / (fwd + bwd time of a layer)
    std::vector<double> share(P);
    double speed_sum = 0.0;
    for (int p = 0; p < P; p++) speed_sum += 1.0 / (stages[p].fwd_ms + stages[p].bwd_ms);
    std::vector<int> lo(P), hi(P);
    for (int p = 0; p < P; p++) {
        share[p] = total_layers * (1.0 / (stages[p].fwd_ms + stages[p].bwd_ms)) / speed_sum;
        lo[p] = std::max(1, (int)std::floor(share[p]) - slack);
        hi[p] = std::min(total_layers - (P - 1), (int)std::ceil(share[p]) + slack);
    }
    // suffix bounds for pruning: what the remaining stages can still take
    std::vector<long> lo_suf(P + 1, 0), hi_suf(P + 1, 0);
    for (int p = P - 1; p >= 0; p--) { lo_suf[p] = lo_suf[p + 1] + lo[p]; hi_suf[p] = hi_suf[p + 1] + hi[p]; }
    std::vector<int32_t> cur(P), best_layers;
    std::vector<uint64_t> peak(P);
    hh_sim_result best_res{};
    bool found = false;
    long evaluated = 0;
    const long budget = 2000000;   // candidates costed before the search stops widening
    // depth-first over the per-stage counts (minimum end-to-end time, rule 2, decides between the leaves)
    struct Frame { int p; int next; long used; };
    std::vector<Frame> stack;
    stack.push_back({0, lo[0], 0});
    while (!stack.empty()) {
        Frame& f = stack.back();
        const int p = f.p;
        if (f.next > hi[p]) { stack.pop_back(); continue; }
        const int take = f.next++;
        const long used = f.used + take;
        const long rest = total_layers - used;
        if (p == P - 1) {
            if (rest != 0) continue;
            cur[p] = take;
            hh_sim_result r{};
            rc = simulate(stages, cur.data(), P, n_micro, micro_batch, seq, hidden, data_parallel, flop_per_layer, &r, nullptr,
                          peak.data());
            if (rc != HH_OK) return rc;
            evaluated++;
            bool fits = true;
            for (int q = 0; q < P; q++)
                if (stages[q].memory_bytes && peak[q] > stages[q].memory_bytes) fits = false;
            if (fits && (!found || r.iter_ms < best_res.iter_ms)) { best_res = r; best_layers = cur; found = true; }
            if (evaluated >= budget) break;
            continue;
        }
        if (rest < lo_suf[p + 1] || rest > hi_suf[p + 1]) continue;
        cur[p] = take;
        stack.push_back({p + 1, lo[p + 1], used});
    }
    if (!found) return fail(HH_ERR_UNSUPPORTED_SHAPE, "no layer split within the search range fits the stages' memory");
    for (int p = 0; p < P; p++) layers_out[p] = best_layers[p];
    *best = best_res;
    return HH_OK;
}

extern "C" int hh_plan_order(const hh_sim_stage* groups, const int32_t* counts, int n_groups, double cross_link_gbytes_per_s,
                             int total_layers, int n_micro, int micro_batch, int seq, int hidden, int data_parallel,
                             double flop_per_layer, int slack, int32_t* order_out, int32_t* layers_out, hh_sim_result* best) {
    if (!groups || !counts) return fail(HH_ERR_INVALID_ARG, "groups / counts is NULL");
    if (n_groups <= 0 || n_groups > 8) return fail(HH_ERR_INVALID_ARG, "n_groups must be in 1..8");
    if (!order_out || !layers_out || !best) return fail(HH_ERR_INVALID_ARG, "order_out / layers_out / best is NULL");
    long P = 0;
    for (int g = 0; g < n_groups; g++) {
        if (counts[g] <= 0) return fail(HH_ERR_INVALID_ARG, "counts must be positive");
        P += counts[g];
    }
    if (P > 4096) return fail(HH_ERR_INVALID_ARG, "more than 4096 stages");
    std::vector<int> perm(n_groups);
    for (int g = 0; g < n_groups; g++) perm[g] = g;
    std::vector<hh_sim_stage> st((size_t)P);
    std::vector<int32_t> layers((size_t)P), best_layers;
    std::vector<int> best_perm;
    hh_sim_result best_res{};
    bool found = false;
    int first_error = HH_OK;
    do {   // std::next_permutation walks the orders lexicographically, so the first of equal times is kept
        size_t at = 0;
        for (int k = 0; k < n_groups; k++) {
            const int g = perm[k];
            for (int c = 0; c < counts[g]; c++) {
                st[at] = groups[g];
                if (c == counts[g] - 1) st[at].link_gbytes_per_s = cross_link_gbytes_per_s;   // to the next group
                at++;
            }
        }
        hh_sim_result r{};
        const int rc = hh_plan_layers(st.data(), (int)P, total_layers, n_micro, micro_batch, seq, hidden, data_parallel,
                                      flop_per_layer, slack, layers.data(), &r);
        if (rc == HH_ERR_UNSUPPORTED_SHAPE) continue;   // this order does not fit in memory
        if (rc != HH_OK) { first_error = rc; break; }
        if (!found || r.iter_ms < best_res.iter_ms) { best_res = r; best_layers = layers; best_perm = perm; found = true; }
    } while (std::next_permutation(perm.begin(), perm.end()));
    if (first_error != HH_OK) return first_error;
    if (!found) return fail(HH_ERR_UNSUPPORTED_SHAPE, "no order of the groups has a layer split that fits the stages' memory");
    for (int k = 0; k < n_groups; k++) order_out[k] = best_perm[k];
    for (long q = 0; q < P; q++) layers_out[q] = best_layers[(size_t)q];
    *best = best_res;
    return HH_OK;
}
