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
    out->search_truncated = 0;
    out->reserved_ = 0;
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
    bool truncated = false;
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
            if (evaluated >= budget) { truncated = true; break; }
            continue;
        }
        if (rest < lo_suf[p + 1] || rest > hi_suf[p + 1]) continue;
        cur[p] = take;
        stack.push_back({p + 1, lo[p + 1], used});
    }
    if (!found) return fail(HH_ERR_UNSUPPORTED_SHAPE, "no layer split within the search range fits the stages' memory");
    for (int p = 0; p < P; p++) layers_out[p] = best_layers[p];
    *best = best_res;
    best->search_truncated = truncated ? 1 : 0;
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
    bool found = false, any_truncated = false;
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
        any_truncated = any_truncated || r.search_truncated;
        if (!found || r.iter_ms < best_res.iter_ms) { best_res = r; best_layers = layers; best_perm = perm; found = true; }
    } while (std::next_permutation(perm.begin(), perm.end()));
    if (first_error != HH_OK) return first_error;
    if (!found) return fail(HH_ERR_UNSUPPORTED_SHAPE, "no order of the groups has a layer split that fits the stages' memory");
    for (int k = 0; k < n_groups; k++) order_out[k] = best_perm[k];
    for (long q = 0; q < P; q++) layers_out[q] = best_layers[(size_t)q];
    *best = best_res;
    best->search_truncated = any_truncated ? 1 : 0;   // some order's split search stopped at its budget
    return HH_OK;
}

// ---------------------------------------------------------------------------------------------------------------
// The whole search tree of the automatic parallel planner (Section 3.3): data-parallel degree (level 2), one
// tensor-parallel degree per accelerator type (level 3), and under every such leaf the pipeline level (stage order
// and layer split, hh_plan_order).
namespace {

struct ClusterSearch {
    const hh_cluster_group* groups;
    int n_groups;
    double cross;
    int total_layers, micro_batch, seq, hidden, slack;
    double flop_per_layer;
    int d, n_micro;                 // current data-parallel degree and micro-batches per replica
    int tp_idx[8];                  // current tensor-parallel degree index per group
    bool found = false;
    int error = HH_OK;
    hh_cluster_plan best{};
    std::vector<int32_t> best_layers;
    int costed = 0;
    bool truncated = false;

    void leaf() {
        std::vector<hh_sim_stage> g((size_t)n_groups);
        std::vector<int32_t> counts((size_t)n_groups);
        long P = 0;
        for (int i = 0; i < n_groups; i++) {
            const hh_cluster_group& c = groups[i];
            const int t = 1 << tp_idx[i];
            const long devices = (long)c.n_nodes * c.devices_per_node;
            if (devices % ((long)d * t)) return;           // every accelerator is used
            counts[i] = (int32_t)(devices / ((long)d * t));
            if (counts[i] < 1) return;
            P += counts[i];
            hh_sim_stage& s = g[i];
            s.n_layers = 0;
            s.n_devices = d * t;
            s.fwd_ms = c.fwd_ms_tp[tp_idx[i]];
            s.bwd_ms = c.bwd_ms_tp[tp_idx[i]];
            s.peak_tflops = c.peak_tflops;
            s.link_gbytes_per_s = c.link_gbytes_per_s;
            s.weight_bytes = c.weight_bytes / (uint64_t)t;
            s.grad_bytes = c.grad_bytes / (uint64_t)t;
            s.optimizer_bytes = c.optimizer_bytes / (uint64_t)t;
            s.saved_act_bytes = c.saved_act_bytes_tp[tp_idx[i]];
            s.memory_bytes = c.memory_bytes;
        }
        if (P > total_layers || P > 4096) return;
        std::vector<int32_t> order((size_t)n_groups), layers((size_t)P);
        hh_sim_result r{};
        const int rc = hh_plan_order(g.data(), counts.data(), n_groups, cross, total_layers, n_micro, micro_batch, seq, hidden, d,
                                     flop_per_layer, slack, order.data(), layers.data(), &r);
        if (rc == HH_ERR_UNSUPPORTED_SHAPE) return;   // nothing fits in memory under this leaf
        if (rc != HH_OK) { error = rc; return; }
        costed++;
        truncated = truncated || r.search_truncated;
        // gradient all-reduce between the d replicas of a stage (ring: 2 (d-1)/d of the stage's fp32 gradient shard)
        double ar = 0.0;
        size_t at = 0;
        for (int k = 0; k < n_groups; k++) {
            const int gi = order[k];
            const hh_cluster_group& c = groups[gi];
            const int t = 1 << tp_idx[gi];
            for (int q = 0; q < counts[gi]; q++, at++) {
                if (d > 1 && c.dp_gbytes_per_s > 0.0) {
                    const double bytes = 2.0 * (d - 1) / d * ((double)c.grad_bytes / t) * layers[at];
                    ar = std::max(ar, bytes / (c.dp_gbytes_per_s * 1e9) * 1e3);
                }
            }
        }
        const double iter = r.iter_ms + ar;
        if (found && !(iter < best.sim.iter_ms)) return;
        hh_cluster_plan p{};
        p.data_parallel = d;
        for (int i = 0; i < n_groups; i++) { p.tensor_parallel[i] = 1 << tp_idx[i]; p.stages[i] = counts[i]; p.order[i] = order[i]; }
        p.n_stages = (int32_t)P;
        p.n_micro = n_micro;
        p.pipeline_ms = r.iter_ms;
        p.grad_allreduce_ms = ar;
        p.sim = r;
        const double scale = r.iter_ms / iter;          // the same work in a longer iteration
        p.sim.iter_ms = iter;
        p.sim.bubble_fraction = 1.0 - (1.0 - r.bubble_fraction) * scale;
        p.sim.tokens_per_s_per_device = r.tokens_per_s_per_device * scale;
        p.sim.tflops_per_device = r.tflops_per_device * scale;
        p.sim.mfu = r.mfu * scale;
        best = p;
        best_layers = layers;
        found = true;
    }

    void descend(int gi) {
        if (error != HH_OK) return;
        if (gi == n_groups) { leaf(); return; }
        for (int i = 0; i < 4; i++) {
            const int t = 1 << i;
            if (groups[gi].devices_per_node % t) continue;                       // tensor parallelism stays inside a node
            if (!(groups[gi].fwd_ms_tp[i] > 0.0) || !(groups[gi].bwd_ms_tp[i] > 0.0)) continue;   // not profiled
            tp_idx[gi] = i;
            descend(gi + 1);
        }
    }
};

}  // namespace

extern "C" int hh_plan_cluster(const hh_cluster_group* groups, int n_groups, double cross_link_gbytes_per_s, int total_layers,
                               int global_batch, int micro_batch, int seq, int hidden, double flop_per_layer, int slack,
                               hh_cluster_plan* plan, int32_t* layers_out, int max_stages) {
    if (!groups || !plan || !layers_out) return fail(HH_ERR_INVALID_ARG, "groups / plan / layers_out is NULL");
    if (n_groups <= 0 || n_groups > 8) return fail(HH_ERR_INVALID_ARG, "n_groups must be in 1..8");
    if (total_layers <= 0 || global_batch <= 0 || micro_batch <= 0 || seq <= 0 || hidden <= 0)
        return fail(HH_ERR_INVALID_ARG, "total_layers, global_batch, micro_batch, seq and hidden must be positive");
    if (!(flop_per_layer >= 0.0)) return fail(HH_ERR_INVALID_ARG, "flop_per_layer must not be negative");
    if (slack < 0) return fail(HH_ERR_INVALID_ARG, "slack must not be negative");
    if (max_stages <= 0) return fail(HH_ERR_INVALID_ARG, "max_stages must be positive");
    long max_devices = 0;
    for (int g = 0; g < n_groups; g++) {
        if (groups[g].n_nodes <= 0 || groups[g].devices_per_node <= 0) return fail(HH_ERR_INVALID_ARG, "every group needs nodes and devices");
        if (!(groups[g].peak_tflops > 0.0)) return fail(HH_ERR_INVALID_ARG, "peak_tflops must be positive");
        max_devices = std::max(max_devices, (long)groups[g].n_nodes * groups[g].devices_per_node);
    }
    ClusterSearch s{};
    s.groups = groups; s.n_groups = n_groups; s.cross = cross_link_gbytes_per_s; s.total_layers = total_layers;
    s.micro_batch = micro_batch; s.seq = seq; s.hidden = hidden; s.slack = slack; s.flop_per_layer = flop_per_layer;
    for (int d = 1; d <= max_devices && s.error == HH_OK; d++) {      // level 2, then level 3 below it, depth first
        if (global_batch % ((long)d * micro_batch)) continue;
        s.d = d;
        s.n_micro = global_batch / (d * micro_batch);
        if (s.n_micro < 1) continue;
        s.descend(0);
    }
    if (s.error != HH_OK) return s.error;
    if (!s.found) return fail(HH_ERR_UNSUPPORTED_SHAPE, "no parallel strategy of the search tree is feasible for this cluster");
    if (s.best.n_stages > max_stages) return fail(HH_ERR_INVALID_ARG, "layers_out is shorter than the best plan's pipeline");
    s.best.strategies_costed = s.costed;
    s.best.sim.search_truncated = s.truncated ? 1 : 0;
    *plan = s.best;
    for (int q = 0; q < s.best.n_stages; q++) layers_out[q] = s.best_layers[(size_t)q];
    return HH_OK;
}
