/* hh_predict.h -- host-side performance predictor for a pipeline of stages
 * (the workload simulator of Section 3.2 and the layer split of the automatic
 * parallel planner, Section 3.3).  It consumes what hh_layer_profile measures
 * per accelerator type.  Pure host arithmetic: no GPU, no allocation visible to
 * the caller, no global state.  Every function returns HH_OK or a negative
 * hh_status (see hh.h); hh_last_error() describes the failure.
 */
#ifndef HH_PREDICT_H
#define HH_PREDICT_H

#include <stdint.h>
#include "hh.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One pipeline stage.  Per-layer figures are those of one hh_profile_rec of the
 * accelerator type that runs the stage. */
typedef struct {
    int32_t n_layers;            /* layers on this stage (non-uniform split, Section 3.3) */
    int32_t n_devices;           /* accelerators running this stage = data-parallel x tensor-parallel degree */
    double fwd_ms, bwd_ms;       /* one layer, one micro-batch */
    double peak_tflops;          /* of one accelerator of this type (Eq. 2) */
    double link_gbytes_per_s;    /* to the next stage, in 1e9 bytes/s; <= 0: free; ignored on the last stage */
    uint64_t weight_bytes;       /* per layer */
    uint64_t grad_bytes;         /* per layer */
    uint64_t optimizer_bytes;    /* per layer (optimizer state kept on the stage) */
    uint64_t saved_act_bytes;    /* per layer and live micro-batch */
    uint64_t memory_bytes;       /* capacity of one accelerator; 0: not checked by hh_plan_layers */
} hh_sim_stage;

typedef struct {
    double iter_ms;                    /* time of one iteration: last backward of any stage */
    double bubble_fraction;            /* 1 - (busy time of the busiest stage) / iter_ms */
    double tokens_per_s_per_device;    /* Eq. (1): seq * global_batch / (devices * iteration time) */
    double tflops_per_device;          /* model flops of the iteration / time / devices */
    double mean_peak_tflops;           /* mean over all devices (Section 4.3: the mixed cluster's peak) */
    double mfu;                        /* Eq. (2): tflops_per_device / mean_peak_tflops */
    int64_t n_devices;
    int32_t search_truncated;          /* planners only: 1 when the depth-first search stopped at its budget of costed
                                          candidates, so a better split inside the search range may exist; 0 otherwise */
    int32_t reserved_;
} hh_sim_result;

/* Simulates one training iteration of n_micro micro-batches through the stages in
 * PipeDream-1F1B order (Sections 2.3, 3.3): stage p runs forward of the first
 * min(n_micro, n_stages - p) micro-batches, then alternates one backward and one
 * forward; an operation starts when its stage is free and its input has arrived,
 * the boundary tensor of Eq. (3), micro_batch*seq*hidden*2 bytes, taking
 * bytes / link speed.  data_parallel replicas run the same schedule side by side
 * (global batch = n_micro * micro_batch * data_parallel).  flop_per_layer: model
 * flops of one layer on one micro-batch, forward + backward.
 * stage_finish_ms, stage_peak_bytes: optional arrays of n_stages (HOST):
 * finish time of each stage, and weights + gradients + optimizer state of its
 * layers plus the saved activations of its live micro-batches. */
int hh_sim_pipeline(const hh_sim_stage *stages, int n_stages, int n_micro, int micro_batch, int seq,
                    int hidden, int data_parallel, double flop_per_layer, hh_sim_result *out,
                    double *stage_finish_ms, uint64_t *stage_peak_bytes);

/* Mean of values[i] weighted by counts[i] (Section 4.3: the theoretical upper
 * bound of a heterogeneous cluster is the mean over all its accelerators). */
int hh_sim_weighted_mean(const double *values, const int64_t *counts, int n, double *out);

/* Layer split of the automatic parallel planner (Section 3.3, first level of
 * the search tree): distributes total_layers over the stages (n_layers of the
 * input is ignored), depth-first over the per-stage counts, every candidate
 * costed by hh_sim_pipeline; keeps the split with the shortest iteration whose
 * stage_peak_bytes fit memory_bytes (where given).  Candidates are limited to
 * `slack` layers around the load-balanced share (layers proportional to stage
 * speed); every stage gets at least one layer.  layers_out: n_stages (HOST).
 * At most 2,000,000 candidates are costed; when the search range holds more, the best of those visited is returned
 * with best->search_truncated = 1.  HH_ERR_UNSUPPORTED_SHAPE when no candidate fits in memory. */
int hh_plan_layers(const hh_sim_stage *stages, int n_stages, int total_layers, int n_micro,
                   int micro_batch, int seq, int hidden, int data_parallel, double flop_per_layer,
                   int slack, int32_t *layers_out, hh_sim_result *best);

/* Stage order of the automatic parallel planner (Section 3.3, second rule: the stages are scheduled onto the
 * accelerator types so that the end-to-end time is smallest, given the stage times on each type and the
 * communication time between stages).  groups[g] describes the counts[g] identical stages that the nodes of one
 * accelerator type form (per-layer figures as for hh_plan_layers; its link_gbytes_per_s is the link between two
 * neighbouring stages of that group); two neighbouring stages of different groups are joined by a link of
 * cross_link_gbytes_per_s.  A group stays contiguous in the pipeline.  Every order of the groups is tried, the
 * layers are split for each with hh_plan_layers (same slack, same memory rule) and the order with the shortest
 * iteration is kept; among equal times the first in lexicographic order of group indices.  n_groups <= 8.
 * order_out: n_groups group indices in pipeline order; layers_out: one count per stage in pipeline order
 * (sum of counts entries); both HOST.  HH_ERR_UNSUPPORTED_SHAPE when no order has a split that fits in memory. */
int hh_plan_order(const hh_sim_stage *groups, const int32_t *counts, int n_groups, double cross_link_gbytes_per_s,
                  int total_layers, int n_micro, int micro_batch, int seq, int hidden, int data_parallel,
                  double flop_per_layer, int slack, int32_t *order_out, int32_t *layers_out, hh_sim_result *best);

/* One accelerator type of a heterogeneous cluster, as the strategy generator of Section 3.2 samples it: the
 * measured layer times of that type at every tensor-parallel degree it may use, its memory and its links.
 * Index i of the *_tp arrays is tensor-parallel degree 2^i (1, 2, 4, 8); fwd_ms_tp[i] <= 0 marks a degree that
 * was not profiled and is not searched.  The times are those of one layer on one micro-batch at that degree's
 * share shape, the tensor-parallel all-reduces included (hh_layer_profile measures the compute of a share). */
typedef struct {
    int32_t n_nodes;             /* homogeneous nodes of this type */
    int32_t devices_per_node;    /* tensor parallelism stays inside a node: its degree divides this */
    double fwd_ms_tp[4], bwd_ms_tp[4];
    uint64_t saved_act_bytes_tp[4];   /* per layer, live micro-batch and device */
    double peak_tflops;          /* of one accelerator (Eq. 2) */
    double link_gbytes_per_s;    /* between neighbouring pipeline stages of this type; <= 0: free */
    double dp_gbytes_per_s;      /* per device, between data-parallel replicas of this type; <= 0: free */
    uint64_t weight_bytes;       /* per layer, whole layer (divided by the tensor-parallel degree per device) */
    uint64_t grad_bytes;         /* per layer, whole layer */
    uint64_t optimizer_bytes;    /* per layer, whole layer */
    uint64_t memory_bytes;       /* capacity of one accelerator; 0: not checked */
} hh_cluster_group;

typedef struct {
    int32_t data_parallel;       /* level 2 of the search tree: replicas, the same for every stage */
    int32_t tensor_parallel[8];  /* level 3: degree used by each group (input order) */
    int32_t stages[8];           /* pipeline stages formed by each group (input order) */
    int32_t order[8];            /* level 1: group index per pipeline position */
    int32_t n_stages;            /* sum of stages[] */
    int32_t n_micro;             /* micro-batches per replica and iteration */
    int32_t strategies_costed;   /* (data-parallel, tensor-parallel) leaves handed to the simulator */
    double pipeline_ms;          /* 1F1B iteration of one replica */
    double grad_allreduce_ms;    /* slowest stage's gradient all-reduce between replicas, added after the pipeline */
    hh_sim_result sim;           /* metrics of the whole iteration (iter_ms = pipeline_ms + grad_allreduce_ms) */
} hh_cluster_plan;

/* The automatic parallel planner over its whole three-level search tree (Section 3.3).  Root: the model of
 * total_layers layers trained on global_batch samples per iteration in micro-batches of micro_batch samples.
 * Level 1 cuts it into pipeline stages of unequal layer counts, ordered over the accelerator types
 * (hh_plan_order: both rules); level 2 replicates every stage data_parallel times over homogeneous nodes (uniform);
 * level 3 splits a stage over tensor_parallel[g] accelerators inside a node (uniform per type).  Every accelerator
 * is used: group g forms n_nodes*devices_per_node / (data_parallel * tensor_parallel[g]) stages, and only degrees
 * for which this is a positive whole number, micro-batches per replica = global_batch / (data_parallel *
 * micro_batch) is a positive whole number and the degree was profiled are visited.  The tree is walked depth-first
 * (data-parallel degree, then one tensor-parallel degree per group); every leaf is costed by the workload
 * simulator with its best stage order and layer split, plus the time of the ring all-reduce of the fp32 gradients
 * between the replicas of the slowest stage, 2 (d-1)/d * grad_bytes * layers / tensor_parallel / dp_gbytes_per_s.
 * Per-device memory of a stage: (weights + gradients + optimizer state) / tensor_parallel per layer, plus the saved
 * activations of its live micro-batches.  The cheapest leaf wins, the first found among equals (ascending
 * data-parallel degree, then ascending tensor-parallel degrees, group 0 varying slowest).  n_groups <= 8.
 * layers_out: one count per stage in pipeline order, at least max_stages entries (HOST); the call fails with
 * HH_ERR_INVALID_ARG when the best plan has more stages than that, and with HH_ERR_UNSUPPORTED_SHAPE when no leaf
 * of the tree is feasible. */
int hh_plan_cluster(const hh_cluster_group *groups, int n_groups, double cross_link_gbytes_per_s, int total_layers,
                    int global_batch, int micro_batch, int seq, int hidden, double flop_per_layer, int slack,
                    hh_cluster_plan *plan, int32_t *layers_out, int max_stages);

#ifdef __cplusplus
}
#endif
#endif
