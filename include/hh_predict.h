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
 * HH_ERR_UNSUPPORTED_SHAPE when no candidate fits in memory. */
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

#ifdef __cplusplus
}
#endif
#endif
