/*
 * bapipe_plan.h - C ABI of the host-side planner that consumes the per-layer profile:
 * the pipeline-schedule cost model (paper Sec. III-B, Tables I and II) and the balanced
 * partition explorer (Sec. III-C: inter-layer partition seeded by Eq. (1), communication
 * bottleneck test with the coarse-grained merge by the feature threshold a_th, and the
 * memory fine-tune).  Pure host code: no device is touched, every pointer is host memory
 * owned by the caller, nothing is retained after a call returns.
 *
 * Every function returns a bapipe_status_t (bapipe_stage.h).  Outputs are written only on
 * BAPIPE_OK, except where stated.
 */
#ifndef BAPIPE_PLAN_H
#define BAPIPE_PLAN_H

#include "bapipe_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Pipeline schedules compared in Tables I and II. */
typedef enum {
    BAPIPE_PLAN_1F1B_AS = 0,  /* asynchronous execution, alternate F / B (Table I)               */
    BAPIPE_PLAN_FBP_AS = 1,   /* asynchronous execution, F and B in parallel (Table I)           */
    BAPIPE_PLAN_1F1B_SNO = 2, /* synchronous, communication not overlapped (Table II)            */
    BAPIPE_PLAN_1F1B_SO = 3   /* synchronous, doubled warm-up overlaps communication (Table II) */
} bapipe_schedule_t;

/* One column of Table I / II evaluated for stage i (1-based) of N with M micro-batches.
 * F, B: forward / backward time of a stage for one micro-batch (equal across stages under a
 * balanced partition); SR: time to send or receive one boundary tensor; a: bytes of the
 * features a stage keeps per in-flight micro-batch; w: bytes of its weights.  Times come
 * back in the unit of F, B, SR; memory in bytes; bandwidth in bytes per time unit. */
typedef struct {
    double minibatch_time;   /* "Mini-batch time"                                          */
    double bubble_fraction;  /* "Pipeline bubble"                                          */
    double features_memory;  /* "Features memory": in-flight micro-batches x a             */
    double weights_memory;   /* "Weights memory": 2 w (weights + gradient, no stashing)    */
    double bandwidth_demand; /* "Bandwidth": what hides the transfer behind compute        */
    int in_flight;           /* micro-batches stage i holds at once: min(M, features/a)    */
} bapipe_schedule_cost_t;

/* E_INVALID unless M >= 1, N >= 1, 1 <= i <= N, F > 0, B > 0, SR >= 0, a >= 0, w >= 0 and
 * schedule is one of the four. */
int bapipe_schedule_cost(int schedule, int M, int N, int i, double F, double B, double SR,
                         double a, double w, bapipe_schedule_cost_t *out);

/* One way of running a mini-batch that the planner may pick (Sec. III-B-2, last paragraph: the
 * schedule is chosen from the hardware limits, the profile and the partition).  A candidate is
 * a schedule together with the micro-batch split it would run at - doubling the warm-up
 * (1F1B-SO) doubles the features memory, so it may only fit with smaller, hence more and
 * possibly less efficient, micro-batches, whose F, B, SR and feature sizes come from a profile
 * taken at that micro-batch size. */
typedef struct {
    int schedule;         /* bapipe_schedule_t                                            */
    int n_micro;          /* M for this candidate                                         */
    double F, B, SR;      /* per micro-batch of this candidate's size, slowest stage      */
    const double *a;      /* [N] features bytes per in-flight micro-batch, per stage      */
} bapipe_schedule_candidate_t;

/* Among the candidates whose every stage i fits (in-flight x a[i] + 2 w[i] <= capacity[i];
 * capacity[i] <= 0 or capacity == NULL: unlimited) pick the one with the smallest mini-batch
 * time; ties go to the earlier candidate.  *best receives its index, *cost (optional) its cost
 * evaluated for stage 1.  BAPIPE_E_UNSUPPORTED if none fits, E_INVALID on bad arguments. */
int bapipe_schedule_choose(const bapipe_schedule_candidate_t *cand, int n_cand, int N, const double *w,
                           const double *capacity, int *best, bapipe_schedule_cost_t *cost);

/* Per-layer profile of the whole network as the explorer reads it (Sec. III-C-1: how many
 * accelerators there are and, for each kind of accelerator, every layer's forward and backward
 * time).  Arrays are indexed [acc * n_layers + layer] where marked per accelerator, else [layer]. */
typedef struct {
    int n_layers;
    int n_acc;                  /* accelerators = pipeline stages, in pipeline order           */
    const double *fwd_ms;       /* [n_acc][n_layers] forward time of one micro-batch           */
    const double *bwd_ms;       /* [n_acc][n_layers] backward time of one micro-batch          */
    const double *out_bytes;    /* [n_layers] bytes of the layer's output for one micro-batch  */
    const double *weight_bytes; /* [n_layers]                                                  */
    const double *stash_bytes;  /* [n_layers] bytes the layer keeps per in-flight micro-batch  */
    const double *mem_capacity; /* [n_acc] bytes available for weights + features, <= 0: unlimited */
    double link_bytes_per_ms;   /* bandwidth between neighbouring accelerators, <= 0: unlimited */
    int n_micro;                /* M                                                           */
    int schedule;               /* bapipe_schedule_t used for in-flight counts and bandwidth   */
} bapipe_plan_input_t;

typedef struct {
    double ideal_stage_ms;       /* T of Eq. (1) from the whole-network times T_n              */
    double seed_bottleneck_ms;   /* slowest stage of the partition seeded by T and iterated    */
    double bottleneck_ms;        /* slowest stage (F + B of one micro-batch) of the result     */
    double a_th_bytes;           /* feature threshold used for the coarse-grained merge, or 0  */
    int comm_bottleneck;         /* 1: the balanced partition needed more bandwidth than the link has */
    int memory_tuned;            /* 1: the partition was moved to fit mem_capacity             */
} bapipe_plan_report_t;

/* Balanced partition (Sec. III-C).  stage_begin: caller's array of n_acc + 1 ints; on BAPIPE_OK
 * stage n (0-based) owns layers [stage_begin[n], stage_begin[n+1]), every stage at least one.
 * Steps, in the paper's order:
 *  1. inter-layer partition: T of Eq. (1); boundaries placed where the running time on each
 *     accelerator reaches T, then moved one layer at a time while the slowest stage gets
 *     faster (report->seed_bottleneck_ms); the result is then replaced by the contiguous
 *     partition with the smallest slowest stage (exact, dynamic programming) if that is better;
 *  2. communication test with the schedule's "Bandwidth" row; if some boundary needs more
 *     than link_bytes_per_ms, boundaries are restricted to layers whose output is at most
 *     a_th = T x link_bytes_per_ms and step 1 is repeated on that coarse-grained network;
 *  3. memory fine-tune: if a stage needs more than its mem_capacity (2 x weights + in-flight
 *     micro-batches x stash), the best partition among those that fit is taken.
 * BAPIPE_E_UNSUPPORTED if no partition satisfies the constraints (report is still written),
 * BAPIPE_E_INVALID on bad arguments (n_acc > n_layers, NULL arrays, negative times). */
int bapipe_partition(const bapipe_plan_input_t *in, int *stage_begin, bapipe_plan_report_t *report);

#ifdef __cplusplus
}
#endif
#endif /* BAPIPE_PLAN_H */
