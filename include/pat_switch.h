/*
 * pat_switch.h -- C ABI of the latency predictor and the online switch decision
 * (host code in libpat_decode.so; no GPU work, no device memory).
 *
 * What it is: the consumer of the profile grid.  The paper's "Online Latency
 * Predictor" (Sec. 4.1) fits, per (TP degree, profiled batch size), a straight
 * line in the aggregate context tokens T to the profiled points and answers a
 * query (B, T) by evaluating the lines of the two nearest profiled batch sizes
 * and interpolating along the batch dimension.  The "Online Switch Strategy"
 * (Sec. 4.1, Algorithm 1) compares the remaining decode time under the current
 * TP degree with remaining time plus one-time switch cost under every candidate
 * and switches only for a strict gain.  The state-handling part of the switch
 * cost is min(T_move, T_recomp) of Sec. 4.2: Eq. (1)-(2) (valid KV bytes per
 * source rank over the one-way per-rank bandwidth) and Eq. (3)-(4) (profiled
 * prefill latency at the RMS context length).
 *
 * Conventions: all pointers are host memory; arrays are read during the call
 * only; times are microseconds unless a name says otherwise; every call returns
 * PAT_OK or a negative PAT_E* code of pat_decode.h and changes nothing on error.
 *
 * Choices where the paper is silent:
 *  - remaining time = sum over the l_max - l_gen steps left of the per-step
 *    latency with every unfinished sample running to l_max (T grows by B per
 *    step); DP groups run in lock step, so the slowest group counts;
 *  - merged batch of a target degree = ceil(sum of batches / (n_gpus / tp')),
 *    context tokens spread evenly likewise;
 *  - outside the profiled batch range the nearest profiled batch size is used
 *    alone, lines are extended in T;
 *  - candidates are visited in the given order and compared with strict "<";
 *  - prefill latencies are looked up piecewise linearly in the length between
 *    profiled lengths (ends extended), then linearly along the batch dimension;
 *    without a prefill table recomputation counts as unavailable.
 */
#ifndef PAT_SWITCH_H
#define PAT_SWITCH_H

#include <stdint.h>
#include "pat_decode.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pat_predictor pat_predictor;

/* Builds a predictor from measured grid rows (rows with skipped != 0 are ignored).
 * At least one measured row is required.  The rows may mix TP degrees. */
int pat_predictor_fit(const pat_grid_row *rows, int32_t n_rows, pat_predictor **out);
void pat_predictor_destroy(pat_predictor *p);

/* The fitted line of a profiled (tp, batch): latency_us = alpha + beta * T.
 * PAT_EINVAL if that pair was not profiled. */
int pat_predictor_line(const pat_predictor *p, int32_t tp, int32_t batch, double *alpha, double *beta);

/* Per-step decode latency l(B, T; TP) in microseconds.  PAT_EINVAL if nothing was
 * profiled for tp or batch < 1. */
int pat_predictor_query(const pat_predictor *p, int32_t tp, int32_t batch, double sum_context, double *latency_us);

/* pat_prefill_row, the profiled prefill latencies of the recomputation estimate, is declared in pat_decode.h
 * (pat_profile_prefill measures them). */

/* Everything one evaluation of Algorithm 1's loop body reads. */
typedef struct pat_switch_input {
    int32_t tp;                     /* current TP degree */
    const int32_t *tp_list;         /* candidate degrees, visited in this order */
    int32_t n_tp;
    int32_t n_gpus;                 /* fixed GPU budget: DP degree of a candidate = n_gpus / tp' */
    const int32_t *group_batch;     /* unfinished samples per current DP group [n_groups] */
    const double  *group_context;   /* aggregate context tokens per current DP group [n_groups] */
    int32_t n_groups;
    int32_t l_max, l_gen;           /* maximum response length, generated length so far */
    const int32_t *lengths;         /* context length of every unfinished sample [n_lengths] */
    int32_t n_lengths;
    int32_t n_layers, hidden, bytes_per_elem;   /* M, H, s of Eq. (1) */
    double  net_bytes_per_s;        /* one-way per-rank bandwidth of Eq. (2) */
    const double *fixed_us;         /* [n_tp][n_tp] measured fixed cost from tp_list[i] to tp_list[j]
                                       (weight resharding, group update, control); the current degree
                                       must be in tp_list */
    const pat_prefill_row *prefill; /* may be NULL.  Rows with latency_us < 0 (or NaN) are pairs the profiler
                                       did not measure and are ignored; a (tp, batch, length) measured twice is
                                       PAT_EINVAL; a degree left without measured rows has no recomputation estimate */
    int32_t n_prefill;
} pat_switch_input;

typedef struct pat_switch_decision {
    int32_t do_switch, tp_new;
    double  t_cur_us, t_best_us;
    /* per candidate, in tp_list order (caller provides n_tp entries each, or NULL) */
    double *t_rem_us, *t_switch_us, *t_total_us;
} pat_switch_decision;

int pat_switch_decide(const pat_predictor *p, const pat_switch_input *in, pat_switch_decision *out);

/* The offline profiler's sparse sampling plan (Sec. 4.1, "Offline Profiler"): one point per
 * (TP degree, batch size, context length) with
 *   - TP degrees 1, 2, 4, 8 up to n_gpus (TP stays inside a node; degrees are powers of two),
 *   - ten batch sizes spanning [1, 256],
 *   - context lengths from 8 to l_max (the paper's grid ends at 128K; a pool that holds less ends earlier),
 *   - a point kept only if batch * length <= t_cap, the deployment's active-token budget,
 *   - a denser ladder below 512 tokens, where the step latency bends.
 * The paper fixes these counts and bounds, not the values in between; this library takes
 *   batch sizes 1, 2, 4, 8, 16, 32, 64, 128, 192, 256 (the octaves, and the middle of the last one, where a
 *     rollout starts and spends its largest steps),
 *   lengths 8 * 2^i and, below 512 only, 12 * 2^i as well (two points per octave there, one above).
 * Points are written in (tp, batch, length) ascending order.  points may be NULL to ask for the count only;
 * otherwise *n_points holds its capacity on entry.  On return *n_points is the number of points of the plan.
 * PAT_EINVAL: a NULL n_points, n_gpus < 1, t_cap < 8, l_max < 8; PAT_ENOMEM: capacity too small (nothing
 * written).  Host only. */
typedef struct pat_plan_point {
    int32_t tp_degree, batch, kv_len, reserved;
} pat_plan_point;
int pat_profile_plan(int32_t n_gpus, int64_t t_cap, int64_t l_max, pat_plan_point *points, int32_t *n_points);

/* Eq. (1)-(2): seconds to move the valid KV states of the given samples. */
double pat_kv_move_seconds(const int32_t *lengths, int32_t n, int32_t n_layers, int32_t hidden, int32_t bytes_per_elem,
                           int32_t tp_src, double net_bytes_per_s);
/* Eq. (3). */
double pat_rms_length(const int32_t *lengths, int32_t n);

#ifdef __cplusplus
}
#endif
#endif
