/*
 * ferret_planner.h -- C ABI of libferret's pipeline planner (host only, no GPU call).
 *
 * Sec. "Model Partitioning and Pipeline Planning" of the paper: choose a partition L of the model's
 * layers into P contiguous stages and a pipeline configuration C = {c_n^d, c_n^r, c_{n,j}^a,
 * c_{n,j}^o} (per worker n: data delay or -1 if the worker is removed, activation recomputation flag;
 * per worker and stage j: gradient-accumulation steps and back-propagation-omission steps) that
 * maximise the adaptation rate R_F^T under a memory budget M (Eq. "objective").  The planner's result
 * is what the update path consumes: the stages, and per stage how many weight versions it keeps,
 * 1 + ceil((P-j-1)/c^a) - c^o, i.e. the ring depth and the maximum staleness to plan
 * ferret_plan_buckets with.
 *
 * Cost model (Eq. "ferret-svre"), for stage aggregates |w_i|, |a_i|, t^f, t^b (appendix "Notations"):
 *   R_F^T = sum over live workers n, stages i of  |w_i|/sum|w| * 1/c^a_{n,i} * sum_{j<c^a_{n,i}} A_{i,j}
 *   A_{i,j} = exp(-c((P+j) t^f + (P-i+j) t^b + c_n^r (P-i+j) t^f)) V_D
 *             / ( LCM{c^o_{n,k}+1 : k in [i,P-1]} * (t^f + t^b + c_n^r t^f) )
 *   M_F   = sum over live workers n, stages i of
 *             (1 + ceil((P-i-1)/c^a_{n,i}) - c^o_{n,i}) * (|w_i| + |a_i| - c_n^r * inner activations of stage i)
 * Search (Alg. 2 "Iterative Configuration Search"): N = ceil((t^f + t^b + c^r t^f)/t^d) workers, all
 * c^a = 1, c^o = 0; while M_F > M apply the applicable move among S2 (raise c^a_{n,j} to the next value
 * that lowers the stored-version count), S3 (c^a_{n,j} = 1, c^o_{n,j} = P-1-j) and S4 (remove worker n)
 * with the largest memory saved per rate lost; run with c^r = 0 and 1 and keep the better.
 * Planning (Alg. 3 "Brute-force planning"): for every candidate stage-time bound t^c (sums of
 * consecutive layers' t^f + t^b, at least the largest single layer) build the partition with the
 * fewest stages by greedy grouping, search it, keep the best rate.
 *
 * Where the printed formulas are garbled the readings are: worker sums run over all live workers; the
 * candidate bounds use t^f + t^b and are kept when >= the largest layer; S3 changes the rate of every
 * stage i <= j; S2 and S3 do not apply to the last stage; a move's memory and rate changes are those
 * of the cost model itself; ties go to the first move in the order worker, S2 < S3 < S4, stage; if no
 * move applies while over budget the search is infeasible (rate 0).
 *
 * All arrays are host memory owned by the caller; results are opaque objects freed with
 * ferret_pipeline_destroy.  Status codes and ferret_last_error() as in ferret.h.
 */
#ifndef FERRET_PLANNER_H
#define FERRET_PLANNER_H

#include "ferret.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Profile of one layer (the output of the paper's profile(theta)): forward and backward time, number
 * of parameters, number of output activations. */
typedef struct {
    double t_f;
    double t_b;
    double n_params;
    double n_acts;
} ferret_layer;

typedef struct ferret_pipeline ferret_pipeline;

/* Cost model on an explicit configuration.
 *   L          int32[n_stages+1], L[0] = 0 < L[1] < ... < L[n_stages] = n_layers
 *   delay      int32[n_workers] (c_n^d; < 0 = worker removed)      recompute  int32[n_workers] (0/1)
 *   accum      int32[n_workers*n_stages] row-major (c^a >= 1)       omit       same shape (c^o >= 0)
 *   c, v_d     decay constant of the data value and the initial data value V_D */
ferret_status ferret_pipeline_evaluate(const ferret_layer *layers, int32_t n_layers, const int32_t *L,
                                       int32_t n_stages, int32_t n_workers, const int32_t *delay,
                                       const int32_t *recompute, const int32_t *accum, const int32_t *omit,
                                       double c, double v_d, double *rate_out, double *memory_out);

/* Alg. 2 on a given partition: t_d = interval between data arrivals, memory_budget = M. */
ferret_status ferret_pipeline_search(const ferret_layer *layers, int32_t n_layers, const int32_t *L,
                                     int32_t n_stages, double t_d, double memory_budget, double c, double v_d,
                                     ferret_pipeline **out);

/* Alg. 3: partition and configuration with the best rate over all candidate stage-time bounds.
 * The distinct partitions are searched independently on up to 16 host threads (environment variable
 * FERRET_PLANNER_THREADS overrides the count); the winner is picked in bound order, so the result does
 * not depend on the number of threads. */
ferret_status ferret_pipeline_plan(const ferret_layer *layers, int32_t n_layers, double t_d,
                                   double memory_budget, double c, double v_d, ferret_pipeline **out);

void ferret_pipeline_destroy(ferret_pipeline *p);

/* Queries (-1 / 0 / NaN-free defaults on NULL or out-of-range indices). */
int32_t ferret_pipeline_feasible(const ferret_pipeline *p);          /* 1 if M_F <= M was reached */
int32_t ferret_pipeline_n_stages(const ferret_pipeline *p);          /* P */
int32_t ferret_pipeline_n_workers(const ferret_pipeline *p);         /* N before any removal */
int32_t ferret_pipeline_stage_begin(const ferret_pipeline *p, int32_t j);   /* L_j, j = 0..P */
double ferret_pipeline_rate(const ferret_pipeline *p);               /* R_F^T */
double ferret_pipeline_memory(const ferret_pipeline *p);             /* M_F */
double ferret_pipeline_stage_bound(const ferret_pipeline *p);        /* t^c that produced L (0 for search) */
int32_t ferret_pipeline_worker_delay(const ferret_pipeline *p, int32_t n);
int32_t ferret_pipeline_worker_recompute(const ferret_pipeline *p, int32_t n);
int32_t ferret_pipeline_worker_accum(const ferret_pipeline *p, int32_t n, int32_t j);
int32_t ferret_pipeline_worker_omit(const ferret_pipeline *p, int32_t n, int32_t j);
/* Weight versions stage j of worker n keeps: 1 + ceil((P-j-1)/c^a) - c^o. */
int32_t ferret_pipeline_stage_versions(const ferret_pipeline *p, int32_t n, int32_t j);
/* The moves the search applied, in order: kind 2/3/4 = S2/S3/S4, stage = -1 for S4. */
int32_t ferret_pipeline_n_moves(const ferret_pipeline *p);
ferret_status ferret_pipeline_move(const ferret_pipeline *p, int32_t k, int32_t *worker, int32_t *kind,
                                   int32_t *stage);

#ifdef __cplusplus
}
#endif
#endif /* FERRET_PLANNER_H */
