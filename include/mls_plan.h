/* mls_plan.h -- the lower level of the parallelization planner: how many layers each pipeline stage gets and how
 * many micro-batches each pipeline gets, from the measured per-layer time tau(b) and the group straggling rates.
 *
 * These are the two integer programs of Sec. 4.2 ("Deriving the Assignments"): the joint problem (Eq. 1) splits
 * into one layer-split problem per pipeline (Eq. 2) and one micro-batch-split problem over the pipelines (Eq. 3).
 * Both are min-max problems over non-negative integers with one sum constraint, solved here exactly by searching
 * the smallest feasible bottleneck value among the finitely many candidates rate x count.  Also: the constant-time
 * comparison of two GPU groupings (Theorem 2, Sec. 4.3.1) and the theoretic optimum of Sec. 7.2.
 *
 * Host code only: all pointers are HOST pointers; nothing here touches the GPU.  The functions are pure (no
 * global state except the error text of mls_last_error) and may be called from any thread.
 * Every function returns 0 (MLS_OK) or a negative MLS_E_* code of mls.h; outputs are untouched on error.
 */
#ifndef MLS_PLAN_H
#define MLS_PLAN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Eq. 2: split L layers over the n stages of one pipeline.
 *   y[n]    group straggling rate of each stage's GPU group (y = rho_n * max x, Sec. 4.2), finite and > 0
 *   cap[n]  most layers stage j can hold, i.e. floor((C_j - nu_j(b)) / mu_j(b)) of the linear memory model; a
 *           negative entry, or cap == NULL, means no limit
 *   l[n]    (out) layers per stage, non-negative, sum L, minimising max_j y[j]*l[j]; stages whose rate is too
 *           high get 0 layers.  Among the optimal splits the one returned also has the smallest sum_j y[j]*l[j]
 *           (the warm-up / cool-down term of the pipeline time model of Sec. 4.2): the fastest stages are filled
 *           first, the earlier of two equally fast stages first.
 *   o       (out, may be NULL) the optimal value max_j y[j]*l[j]
 * MLS_E_RANGE if the caps cannot hold L layers; MLS_E_CONFIG for n < 1, L < 0 or a bad rate. */
int mls_plan_layers(const double* y, const int64_t* cap, int32_t n, int64_t L, int64_t* l, double* o);

/* Eq. 3: split n_mb = B / b micro-batches over dp pipelines.
 *   o[dp]   per-micro-batch bottleneck of each pipeline (the optimal values of Eq. 2), finite and > 0
 *   m[dp]   (out) micro-batches per pipeline, non-negative, sum n_mb, minimising max_i o[i]*m[i] (same tie rule)
 *   t       (out, may be NULL) the optimal value max_i o[i]*m[i]; times tau(b) it is the estimated step time */
int mls_plan_microbatches(const double* o, int32_t dp, int64_t n_mb, int64_t* m, double* t);

/* Eq. 1 for a given orchestration: dp pipelines, pipeline i has pp[i] stages; y and cap list the stages of
 * pipeline 0, then pipeline 1, ... (sum pp[i] entries; cap may be NULL).  Writes l (same order), m[dp] and the
 * estimated step time  tau * max_i m[i] * max_j y[i,j]*l[i,j]  (the simplified time model of Sec. 4.2). */
int mls_plan_lower_level(const double* y, const int64_t* cap, const int32_t* pp, int32_t dp, int64_t L, int64_t n_mb,
                         double tau, int64_t* l, int64_t* m, double* step_time);

/* Appendix B.4: the most layers stage j (1-based) of a 1F1B pipeline with pp stages can hold under the linear
 * memory model l * mu + nu <= capacity - reserve, where the stage keeps the forward activations of pp - j earlier
 * micro-batches beside the one in flight:  mu = a_f * (pp - j) + a_fb + s.
 *   a_f   bytes of forward activations kept per layer for one micro-batch (of the micro-batch size in use)
 *   a_fb  peak activation bytes per layer while one micro-batch runs forward and backward
 *   s     bytes of parameters, gradients and optimizer states per layer
 *   nu    bytes that do not grow with the layer count (workspace; first / last stage: the non-uniform layers)
 * Returns floor((capacity - reserve - nu) / mu), at least 0; -1 on bad input (pp < 1, j outside [1, pp], mu <= 0). */
int64_t mls_plan_layer_cap(double a_f, double a_fb, double s, double nu, int32_t pp, int32_t j, double capacity,
                           double reserve);

/* Theorem 2: T'/T'' of two groupings with group rates y1[n1] and y2[n2] under the relaxed problem (no memory
 * limit, real-valued assignments) = (sum 1/y2) / (sum 1/y1).  NaN on bad input. */
double mls_grouping_time_ratio(const double* y1, int32_t n1, const double* y2, int32_t n2);

/* Group splitting (Sec. 4.3.1; Appendix B.7): n GPUs of one node with straggling rates x[n] are to form k groups of
 * sizes[k] GPUs (sum of sizes = n), e.g. the 7 GPUs left after isolating a heavy straggler into groups of 1, 2, 4.
 * By the appendix's proposition an optimal grouping puts GPUs that are consecutive in the order of their rates into
 * the same group, so the candidates are: sort by rate, cut into consecutive runs, one run per group, for every
 * order of the groups along the sorted list (6 candidates for sizes 1, 2, 4).  The rate of a group is
 * y = rho[g] * max x over its members (rho[g]: the efficiency coefficient rho_n of a group of sizes[g] GPUs,
 * Sec. 4.2); the candidate with the largest sum of 1/y wins (Theorem 2: training time is proportional to the
 * inverse of that sum).  Ties: the candidate that comes first when the orders of the groups are enumerated
 * lexicographically.
 *   group_of[n]  (out) index into sizes[] of the group each GPU joins
 *   inv_sum      (out, may be NULL) sum over the groups of 1 / y for the winner
 * k <= 8.  MLS_E_CONFIG on bad sizes or rates. */
int mls_plan_split_groups(const double* x, int32_t n, const int32_t* sizes, const double* rho, int32_t k,
                          int32_t* group_of, double* inv_sum);

/* Sec. 7.2: best possible ratio of the step time with stragglers to the step time without, for N GPUs of which n
 * straggle with rates x[n]: N / ((N - n) + sum 1/x).  NaN on bad input. */
double mls_theoretic_slowdown(int64_t N, const double* x, int32_t n);

#ifdef __cplusplus
}
#endif
#endif
