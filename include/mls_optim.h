/* mls_optim.h -- what one GPU does between two steps: the optimizer update of the parameters it holds, and the
 * straggling-rate probe that tells the planner when to re-plan.
 *
 * Optimizer.  The paper shards the model states with the ZeRO-1 optimizer (Sec. 5.1) and does not spell the update
 * rule out; this is the single-GPU part of it for the usual choice, AdamW on fp32 master weights: the handle owns
 * the fp32 master copy and the two moment vectors of the n parameters it is created for (a stage's, or the
 * first/last-stage layers', in their public layout), takes the fp32 gradients the backward calls accumulated, and
 * writes the updated parameters in the storage type for mls_stage_set_params / mls_ends_set_params:
 *     g = grad_scale * grads                    (e.g. 1 / number of micro-batches, or the loss-scale inverse)
 *     m = beta1 m + (1 - beta1) g;   v = beta2 v + (1 - beta2) g^2
 *     w = w - lr * ( (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps) + weight_decay * w ),   t = 1, 2, ...
 *     params_out = w rounded once to the storage type
 * One HBM-bound kernel: 28 B read + 12 B (+ 2 or 4 B) written per parameter.
 *
 * Probe.  The profiler of Sec. 3 measures the running time of each GPU, turns it into a straggling rate by
 * comparing with the non-stragglers, and notifies the planner when a rate changes by more than 5 % between two
 * consecutive iterations.  mls_probe is that logic for one GPU: it brackets a step with HIP events on the
 * caller's stream, converts the elapsed time into tau = time / (layers x micro-batches) (the cost model's unit,
 * Sec. 4.2), and reports x = tau / tau_ref and whether x moved by more than the threshold since the last step.
 *
 * Conventions as in mls.h: int functions return 0 or a negative MLS_E_* code; device pointers are 16-byte aligned
 * and owned by the caller; nothing is allocated after init.
 */
#ifndef MLS_OPTIM_H
#define MLS_OPTIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mls_optim mls_optim;

typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
} mls_adamw;

/* n parameters of storage type `dtype` (MLS_BF16 / MLS_FP32); `params` (device, n elements of that type) gives the
 * initial values of the fp32 master copy; the moments start at zero.  Multiples of 8 parameters only. */
int mls_optim_init(size_t n, const void* params, int32_t dtype, void* hip_stream, mls_optim** out);
void mls_optim_free(mls_optim* o);
/* One AdamW step (enqueued on the stream; no synchronisation).  grads: device fp32 [n], not modified;
 * params_out: device [n] in the storage type (may be the buffer given at init). */
int mls_optim_step(mls_optim* o, const float* grads, const mls_adamw* hp, float grad_scale, void* params_out);
int64_t mls_optim_steps(const mls_optim* o); /* t: steps taken so far */
/* copy of the master weights (which = 0), first (1) or second (2) moments: device fp32 [n]; synchronises */
int mls_optim_read(mls_optim* o, int32_t which, float* dst);

typedef struct mls_probe mls_probe;

/* tau_ref_ms: per-layer per-micro-batch time of a non-straggling GPU (profiled in advance, e.g. by bench.py);
 * threshold: relative change of the straggling rate that counts as a shift (the paper uses 0.05). */
int mls_probe_init(double tau_ref_ms, double threshold, void* hip_stream, mls_probe** out);
void mls_probe_free(mls_probe* p);
/* Record the start / the end of a step on the stream (no synchronisation). */
int mls_probe_begin(mls_probe* p);
int mls_probe_end(mls_probe* p, int32_t layers, int32_t microbatches);
/* Wait for the end event of the last bracketed step; *rate = straggling rate x of that step, *tau_ms its measured
 * per-unit time, *shift = 1 if |x - x_prev| / x_prev exceeds the threshold (0 for the first step).  Either output
 * may be NULL.  MLS_E_RANGE if no step has been bracketed or layers x micro-batches was 0. */
int mls_probe_read(mls_probe* p, double* rate, double* tau_ms, int32_t* shift);
/* The same decision from a given elapsed time instead of events (host only; for replaying traces). */
int mls_probe_feed(mls_probe* p, double elapsed_ms, int32_t layers, int32_t microbatches, double* rate, int32_t* shift);

#ifdef __cplusplus
}
#endif
#endif
