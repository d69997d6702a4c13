/* mls_ends.h -- the non-uniform layers of the first and the last pipeline stage: token embedding in front of the
 * first decoder layer; final RMSNorm, LM head and mean cross-entropy loss behind the last one.
 *
 * Appendix B.4 of the paper (memory model of a 1F1B pipeline) separates a model into uniform layers, which every
 * stage holds l_{i,j} of, and a handful of non-uniform layers (embedding table, LM head) that live only in the
 * first and the last stage and give the constant terms nu_{i,1}, nu_{i,pp} of the stage cost.  This header is that
 * part of a LLaMA-2 style model (Sec. 7.1), forward and backward, as hand-written gfx950 kernels; together with
 * mls_stage_* of mls.h a complete model step runs on one GPU:
 *     tokens -> mls_embed_forward -> mls_stage_forward -> mls_head_forward -> loss
 *     mls_head_backward -> mls_stage_backward -> mls_embed_backward -> grads
 *
 * Conventions as in mls.h: int functions return 0 or a negative MLS_E_* code (text via mls_last_error); every data
 * pointer is a DEVICE pointer, 16-byte aligned, owned by the caller; work is enqueued on the stream given at init
 * and nothing synchronises or allocates after init; one handle is used by one host thread at a time.
 *
 * Parameters (untied), in this order, each row-major, in the storage type; `grads` is the same layout in fp32 and
 * is only ever added to:
 *     embed  [vocab, hidden]   token embedding table          0.02*z
 *     gamma_f[hidden]          gain of the final RMSNorm      1 + 0.02*z
 *     w_lm   [hidden, vocab]   LM head                        0.02*z
 * drawn from the generator documented at mls_stage_init with tensor ids 6, 7, 8 and layer 0.
 */
#ifndef MLS_ENDS_H
#define MLS_ENDS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mls_ends mls_ends; /* opaque; owns its parameters, the stash and the workspace */

enum { MLS_PE_EMBED = 0, MLS_PE_GAMMA_F = 1, MLS_PE_WLM = 2 };

typedef struct {
  int32_t hidden;       /* h; multiple of 8, at most 16384                                            */
  int32_t vocab;        /* V; multiple of 8                                                           */
  int32_t seq;          /* S                                                                          */
  int32_t micro_batch;  /* b sequences per micro-batch; T = b*S tokens per call                       */
  int32_t max_inflight; /* stash depth, separately for the embedding side and the head side           */
  float rms_eps;        /* final RMSNorm: added to the mean of squares inside the square root         */
  int32_t dtype;        /* MLS_BF16 or MLS_FP32: storage type of activations and parameters           */
} mls_ends_config;

int mls_ends_init(const mls_ends_config* cfg, uint64_t seed, void* hip_stream, mls_ends** out);
void mls_ends_free(mls_ends* e);

/* x[t, :] = embed[tokens[t], :] for the T tokens (int32) of one micro-batch; a token id outside [0, vocab) gives a
 * zero row and no gradient.  Keeps the token ids for the backward (FIFO; MLS_E_STASH when max_inflight are held). */
int mls_embed_forward(mls_ends* e, const int32_t* tokens, void* x);

/* grads_embed[v, :] += sum over the positions t of the n oldest kept micro-batches with tokens[t] == v of dX[t, :],
 * in ascending (micro-batch, position) order: no float atomics, bitwise reproducible.  dX: [n, b, S, hidden]. */
int mls_embed_backward(mls_ends* e, const void* dX, float* grads, int32_t n);

/* One micro-batch through the final RMSNorm, the LM head and the loss:
 *     nrm = RMSNorm(y; gamma_f);  logits = nrm w_lm;  loss = (1/T) sum_t (logsumexp(logits_t) - logits_t[targets_t])
 * A target outside [0, vocab) is ignored: its token adds nothing to the sum (the divisor stays T) and gets a zero
 * gradient.  *loss (device, fp32) receives the unweighted loss of this micro-batch.  The gradient of
 * loss_weight * loss w.r.t. the logits is formed at once, in place of the logits, so the weight of this micro-batch
 * in the step's objective (normally 1 / number of micro-batches) is given here.  Keeps y, the RMS reciprocals, nrm
 * and that gradient for the backward (FIFO; MLS_E_STASH when max_inflight are held). */
int mls_head_forward(mls_ends* e, const void* y, const int32_t* targets, float loss_weight, float* loss);

/* For callers that cannot allocate device memory or do not want the library to (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): mls_head_forward with the per-token loss terms, the one
 * scratch buffer of its kernels, kept in a fixed array inside the library's code object (256 KiB per GPU, held until
 * the process ends) instead of the handle's allocation.  Same arguments, same results bit for bit.  At most 65536
 * tokens per micro-batch (seq * micro_batch), else MLS_E_RANGE.  Calls no hipMalloc / hipFree.  All calls on one GPU
 * share that array, whatever their handle or stream: calls that overlap in time on one GPU race on it; calls that
 * follow each other on one stream do not (every term a call reads it has written before). */
int mls_head_forward_static(mls_ends* e, const void* y, const int32_t* targets, float loss_weight, float* loss);

/* Backward of the n oldest kept head micro-batches, in push order: dY[i] = gradient w.r.t. y of micro-batch i
 * ([n, b, S, hidden], the dY that mls_stage_backward takes); grads_w_lm += sum_i nrm_i^T dlogits_i (one
 * contraction over all n, fp32); grads_gamma_f +=. */
int mls_head_backward(mls_ends* e, float* grads, int32_t n, void* dY);

size_t mls_ends_grad_elems(const mls_ends* e); /* vocab*hidden + hidden + hidden*vocab */
/* offset (elements), rows, cols of parameter `which` (MLS_PE_*) in the parameter / gradient vector */
int mls_ends_param_layout(const mls_ends* e, int32_t which, size_t* offset, size_t* rows, size_t* cols);
int mls_ends_get_params(mls_ends* e, void* dst);       /* device buffer of mls_ends_grad_elems storage elements */
int mls_ends_set_params(mls_ends* e, const void* src);
/* kept micro-batches: embedding side in *embed, head side in *head (either may be NULL) */
int mls_ends_inflight(const mls_ends* e, int32_t* embed, int32_t* head);
/* logits gradient of kept head micro-batch `slot` (0 = oldest): dense [T, vocab] in the storage type, for tests */
int mls_ends_debug_dlogits(mls_ends* e, int32_t slot, void* dst);

#ifdef __cplusplus
}
#endif
#endif
