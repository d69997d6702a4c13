/*
 * mls.h - C ABI of the decoder-stage library (HIP, gfx950).
 *
 * One handle = one GPU's pipeline stage in a hybrid-parallel training step: up to `max_layers` LLaMA-style
 * decoder layers (pre-norm RMSNorm, rotary embedding, causal grouped-query attention, SwiGLU, no biases).
 * The two integers a parallelization plan assigns to a GPU, the stage's layer count l_{i,j} and the
 * pipeline's micro-batch count m_i (paper Sec. 3, Table 1 of notations; Sec. 4.2, Eq. 1), are run-time arguments:
 * `k_layers` of mls_stage_forward and `n_microbatches` of mls_stage_backward.  Both may be zero (Eq. 1
 * lets l and m range over the non-negative integers).  One forward + backward of one layer on one
 * micro-batch is the paper's tau(b) (Sec. 4.2, time cost model); the stage costs l * tau(b) per
 * micro-batch and about m * l * tau(b) per step.
 *
 * All data pointers are DEVICE pointers unless a comment says "host".  Tensors are row-major, token-major:
 * activations are [micro_batch, seq, hidden] with hidden contiguous.  The storage type (bf16 or fp32) is
 * fixed per handle; parameter gradients are always fp32.  Every call enqueues work on the HIP stream given
 * at init and returns without synchronising (exceptions: init, free, get/set params and debug reads, which
 * synchronise that stream).  The caller owns x, y, dY, dX and grads; the library owns weights, rotary
 * tables, the activation stash and its workspace, all allocated in mls_stage_init (the forward and
 * backward calls allocate nothing).  x, y, dY, dX, grads and the operands of mls_gemm must be 16-byte aligned
 * (MLS_E_CONFIG otherwise).
 *
 * Every function that returns int returns MLS_OK (0) or a negative MLS_E_* code; a message for the last
 * failure on the calling thread is available from mls_last_error().  No C++ exception crosses this ABI.
 *
 * Public parameter layout, per layer, in this order, each matrix row-major [in, out]:
 *     gamma1[hidden]
 *     w_qkv [hidden, q_dim + 2*kv_dim]     columns: q heads | k heads | v heads
 *     w_o   [q_dim, hidden]
 *     gamma2[hidden]
 *     w_gu  [hidden, 2*ffn]                columns: gate | up
 *     w_d   [ffn, hidden]
 * with q_dim = n_q_heads*head_dim and kv_dim = n_kv_heads*head_dim.  Layers follow each other without
 * gaps.  `grads` uses the same layout in fp32.
 */
#ifndef MLS_H
#define MLS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mls_stage mls_stage; /* opaque */

enum { MLS_BF16 = 0, MLS_FP32 = 1 };

enum {
  MLS_OK = 0,
  MLS_E_CONFIG = -1,   /* invalid configuration value                                  */
  MLS_E_NULL = -2,     /* a required pointer is null                                   */
  MLS_E_RANGE = -3,    /* k_layers / n_microbatches / index out of range               */
  MLS_E_STASH = -4,    /* forward with a full stash, or backward over more than stashed */
  MLS_E_HIP = -5,      /* a HIP runtime call failed                                    */
  MLS_E_NOMEM = -6     /* device allocation failed                                     */
};

/* Which parameter tensor, for mls_stage_param_layout. */
enum { MLS_P_GAMMA1 = 0, MLS_P_WQKV = 1, MLS_P_WO = 2, MLS_P_GAMMA2 = 3, MLS_P_WGU = 4, MLS_P_WD = 5 };

/* Tensors mls_stage_debug_read can copy out of a stash entry (all in the storage type unless noted). */
enum {
  MLS_T_X = 0,    /* layer input              [T, hidden]                                   */
  MLS_T_A = 1,    /* RMSNorm-1 output         [T, hidden]                                   */
  MLS_T_QKV = 2,  /* q|k|v after rotary       [T, q_dim + 2*kv_dim]                         */
  MLS_T_O = 3,    /* attention output         [T, q_dim]                                    */
  MLS_T_H = 4,    /* x + o*w_o                [T, hidden]                                   */
  MLS_T_B = 5,    /* RMSNorm-2 output         [T, hidden]                                   */
  MLS_T_GU = 6,   /* gate|up                  [T, 2*ffn]                                    */
  MLS_T_Z = 7,    /* SwiGLU output            [T, ffn]                                      */
  MLS_T_LSE = 8,  /* natural-log softmax denominators, fp32 [micro_batch, n_q_heads, seq]   */
  /* the upstream-gradient operands of layer 0 of one micro-batch of the most recent backward call (workspace,
     overwritten by later calls); `slot` is the index of the micro-batch inside that call: */
  MLS_T_DY = 16,   /* gradient w.r.t. the layer output   [T, hidden]                        */
  MLS_T_DGU = 17,  /* gradient w.r.t. gate|up            [T, 2*ffn]                         */
  MLS_T_DH = 18,   /* gradient w.r.t. h                  [T, hidden]                        */
  MLS_T_DQKV = 19  /* gradient w.r.t. q|k|v (pre-rotary) [T, q_dim + 2*kv_dim]             */
};

typedef struct {
  int32_t hidden;       /* h; multiple of 8                                                          */
  int32_t n_q_heads;    /* query heads; q_dim = n_q_heads*head_dim need not equal hidden             */
  int32_t n_kv_heads;   /* KV heads; must divide n_q_heads; query head hq reads hq / (n_q/n_kv)      */
  int32_t head_dim;     /* 64 or 128 for bf16 storage; any even value up to 128 for fp32             */
  int32_t ffn;          /* f; multiple of 8                                                          */
  int32_t seq;          /* S; rotary position = index inside the sequence                            */
  int32_t micro_batch;  /* b sequences per micro-batch; T = b*S tokens, fixed for the handle         */
  int32_t max_layers;   /* upper bound of k_layers; weights for this many layers are held            */
  int32_t max_inflight; /* stash depth: forwarded micro-batches not yet consumed by a backward       */
  float rms_eps;        /* added to the mean of squares inside the square root                       */
  float rope_base;      /* theta_i = rope_base^(-2i/head_dim), pairs (i, i + head_dim/2)             */
  int32_t dtype;        /* MLS_BF16 or MLS_FP32: storage type of activations and weights             */
  int32_t recompute;    /* 1: activation recomputation -- keep only each layer's input and rebuild its   */
                        /* other tensors in the backward (one more forward per layer, bit-identical      */
                        /* results, 1/16 of the stash at the 7B shape); 0: keep everything               */
} mls_config;

/* Create a stage on the current HIP device.  Weights are drawn from the counter-based generator below
 * with `seed`: projections 0.02*z, gains 1 + 0.02*z, z ~ N(0,1), rounded once to the storage type.
 *     mix(z): z += 0x9E3779B97F4A7C15; z = (z ^ z>>30)*0xBF58476D1CE4E5B9;
 *             z = (z ^ z>>27)*0x94D049BB133111EB; return z ^ z>>31           (mod 2^64)
 *     stream = mix(mix(seed) ^ (tensor<<32 | layer));  r1 = mix(stream + 2i);  r2 = mix(stream + 2i + 1)
 *     z = sqrt(-2 ln(((r1>>11)+1) 2^-53)) * cos(2 pi (r2>>11) 2^-53)        i = flat index, public layout
 * hip_stream: a hipStream_t (host value) or NULL for the default stream.  *out receives the handle.
 * Errors: MLS_E_NULL, MLS_E_CONFIG, MLS_E_NOMEM, MLS_E_HIP. */
int mls_stage_init(const mls_config* cfg /*host*/, uint64_t seed, void* hip_stream, mls_stage** out /*host*/);

/* Forward of one micro-batch through layers 0..k_layers-1 (the l_{i,j} of Eq. 1).  x, y: [b, S, hidden]
 * in the storage type; y may not alias x.  Pushes one stash entry (FIFO) that records k_layers.
 * k_layers = 0 copies x to y.  Errors: MLS_E_NULL, MLS_E_RANGE (k_layers outside [0, max_layers]),
 * MLS_E_STASH (max_inflight entries already stashed), MLS_E_HIP. */
int mls_stage_forward(mls_stage* s, const void* x, int32_t k_layers, void* y);

/* Backward over the n_microbatches oldest stash entries, in push order (the m_i of Eq. 1).
 * dY, dX: [n, b, S, hidden] in the storage type (entry i uses slice i); dX may alias dY.
 * grads: fp32, public layout, mls_stage_grad_elems() floats; the library only ever adds to it
 * (G += sum over the micro-batches: per layer the contributions of all n micro-batches are contracted in one
 * pass, in ascending order, and added to G once), it never zeroes it.  Entries forwarded with different k_layers
 * may be mixed.  n = 0 is a no-op.  Errors: MLS_E_NULL, MLS_E_RANGE (n < 0),
 * MLS_E_STASH (n exceeds the stashed entries), MLS_E_HIP. */
int mls_stage_backward(mls_stage* s, const void* dY, float* grads, int32_t n_microbatches, void* dX);

/* mls_stage_backward with flags.  MLS_BWD_OVERWRITE: `grads` is written, not added to -- every layer some entry of
 * this call reached receives exactly the gradient of this call (bit-identical to zeroing grads and calling
 * mls_stage_backward), all other layers up to max_layers are set to zero; the fp32 gradient vector is then never
 * read, which saves the caller's zeroing pass and the read half of the accumulation (n = 0 zeroes everything).
 * Use it for the first backward call of a step and plain accumulation for the following ones. */
enum { MLS_BWD_OVERWRITE = 1 };
int mls_stage_backward_ex(mls_stage* s, const void* dY, float* grads, int32_t n_microbatches, void* dX, int32_t flags);

/* Release everything the handle owns (synchronises the stream first).  NULL is allowed. */
void mls_stage_free(mls_stage* s);

/* ---- support calls, off the hot path ---- */

/* Number of floats in `grads` (= number of parameters) for max_layers layers; 0 if s is NULL. */
size_t mls_stage_grad_elems(const mls_stage* s);

/* Device memory a stage of this configuration allocates in mls_stage_init, without creating one: the inputs of the
 * linear memory model l*mu(b) + nu(b) <= C of the paper's cost model (Sec. 4.2; Appendix B.4).  In that model's
 * terms, per layer: the forward activations of one kept micro-batch a_f = stash_bytes_per_layer_microbatch (the
 * stash holds max_inflight of them: a stage j of a 1F1B pipeline with pp stages needs max_inflight = pp - j + 1),
 * the model states s = param_bytes_per_layer + grad_bytes_per_layer (+ 12 B per parameter of optimizer state,
 * mls_optim.h); workspace_bytes does not grow with the layer count. */
typedef struct {
  size_t total_bytes;                       /* = param_bytes + stash_bytes + workspace_bytes              */
  size_t param_bytes;                       /* max_layers layers, storage type, internal row-padded layout;
                                               bf16: plus the transposed copy of the four matrices of a layer
                                               that the forward products read                               */
  size_t stash_bytes;                       /* max_inflight * max_layers entries                           */
  size_t workspace_bytes;                   /* backward workspace, recomputation scratch, rotary tables    */
  size_t param_bytes_per_layer;
  size_t grad_bytes_per_layer;              /* fp32, the caller's buffer (not part of total_bytes)         */
  size_t stash_bytes_per_layer_microbatch;
} mls_memory;
int mls_stage_memory(const mls_config* cfg, mls_memory* out);

/* Offset (in elements, from the start of the flat parameter/grad vector), rows and cols of tensor `which`
 * (MLS_P_*) of `layer`; gains report rows = 1.  Errors: MLS_E_NULL, MLS_E_RANGE. */
int mls_stage_param_layout(const mls_stage* s, int32_t layer, int32_t which, size_t* offset /*host*/,
                           size_t* rows /*host*/, size_t* cols /*host*/);

/* Copy all parameters (storage type, public layout) to / from a DEVICE buffer of mls_stage_grad_elems()
 * elements.  Errors: MLS_E_NULL, MLS_E_HIP. */
int mls_stage_get_params(mls_stage* s, void* dst);
int mls_stage_set_params(mls_stage* s, const void* src);

/* Number of stash entries currently held; negative error code if s is NULL. */
int mls_stage_inflight(const mls_stage* s);

/* Drop all stash entries without running a backward. */
int mls_stage_reset(mls_stage* s);

/* Operand capture for tests: copy tensor `tensor_id` (MLS_T_*) of `layer` of the stash entry that is
 * `slot` pushes old (0 = oldest) into the DEVICE buffer dst, which must hold the tensor (with recomputation
 * only MLS_T_X is kept: the other stash tensors give MLS_E_RANGE).  For the MLS_T_D* ids `layer` is ignored
 * (always layer 0) and `slot` counts the micro-batches of the most recent backward call (0 = its first; an
 * entry that ran no layer gives MLS_E_RANGE).  Errors: MLS_E_NULL, MLS_E_RANGE, MLS_E_HIP. */
int mls_stage_debug_read(mls_stage* s, int32_t tensor_id, int32_t layer, int32_t slot, void* dst);

/* Per-kernel-class timing with HIP events recorded on the stage's stream, for the benchmark's roofline figure.
 * enable != 0 brackets every kernel launch of forward/backward with a pair of events (no synchronisation unless
 * more than 4096 launches are pending); enable = 0 stops it.  mls_stage_timing_read synchronises on the last
 * event, writes the accumulated milliseconds and launch counts per class into two HOST arrays of
 * MLS_TIMING_CLASSES entries (order: GEMM forward, GEMM data-gradient, GEMM weight-gradient, attention
 * forward, attention backward, RMSNorm, rotary, SwiGLU) and clears the accumulators.  A step that runs fused into
 * a neighbouring kernel (bf16 storage: the rotary steps, SwiGLU forward when ffn % 32 == 0) is counted with that
 * kernel's class and leaves its own class at zero.
 * Errors: MLS_E_NULL, MLS_E_HIP. */
#define MLS_TIMING_CLASSES 8
int mls_stage_timing(mls_stage* s, int32_t enable);
int mls_stage_timing_read(mls_stage* s, double* ms /*host*/, int64_t* launches /*host*/);

/* Stand-alone GEMM entry used by tests and micro-benchmarks of the stage's contraction kernel:
 * mode 0: C[M,N] = A[M,K] * B[K,N] (+ R[M,N] if R != NULL)   forward projections (+ residual)
 * mode 1: C[M,N] = A[M,K] * B[N,K]^T                          data gradients
 * mode 2: C[M,N] += A[K,M]^T * B[K,N], C fp32                 weight gradients, accumulated
 * A, B, R and (modes 0/1) C are in storage type `dtype`; all dims multiples of 8.  lda, ldb, ldc are the row
 * strides in elements of A, B and C (R shares ldc); 0 means dense (the row length of that operand); otherwise
 * a multiple of 8 not below the row length.
 * Runs on `hip_stream`.  Errors: MLS_E_NULL, MLS_E_CONFIG, MLS_E_HIP. */
int mls_gemm(int32_t dtype, int32_t mode, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
             const void* R, int64_t M, int64_t N, int64_t K, void* hip_stream);

/* Message for the last error returned on this thread (host string, never NULL). */
const char* mls_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MLS_H */
