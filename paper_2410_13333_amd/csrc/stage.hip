// Host side of the decoder-stage library: the handle, the activation stash, the fixed kernel sequence of a
// layer's forward and backward, and the C ABI declared in include/mls.h.  No kernel lives here.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/mls.h"
#include "kernels.h"

namespace {

thread_local std::string g_err;

int fail(int code, const std::string& msg) {
  g_err = msg;
  return code;
}
int fail_hip(hipError_t e, const char* what) {
  return fail(e == hipErrorOutOfMemory ? MLS_E_NOMEM : MLS_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
}  // namespace
namespace mls {
int set_error(int code, const char* msg) { return fail(code, msg); }
}  // namespace mls
namespace {
#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) return fail_hip(e_, #expr);   \
  } while (0)

// Optional per-kernel-class timing with HIP events recorded on the stage's own stream (off by default; the
// events add no synchronisation unless the pool runs out, which only happens while timing is on).
enum { CLS_GEMM_NN = 0, CLS_GEMM_NT, CLS_GEMM_TN, CLS_ATTN_FWD, CLS_ATTN_BWD, CLS_NORM, CLS_ROPE, CLS_SWIGLU, CLS_COUNT };

struct Timing {
  bool on = false;
  std::vector<hipEvent_t> ev;  // pairs: start, stop
  std::vector<int> cls;
  size_t used = 0;
  double ms[CLS_COUNT] = {};
  int64_t launches[CLS_COUNT] = {};

  hipError_t flush() {
    if (used == 0) return hipSuccess;
    hipError_t e = hipEventSynchronize(ev[2 * used - 1]);
    if (e != hipSuccess) return e;
    for (size_t i = 0; i < used; i++) {
      float t = 0.f;
      if ((e = hipEventElapsedTime(&t, ev[2 * i], ev[2 * i + 1])) != hipSuccess) return e;
      ms[cls[i]] += t;
      launches[cls[i]]++;
    }
    used = 0;
    return hipSuccess;
  }
  hipError_t begin(int c, hipStream_t st) {
    if (used * 2 == ev.size()) {
      hipError_t e = flush();
      if (e != hipSuccess) return e;
    }
    cls[used] = c;
    return hipEventRecord(ev[2 * used], st);
  }
  hipError_t end(hipStream_t st) { return hipEventRecord(ev[2 * used++ + 1], st); }
};

// Byte offsets of one layer's tensors inside one stash entry.
struct LayerStash {
  size_t x, a, qkv, o, h, b, gu, z, r1, r2, lse, bytes;
};

}  // namespace

struct mls_stage {
  mls_config c;
  int dt;         // mls::DT_*
  size_t es;      // bytes per stored element
  int T, qd, kvd, qkvw;
  hipStream_t st;
  size_t layer_params;  // elements per layer, public (dense) layout
  size_t off_g1, off_wqkv, off_wo, off_g2, off_wgu, off_wd;  // public offsets (also the layout of grads)
  // Internal row strides (elements).  Widths whose byte size is a multiple of 512 get 64 extra elements so that
  // the rows of a GEMM tile do not all fall on the same L2 / memory channel.
  int64_t ld_h, ld_qkv, ld_qd, ld_gu, ld_f;
  // SwiGLU runs as the epilogue of the gate/up contraction; w_gu, gu and dgu are then kept in the interleaved
  // gate/up column order (bf16 storage, ffn % 32 == 0)
  bool fuse_gu = false;
  bool fuse_rope = false;  // the forward rotary step runs as the epilogue of the q|k|v projection (bf16 storage)
  size_t ilayer_params;  // elements per layer, internal (row-padded) layout
  size_t ioff_g1, ioff_wqkv, ioff_wo, ioff_g2, ioff_wgu, ioff_wd;
  char* params = nullptr;  // storage type, internal layout
  // Transposed copies of the four weight matrices of every layer (bf16 storage only): the forward contractions
  // Y = X W then read W^T as a [row][k] operand, like the data-gradient contractions dX = dY W^T read W itself: that
  // form of the bf16 GEMM measured the fastest of the three, by up to 19 % at the q|k|v shape.  Refreshed whenever the
  // weights change.
  char* params_t = nullptr;
  size_t tlayer_params = 0, toff_wqkv = 0, toff_wo = 0, toff_wgu = 0, toff_wd = 0;  // elements per layer, offsets
  float *cos_tab = nullptr, *sin_tab = nullptr;
  LayerStash ls;
  // Stash entry of one (micro-batch, layer): the full LayerStash, or with activation recomputation only the
  // layer input x (offset 0 in both).  rc_scratch: max_inflight full entries the recomputed tensors live in.
  size_t entry_bytes = 0;
  char* rc_scratch = nullptr;
  char* stash = nullptr;  // [max_inflight][max_layers] entries
  std::vector<int> slot_k;
  int head = 0, count = 0;  // FIFO ring over the slots
  // backward workspace.  g0, g1 (ping-pong gradient of the residual stream), dgu, dh and dqkv exist once per
  // in-flight micro-batch (they are the operands of the weight-gradient contractions, which run once per layer
  // over all micro-batches of a backward call); dz, dbuf and dc are transient and shared.
  char *g0 = nullptr, *g1 = nullptr, *dz = nullptr, *dgu = nullptr, *dbuf = nullptr, *dh = nullptr, *dc = nullptr,
       *dqkv = nullptr;
  size_t mb_h = 0, mb_gu = 0, mb_qkv = 0;  // bytes per micro-batch of the [T,ld_h], [T,ld_gu], [T,ld_qkv] buffers
  // partial, partial2: row-block sums of the two gain gradients of a layer, summed over a call's micro-batches
  float *delta = nullptr, *partial = nullptr, *partial2 = nullptr, *gqa_part = nullptr;  // gqa_part: partial dK/dV sums (few KV heads)
  std::vector<int> last_k;  // layer counts of the entries of the most recent backward call (for mls_stage_debug_read)
  Timing tm;

  char* slot_layer(int slot, int layer) const {
    return stash + (size_t(slot) * c.max_layers + layer) * entry_bytes;
  }
  char* param(int layer, size_t ioff) const { return params + (size_t(layer) * ilayer_params + ioff) * es; }
  char* param_t(int layer, size_t toff) const { return params_t + (size_t(layer) * tlayer_params + toff) * es; }
};

namespace {

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

// launch `expr` (a hipError_t expression), bracketed by events of class `c` while timing is on
#define LAUNCH(c, expr)                                  \
  do {                                                   \
    if (s->tm.on) HIP_TRY(s->tm.begin(c, s->st));        \
    HIP_TRY(expr);                                       \
    if (s->tm.on) HIP_TRY(s->tm.end(s->st));             \
  } while (0)

hipError_t gemm(const mls_stage* s, int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K,
                int64_t lda, int64_t ldb, int64_t ldc, int64_t ldr = 0) {
  return s->dt == mls::DT_BF16 ? mls::gemm_bf16(mode, A, B, C, R, M, N, K, lda, ldb, ldc, ldr, s->st)
                               : mls::gemm_f32(mode, A, B, C, R, M, N, K, lda, ldb, ldc, ldr, s->st);
}

int check_config(const mls_config& c) {
  if (c.dtype != MLS_BF16 && c.dtype != MLS_FP32) return fail(MLS_E_CONFIG, "dtype must be MLS_BF16 or MLS_FP32");
  if (c.hidden < 8 || c.hidden % 8 || c.hidden > 16384) return fail(MLS_E_CONFIG, "hidden must be a multiple of 8 in [8, 16384]");
  if (c.ffn < 8 || c.ffn % 8) return fail(MLS_E_CONFIG, "ffn must be a positive multiple of 8");
  if (c.n_q_heads < 1 || c.n_kv_heads < 1 || c.n_q_heads % c.n_kv_heads)
    return fail(MLS_E_CONFIG, "n_kv_heads must be positive and divide n_q_heads");
  if (c.dtype == MLS_BF16 && c.head_dim != 64 && c.head_dim != 128)
    return fail(MLS_E_CONFIG, "head_dim must be 64 or 128 for bf16 storage");
  if (c.dtype == MLS_FP32 && (c.head_dim < 16 || c.head_dim > 128 || c.head_dim % 16))
    return fail(MLS_E_CONFIG, "head_dim must be a multiple of 16 up to 128 for fp32 storage");
  if (c.seq < 1 || c.micro_batch < 1) return fail(MLS_E_CONFIG, "seq and micro_batch must be positive");
  if (c.max_layers < 0 || c.max_inflight < 1) return fail(MLS_E_CONFIG, "max_layers >= 0 and max_inflight >= 1 required");
  if (c.recompute != 0 && c.recompute != 1) return fail(MLS_E_CONFIG, "recompute must be 0 or 1");
  if (!(c.rms_eps >= 0.f) || !(c.rope_base > 0.f)) return fail(MLS_E_CONFIG, "rms_eps >= 0 and rope_base > 0 required");
  const int64_t T = int64_t(c.seq) * c.micro_batch;
  const int64_t widest = std::max<int64_t>(2 * int64_t(c.ffn), int64_t(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim);
  if (T > (1 << 24) || widest > (1 << 24) || T * widest > (int64_t(1) << 40))
    return fail(MLS_E_CONFIG, "tokens per micro-batch or layer width too large");
  if (c.dtype == MLS_BF16 && int64_t(c.seq + 128) * ((c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim + 64) * 2 >= (int64_t(1) << 31))
    return fail(MLS_E_CONFIG, "seq * (q_dim + 2 kv_dim) must stay below 2^30 elements for bf16 storage");
  return MLS_OK;
}

int64_t padded(int64_t n) { return n % 256 == 0 ? n + 64 : n; }

// the six parameter tensors of a layer: public offset, internal offset, rows, cols, internal row stride
struct PTensor { size_t off, ioff; int64_t rows, cols, ld; uint32_t tid; double scale, offset; };
void param_tensors(const mls_stage* s, PTensor (&t)[6]) {
  const mls_config& c = s->c;
  t[0] = {s->off_g1, s->ioff_g1, 1, c.hidden, c.hidden, MLS_P_GAMMA1, 0.02, 1.0};
  t[1] = {s->off_wqkv, s->ioff_wqkv, c.hidden, s->qkvw, s->ld_qkv, MLS_P_WQKV, 0.02, 0.0};
  t[2] = {s->off_wo, s->ioff_wo, s->qd, c.hidden, s->ld_h, MLS_P_WO, 0.02, 0.0};
  t[3] = {s->off_g2, s->ioff_g2, 1, c.hidden, c.hidden, MLS_P_GAMMA2, 0.02, 1.0};
  t[4] = {s->off_wgu, s->ioff_wgu, c.hidden, 2 * int64_t(c.ffn), s->ld_gu, MLS_P_WGU, 0.02, 0.0};
  t[5] = {s->off_wd, s->ioff_wd, c.ffn, c.hidden, s->ld_h, MLS_P_WD, 0.02, 0.0};
}

int init_weights(mls_stage* s, uint64_t seed) {
  PTensor t[6];
  param_tensors(s, t);
  for (int l = 0; l < s->c.max_layers; l++)
    for (auto& e : t)
      HIP_TRY(mls::fill_normal(s->dt, s->param(l, e.ioff), e.rows, e.cols, e.ld, seed, e.tid, (uint32_t)l, e.scale,
                               e.offset, s->st, e.tid == MLS_P_WGU && s->fuse_gu ? s->c.ffn : 0));
  return MLS_OK;
}

// the transposed weight copies of every layer from the current weights (bf16 storage)
int refresh_transposed(mls_stage* s) {
  if (!s->params_t) return MLS_OK;
  const mls_config& c = s->c;
  for (int l = 0; l < c.max_layers; l++) {
    HIP_TRY(mls::transpose_bf16(s->param(l, s->ioff_wqkv), s->ld_qkv, s->param_t(l, s->toff_wqkv), s->ld_h, c.hidden, s->qkvw, s->st));
    HIP_TRY(mls::transpose_bf16(s->param(l, s->ioff_wo), s->ld_h, s->param_t(l, s->toff_wo), s->ld_qd, s->qd, c.hidden, s->st));
    HIP_TRY(mls::transpose_bf16(s->param(l, s->ioff_wgu), s->ld_gu, s->param_t(l, s->toff_wgu), s->ld_h, c.hidden, 2 * c.ffn, s->st));
    HIP_TRY(mls::transpose_bf16(s->param(l, s->ioff_wd), s->ld_h, s->param_t(l, s->toff_wd), s->ld_f, c.ffn, c.hidden, s->st));
  }
  return MLS_OK;
}

// dense <-> row-padded copies of a rows x cols matrix of the storage type
hipError_t copy2d(const mls_stage* s, void* dst, int64_t ld_dst, const void* src, int64_t ld_src, int64_t rows,
                  int64_t cols) {
  return hipMemcpy2DAsync(dst, size_t(ld_dst) * s->es, src, size_t(ld_src) * s->es, size_t(cols) * s->es, size_t(rows),
                          hipMemcpyDeviceToDevice, s->st);
}

// ---- one decoder layer, forward.  `x` lives in the stash entry already; `out` receives x + attention + MLP.
// `x`: the layer input (row stride ld_h); `e`: the entry that receives the layer's other tensors (e + L.x itself
// is not touched); out == nullptr skips the last contraction (recomputation needs only its operands).
int layer_forward(mls_stage* s, int layer, const char* x, char* e, void* out, int64_t ld_out) {
  const mls_config& c = s->c;
  const LayerStash& L = s->ls;
  const int T = s->T, h = c.hidden, f = c.ffn;
  const int64_t lh = s->ld_h, lq = s->ld_qkv, lo = s->ld_qd, lg = s->ld_gu, lf = s->ld_f;
  LAUNCH(CLS_NORM, mls::rmsnorm_fwd(s->dt, x, lh, s->param(layer, s->ioff_g1), e + L.a, lh, (float*)(e + L.r1), T, h,
                                    c.rms_eps, s->st));
  // with the transposed weight copies every product runs as X (W^T)^T, W^T being the [row][k] operand
  const bool wt = s->params_t != nullptr;
  if (s->fuse_rope) {  // the rotation of q and k is the epilogue of their projection
    if (wt)
      LAUNCH(CLS_GEMM_NN, mls::gemm_bf16_rope(e + L.a, s->param_t(layer, s->toff_wqkv), e + L.qkv, T, s->qkvw, h, lh, lh, lq, s->cos_tab,
                                              s->sin_tab, c.seq, s->qd + s->kvd, c.head_dim, s->st, true));
    else
      LAUNCH(CLS_GEMM_NN, mls::gemm_bf16_rope(e + L.a, s->param(layer, s->ioff_wqkv), e + L.qkv, T, s->qkvw, h, lh, lq, lq, s->cos_tab,
                                              s->sin_tab, c.seq, s->qd + s->kvd, c.head_dim, s->st));
  } else {
    LAUNCH(CLS_GEMM_NN, gemm(s, mls::GEMM_NN, e + L.a, s->param(layer, s->ioff_wqkv), e + L.qkv, nullptr, T, s->qkvw, h, lh, lq, lq));
    LAUNCH(CLS_ROPE, mls::rope_inplace(s->dt, e + L.qkv, s->cos_tab, s->sin_tab, T, c.seq, c.n_q_heads + c.n_kv_heads,
                                       c.head_dim, lq, 1.f, s->st));
  }
  LAUNCH(CLS_ATTN_FWD, mls::attn_fwd(s->dt, e + L.qkv, lq, e + L.o, lo, (float*)(e + L.lse), c.micro_batch, c.seq,
                                     c.n_q_heads, c.n_kv_heads, c.head_dim, s->st));
  if (wt) LAUNCH(CLS_GEMM_NN, gemm(s, mls::GEMM_NT, e + L.o, s->param_t(layer, s->toff_wo), e + L.h, x, T, h, s->qd, lo, lo, lh, lh));
  else LAUNCH(CLS_GEMM_NN, gemm(s, mls::GEMM_NN, e + L.o, s->param(layer, s->ioff_wo), e + L.h, x, T, h, s->qd, lo, lh, lh, lh));
  LAUNCH(CLS_NORM, mls::rmsnorm_fwd(s->dt, e + L.h, lh, s->param(layer, s->ioff_g2), e + L.b, lh, (float*)(e + L.r2), T, h,
                                    c.rms_eps, s->st));
  if (s->fuse_gu) {
    if (wt) LAUNCH(CLS_GEMM_NN, mls::gemm_bf16_swiglu(e + L.b, s->param_t(layer, s->toff_wgu), e + L.gu, e + L.z, T, f, h, lh, lh, lg, lf, s->st, true));
    else LAUNCH(CLS_GEMM_NN, mls::gemm_bf16_swiglu(e + L.b, s->param(layer, s->ioff_wgu), e + L.gu, e + L.z, T, f, h, lh, lg, lg, lf, s->st));
  } else {
    LAUNCH(CLS_GEMM_NN, gemm(s, mls::GEMM_NN, e + L.b, s->param(layer, s->ioff_wgu), e + L.gu, nullptr, T, 2 * f, h, lh, lg, lg));
    LAUNCH(CLS_SWIGLU, mls::swiglu_fwd(s->dt, e + L.gu, lg, e + L.z, lf, T, f, s->st));
  }
  // `out` is either the next layer's x (row stride ld_h) or the caller's dense y
  if (out) {
    if (wt) LAUNCH(CLS_GEMM_NN, gemm(s, mls::GEMM_NT, e + L.z, s->param_t(layer, s->toff_wd), out, e + L.h, T, h, f, lf, lf, ld_out, lh));
    else LAUNCH(CLS_GEMM_NN, gemm(s, mls::GEMM_NN, e + L.z, s->param(layer, s->ioff_wd), out, e + L.h, T, h, f, lf, lh, ld_out, lh));
  }
  return MLS_OK;
}

// ---- one decoder layer, backward, for micro-batch workspace `w`: everything except the four weight-gradient
// contractions, whose operands (dy, dgu, dh, dqkv of this micro-batch) stay in the workspace for them.
// dy: gradient w.r.t. the layer output (row stride ld_dy); dx receives the gradient w.r.t. its input (row stride
// ld_dx); g: this layer's slice of the caller's fp32 gradient vector (gains only here).
int layer_backward_data(mls_stage* s, int layer, const char* x, const char* e, int w, const void* dy, int64_t ld_dy,
                        void* dx, int64_t ld_dx, float* g, bool ow, bool first, bool last) {
  const mls_config& c = s->c;
  const LayerStash& L = s->ls;
  const int T = s->T, h = c.hidden, f = c.ffn, qd = s->qd, wq = s->qkvw;
  const int64_t lh = s->ld_h, lq = s->ld_qkv, lo = s->ld_qd, lg = s->ld_gu, lf = s->ld_f;
  char* dgu = s->dgu + size_t(w) * s->mb_gu;
  char* dh = s->dh + size_t(w) * s->mb_h;
  char* dqkv = s->dqkv + size_t(w) * s->mb_qkv;
  // MLP
  // data gradients dX = dY W^T: W is the [row][k] operand
  LAUNCH(CLS_GEMM_NT, gemm(s, mls::GEMM_NT, dy, s->param(layer, s->ioff_wd), s->dz, nullptr, T, f, h, ld_dy, lh, lf));
  LAUNCH(CLS_SWIGLU, mls::swiglu_bwd(s->dt, s->dz, lf, e + L.gu, lg, dgu, lg, T, f, s->st, s->fuse_gu));
  LAUNCH(CLS_GEMM_NT, gemm(s, mls::GEMM_NT, dgu, s->param(layer, s->ioff_wgu), s->dbuf, nullptr, T, h, 2 * f, lg, lg, lh));
  LAUNCH(CLS_NORM, mls::rmsnorm_bwd(s->dt, s->dbuf, lh, e + L.h, lh, s->param(layer, s->ioff_g2), (const float*)(e + L.r2),
                                    dy, ld_dy, dh, lh, g + s->off_g2, s->partial2, T, h, s->st, ow, !first, last));
  // attention
  LAUNCH(CLS_GEMM_NT, gemm(s, mls::GEMM_NT, dh, s->param(layer, s->ioff_wo), s->dc, nullptr, T, qd, h, lh, lh, lo));
  // the bf16 attention-backward kernels turn dq and dk back by the rotary angle as they store them
  const bool unrot = s->dt == mls::DT_BF16;
  LAUNCH(CLS_ATTN_BWD, mls::attn_bwd(s->dt, e + L.qkv, lq, e + L.o, lo, (const float*)(e + L.lse), s->dc, lo, dqkv, lq,
                                     s->delta, c.micro_batch, c.seq, c.n_q_heads, c.n_kv_heads, c.head_dim, s->st, s->gqa_part,
                                     unrot ? s->cos_tab : nullptr, unrot ? s->sin_tab : nullptr));
  if (!unrot)
    LAUNCH(CLS_ROPE, mls::rope_inplace(s->dt, dqkv, s->cos_tab, s->sin_tab, T, c.seq, c.n_q_heads + c.n_kv_heads,
                                       c.head_dim, lq, -1.f, s->st));
  LAUNCH(CLS_GEMM_NT, gemm(s, mls::GEMM_NT, dqkv, s->param(layer, s->ioff_wqkv), s->dbuf, nullptr, T, h, wq, lq, lq, lh));
  LAUNCH(CLS_NORM, mls::rmsnorm_bwd(s->dt, s->dbuf, lh, x, lh, s->param(layer, s->ioff_g1), (const float*)(e + L.r1),
                                    dh, lh, dx, ld_dx, g + s->off_g1, s->partial, T, h, s->st, ow, !first, last));
  return MLS_OK;
}

// C[M,N] += sum_i A_i[T,M]^T B_i[T,N] over n micro-batches (fp32 C): one launch per 16 micro-batches on the bf16
// DMA path, one launch per micro-batch otherwise
int wgrad(mls_stage* s, const void* const* A, const void* const* B, int n, float* C, int M, int N, int64_t lda,
          int64_t ldb, int gu_f, bool ow) {
  if (s->dt == mls::DT_BF16 && mls::gemm_tn_segments_ok(s->T, lda, ldb)) {  // always true when gu_f > 0
    for (int i = 0; i < n; i += 16)
      LAUNCH(CLS_GEMM_TN, mls::gemm_bf16_tn_segments(A + i, B + i, n - i < 16 ? n - i : 16, C, M, N, s->T, lda, ldb, N, s->st,
                                                     gu_f, ow && i == 0));
  } else {
    if (ow) HIP_TRY(mls::fill_zero_f32(C, size_t(M) * N, s->st));  // this path only accumulates
    for (int i = 0; i < n; i++) LAUNCH(CLS_GEMM_TN, gemm(s, mls::GEMM_TN, A[i], B[i], C, nullptr, M, N, s->T, lda, ldb, N));
  }
  return MLS_OK;
}

// every size and offset that follows from the configuration (no allocation)
void layout(mls_stage* s) {
  const mls_config& c = s->c;
  s->dt = c.dtype == MLS_BF16 ? mls::DT_BF16 : mls::DT_FP32;
  s->es = c.dtype == MLS_BF16 ? 2 : 4;
  s->T = c.seq * c.micro_batch;
  s->qd = c.n_q_heads * c.head_dim;
  s->kvd = c.n_kv_heads * c.head_dim;
  s->qkvw = s->qd + 2 * s->kvd;
  const size_t h = c.hidden, f = c.ffn, T = s->T;
  s->off_g1 = 0;
  s->off_wqkv = h;
  s->off_wo = s->off_wqkv + h * s->qkvw;
  s->off_g2 = s->off_wo + size_t(s->qd) * h;
  s->off_wgu = s->off_g2 + h;
  s->off_wd = s->off_wgu + h * 2 * f;
  s->layer_params = s->off_wd + f * h;
  s->ld_h = padded(c.hidden);
  s->ld_qkv = padded(s->qkvw);
  s->ld_qd = padded(s->qd);
  s->ld_gu = padded(2 * int64_t(c.ffn));
  s->ld_f = padded(c.ffn);
  s->ioff_g1 = 0;
  s->ioff_wqkv = h;
  s->ioff_wo = s->ioff_wqkv + h * s->ld_qkv;
  s->ioff_g2 = s->ioff_wo + size_t(s->qd) * s->ld_h;
  s->ioff_wgu = s->ioff_g2 + h;
  s->ioff_wd = s->ioff_wgu + h * s->ld_gu;
  s->ilayer_params = s->ioff_wd + f * s->ld_h;
  // transposed copies: w_qkv^T [qkvw, ld_h], w_o^T [h, ld_qd], w_gu^T [2f, ld_h], w_d^T [h, ld_f]
  s->toff_wqkv = 0;
  s->toff_wo = s->toff_wqkv + size_t(s->qkvw) * s->ld_h;
  s->toff_wgu = s->toff_wo + h * s->ld_qd;
  s->toff_wd = s->toff_wgu + 2 * f * s->ld_h;
  s->tlayer_params = s->toff_wd + h * s->ld_f;
  s->fuse_gu = s->dt == mls::DT_BF16 && mls::gemm_swiglu_ok(s->T, c.ffn, c.hidden, s->ld_h, s->ld_gu) &&
               mls::gemm_tn_segments_ok(s->T, s->ld_h, s->ld_gu);

  s->fuse_rope = s->dt == mls::DT_BF16 && mls::gemm_rope_ok(s->T, s->qkvw, c.hidden, s->ld_h, s->ld_qkv, c.seq,
                                                            s->qd + s->kvd, c.head_dim);

  LayerStash& L = s->ls;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes); return at; };
  L.x = take(T * s->ld_h * s->es);
  L.a = take(T * s->ld_h * s->es);
  L.qkv = take(T * s->ld_qkv * s->es);
  L.o = take(T * s->ld_qd * s->es);
  L.h = take(T * s->ld_h * s->es);
  L.b = take(T * s->ld_h * s->es);
  L.gu = take(T * s->ld_gu * s->es);
  L.z = take(T * s->ld_f * s->es);
  L.r1 = take(T * 4);
  L.r2 = take(T * 4);
  L.lse = take(size_t(c.micro_batch) * c.n_q_heads * c.seq * 4);
  L.bytes = o;
  s->slot_k.assign(c.max_inflight, 0);

  s->entry_bytes = c.recompute ? align256(T * s->ld_h * s->es) : L.bytes;
  s->mb_h = align256(T * s->ld_h * s->es);
  s->mb_gu = align256(T * s->ld_gu * s->es);
  s->mb_qkv = align256(T * s->ld_qkv * s->es);
}

// the device allocations of a stage: name, bytes (what mls_stage_init allocates and mls_stage_memory reports)
struct Alloc { void** p; size_t bytes; int kind; };  // kind: 0 parameters, 1 stash, 2 workspace
std::vector<Alloc> allocations(mls_stage* s) {
  const mls_config& c = s->c;
  const size_t T = s->T, nmb = c.max_inflight, h = c.hidden;
  const int nb = mls::rmsnorm_bwd_blocks(s->T);
  return {
      {(void**)&s->params, size_t(c.max_layers) * s->ilayer_params * s->es, 0},
      {(void**)&s->params_t, s->dt == mls::DT_BF16 ? size_t(c.max_layers) * s->tlayer_params * s->es : 0, 0},
      {(void**)&s->cos_tab, size_t(c.seq) * (c.head_dim / 2) * 4, 2},
      {(void**)&s->sin_tab, size_t(c.seq) * (c.head_dim / 2) * 4, 2},
      {(void**)&s->stash, nmb * c.max_layers * s->entry_bytes, 1},
      {(void**)&s->rc_scratch, c.recompute ? nmb * s->ls.bytes : 0, 2},
      {(void**)&s->g0, nmb * s->mb_h, 2},
      {(void**)&s->g1, nmb * s->mb_h, 2},
      {(void**)&s->dz, T * s->ld_f * s->es, 2},
      {(void**)&s->dgu, nmb * s->mb_gu, 2},
      {(void**)&s->dbuf, T * s->ld_h * s->es, 2},
      {(void**)&s->dh, nmb * s->mb_h, 2},
      {(void**)&s->dc, T * s->ld_qd * s->es, 2},
      {(void**)&s->dqkv, nmb * s->mb_qkv, 2},
      {(void**)&s->delta, size_t(c.micro_batch) * c.n_q_heads * c.seq * 4, 2},
      {(void**)&s->partial, size_t(nb) * h * 4, 2},
      {(void**)&s->partial2, size_t(nb) * h * 4, 2},
      {(void**)&s->gqa_part, mls::attn_bwd_scratch_floats(s->dt, c.micro_batch, c.seq, c.n_q_heads, c.n_kv_heads, c.head_dim) * 4, 2},
  };
}

void release(mls_stage* s) {
  void* p[] = {s->params, s->params_t, s->cos_tab, s->sin_tab, s->stash, s->rc_scratch, s->g0, s->g1, s->dz, s->dgu, s->dbuf, s->dh, s->dc, s->dqkv,
               s->delta, s->partial, s->partial2, s->gqa_part};
  for (void* q : p)
    if (q) (void)hipFree(q);
  for (hipEvent_t e : s->tm.ev) (void)hipEventDestroy(e);
  delete s;
}

}  // namespace

extern "C" {

const char* mls_last_error(void) { return g_err.c_str(); }

int mls_stage_init(const mls_config* cfg, uint64_t seed, void* hip_stream, mls_stage** out) {
  if (!cfg || !out) return fail(MLS_E_NULL, "mls_stage_init: cfg and out must not be null");
  *out = nullptr;
  if (int rc = check_config(*cfg)) return rc;
  mls_stage* s = new (std::nothrow) mls_stage();
  if (!s) return fail(MLS_E_NOMEM, "host allocation failed");
  s->c = *cfg;
  s->st = (hipStream_t)hip_stream;
  layout(s);
  const mls_config& c = s->c;
  hipError_t e = hipSuccess;
  for (const Alloc& al : allocations(s))
    if (al.bytes && (e = hipMalloc(al.p, al.bytes)) != hipSuccess) {
      release(s);
      return fail_hip(e, "hipMalloc");
    }

  // rotary table: angle(p, i) = p * base^(-2i/d), evaluated in fp64 on the host, stored as fp32
  {
    const int d2 = c.head_dim / 2;
    std::vector<float> cs(size_t(c.seq) * d2), sn(cs.size());
    for (int i = 0; i < d2; i++) {
      const double theta = std::pow((double)c.rope_base, -2.0 * i / c.head_dim);
      for (int p = 0; p < c.seq; p++) {
        cs[size_t(p) * d2 + i] = (float)std::cos(p * theta);
        sn[size_t(p) * d2 + i] = (float)std::sin(p * theta);
      }
    }
    if ((e = hipMemcpy(s->cos_tab, cs.data(), cs.size() * 4, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(s->sin_tab, sn.data(), sn.size() * 4, hipMemcpyHostToDevice)) != hipSuccess) {
      release(s);
      return fail_hip(e, "hipMemcpy(rotary table)");
    }
  }
  if (int rc = init_weights(s, seed)) {
    release(s);
    return rc;
  }
  if (int rc = refresh_transposed(s)) {
    release(s);
    return rc;
  }
  if ((e = hipStreamSynchronize(s->st)) != hipSuccess) {
    release(s);
    return fail_hip(e, "hipStreamSynchronize");
  }
  *out = s;
  return MLS_OK;
}

int mls_stage_forward(mls_stage* s, const void* x, int32_t k_layers, void* y) {
  if (!s || !x || !y) return fail(MLS_E_NULL, "mls_stage_forward: null argument");
  if ((uintptr_t(x) | uintptr_t(y)) & 15) return fail(MLS_E_CONFIG, "mls_stage_forward: x and y must be 16-byte aligned");
  if (k_layers < 0 || k_layers > s->c.max_layers) return fail(MLS_E_RANGE, "k_layers outside [0, max_layers]");
  if (s->count >= s->c.max_inflight) return fail(MLS_E_STASH, "stash full: max_inflight micro-batches already forwarded");
  const size_t act = size_t(s->T) * s->c.hidden * s->es;
  const int slot = (s->head + s->count) % s->c.max_inflight;
  if (k_layers == 0) {
    HIP_TRY(hipMemcpyAsync(y, x, act, hipMemcpyDeviceToDevice, s->st));
  } else {
    HIP_TRY(copy2d(s, s->slot_layer(slot, 0) + s->ls.x, s->ld_h, x, s->c.hidden, s->T, s->c.hidden));
    for (int l = 0; l < k_layers; l++) {
      const bool last = l + 1 == k_layers;
      void* out = last ? y : (void*)(s->slot_layer(slot, l + 1) + s->ls.x);
      char* e = s->slot_layer(slot, l);
      // with recomputation only x is kept; the layer's other tensors are temporaries in the first scratch entry
      if (int rc = layer_forward(s, l, e + s->ls.x, s->c.recompute ? s->rc_scratch : e, out, last ? s->c.hidden : s->ld_h))
        return rc;
    }
  }
  s->slot_k[slot] = k_layers;
  s->count++;
  return MLS_OK;
}

int mls_stage_backward(mls_stage* s, const void* dY, float* grads, int32_t n, void* dX) {
  return mls_stage_backward_ex(s, dY, grads, n, dX, 0);
}

int mls_stage_backward_ex(mls_stage* s, const void* dY, float* grads, int32_t n, void* dX, int32_t flags) {
  if (!s) return fail(MLS_E_NULL, "mls_stage_backward: null handle");
  if (flags & ~MLS_BWD_OVERWRITE) return fail(MLS_E_CONFIG, "mls_stage_backward_ex: unknown flag");
  const bool ow = (flags & MLS_BWD_OVERWRITE) != 0;
  if (n < 0) return fail(MLS_E_RANGE, "n_microbatches must be >= 0");
  if (n == 0 && !ow) return MLS_OK;
  if (!grads || (n > 0 && (!dY || !dX))) return fail(MLS_E_NULL, "mls_stage_backward: null argument");
  if ((uintptr_t(dY) | uintptr_t(dX) | uintptr_t(grads)) & 15)
    return fail(MLS_E_CONFIG, "mls_stage_backward: dY, dX and grads must be 16-byte aligned");
  if (n > s->count) return fail(MLS_E_STASH, "n_microbatches exceeds the stashed micro-batches");
  const mls_config& c = s->c;
  const LayerStash& L = s->ls;
  const size_t act = size_t(s->T) * c.hidden * s->es;
  const int h = c.hidden, f = c.ffn;
  // Layer-major order: for each layer, top down, first the data-gradient chain of every micro-batch that has this
  // layer (entries may have been forwarded with different layer counts), then ONE weight-gradient contraction
  // per weight over all of them, so the fp32 gradient is read and written once per layer, not once per micro-batch.
  // The gradient w.r.t. the output of layer l of micro-batch i lives in its ping-pong buffer (l+1) & 1.
  auto pp = [&](int i, int which) { return (which ? s->g1 : s->g0) + size_t(i) * s->mb_h; };
  int kmax = 0;
  std::vector<int> slot(n), k(n);
  for (int i = 0; i < n; i++) {
    slot[i] = (s->head + i) % c.max_inflight;
    k[i] = s->slot_k[slot[i]];
    kmax = k[i] > kmax ? k[i] : kmax;
    const char* dy = (const char*)dY + size_t(i) * act;
    char* dx = (char*)dX + size_t(i) * act;
    if (k[i] == 0) {
      if (dx != dy) HIP_TRY(hipMemcpyAsync(dx, dy, act, hipMemcpyDeviceToDevice, s->st));
    } else {
      HIP_TRY(copy2d(s, pp(i, k[i] & 1), s->ld_h, dy, h, s->T, h));
    }
  }
  std::vector<const void*> az, ab, ao, aa, bdy, bdgu, bdh, bdqkv;
  for (int l = kmax - 1; l >= 0; l--) {
    float* g = grads + size_t(l) * s->layer_params;
    az.clear(); ab.clear(); ao.clear(); aa.clear(); bdy.clear(); bdgu.clear(); bdh.clear(); bdqkv.clear();
    int have = 0, seen = 0;  // micro-batches of this call that contain layer l
    for (int i = 0; i < n; i++) have += k[i] > l;
    for (int i = 0; i < n; i++) {
      if (k[i] <= l) continue;
      seen++;
      const char* x = s->slot_layer(slot[i], l) + L.x;
      const char* e = s->slot_layer(slot[i], l);
      if (c.recompute) {  // rebuild this layer's tensors from its kept input, into scratch entry i
        char* sc = s->rc_scratch + size_t(i) * L.bytes;
        if (int rc = layer_forward(s, l, x, sc, nullptr, 0)) return rc;
        e = sc;
      }
      const char* dy = pp(i, (l + 1) & 1);
      void* dx = l == 0 ? (void*)((char*)dX + size_t(i) * act) : (void*)pp(i, l & 1);
      if (int rc = layer_backward_data(s, l, x, e, i, dy, s->ld_h, dx, l == 0 ? h : s->ld_h, g, ow, seen == 1, seen == have)) return rc;
      az.push_back(e + L.z); ab.push_back(e + L.b); ao.push_back(e + L.o); aa.push_back(e + L.a);
      bdy.push_back(dy);
      bdgu.push_back(s->dgu + size_t(i) * s->mb_gu);
      bdh.push_back(s->dh + size_t(i) * s->mb_h);
      bdqkv.push_back(s->dqkv + size_t(i) * s->mb_qkv);
    }
    const int m = (int)az.size();
    if (int rc = wgrad(s, az.data(), bdy.data(), m, g + s->off_wd, f, h, s->ld_f, s->ld_h, 0, ow)) return rc;
    if (int rc = wgrad(s, ab.data(), bdgu.data(), m, g + s->off_wgu, h, 2 * f, s->ld_h, s->ld_gu, s->fuse_gu ? f : 0, ow)) return rc;
    if (int rc = wgrad(s, ao.data(), bdh.data(), m, g + s->off_wo, s->qd, h, s->ld_qd, s->ld_h, 0, ow)) return rc;
    if (int rc = wgrad(s, aa.data(), bdqkv.data(), m, g + s->off_wqkv, h, s->qkvw, s->ld_h, s->ld_qkv, 0, ow)) return rc;
  }
  // overwrite mode: the layers no entry of this call reached hold no gradient
  if (ow && kmax < c.max_layers)
    HIP_TRY(mls::fill_zero_f32(grads + size_t(kmax) * s->layer_params, size_t(c.max_layers - kmax) * s->layer_params, s->st));
  s->head = (s->head + n) % c.max_inflight;
  s->count -= n;
  s->last_k = k;
  return MLS_OK;
}

int mls_stage_memory(const mls_config* cfg, mls_memory* out) {
  if (!cfg || !out) return fail(MLS_E_NULL, "mls_stage_memory: null argument");
  if (int rc = check_config(*cfg)) return rc;
  mls_stage tmp;
  tmp.c = *cfg;
  layout(&tmp);
  mls_memory m = {};
  for (const Alloc& al : allocations(&tmp)) (al.kind == 0 ? m.param_bytes : al.kind == 1 ? m.stash_bytes : m.workspace_bytes) += al.bytes;
  m.total_bytes = m.param_bytes + m.stash_bytes + m.workspace_bytes;
  m.param_bytes_per_layer = (tmp.ilayer_params + (tmp.dt == mls::DT_BF16 ? tmp.tlayer_params : 0)) * tmp.es;
  m.stash_bytes_per_layer_microbatch = tmp.entry_bytes;
  m.grad_bytes_per_layer = tmp.layer_params * 4;
  *out = m;
  return MLS_OK;
}

void mls_stage_free(mls_stage* s) {
  if (!s) return;
  (void)hipStreamSynchronize(s->st);
  release(s);
}

size_t mls_stage_grad_elems(const mls_stage* s) { return s ? size_t(s->c.max_layers) * s->layer_params : 0; }

int mls_stage_param_layout(const mls_stage* s, int32_t layer, int32_t which, size_t* offset, size_t* rows, size_t* cols) {
  if (!s || !offset || !rows || !cols) return fail(MLS_E_NULL, "mls_stage_param_layout: null argument");
  if (layer < 0 || layer >= s->c.max_layers) return fail(MLS_E_RANGE, "layer out of range");
  const size_t h = s->c.hidden, f = s->c.ffn;
  size_t off, r, c;
  switch (which) {
    case MLS_P_GAMMA1: off = s->off_g1; r = 1; c = h; break;
    case MLS_P_WQKV: off = s->off_wqkv; r = h; c = s->qkvw; break;
    case MLS_P_WO: off = s->off_wo; r = s->qd; c = h; break;
    case MLS_P_GAMMA2: off = s->off_g2; r = 1; c = h; break;
    case MLS_P_WGU: off = s->off_wgu; r = h; c = 2 * f; break;
    case MLS_P_WD: off = s->off_wd; r = f; c = h; break;
    default: return fail(MLS_E_RANGE, "unknown parameter tensor");
  }
  *offset = size_t(layer) * s->layer_params + off;
  *rows = r;
  *cols = c;
  return MLS_OK;
}

int mls_stage_get_params(mls_stage* s, void* dst) {
  if (!s || !dst) return fail(MLS_E_NULL, "mls_stage_get_params: null argument");
  PTensor t[6];
  param_tensors(s, t);
  for (int l = 0; l < s->c.max_layers; l++)
    for (auto& e : t) {
      char* d = (char*)dst + (size_t(l) * s->layer_params + e.off) * s->es;
      if (e.tid == MLS_P_WGU && s->fuse_gu)
        HIP_TRY(mls::gu_permute(s->param(l, e.ioff), e.ld, d, e.cols, e.rows, s->c.ffn, false, s->st));
      else
        HIP_TRY(copy2d(s, d, e.cols, s->param(l, e.ioff), e.ld, e.rows, e.cols));
    }
  HIP_TRY(hipStreamSynchronize(s->st));
  return MLS_OK;
}

int mls_stage_set_params(mls_stage* s, const void* src) {
  if (!s || !src) return fail(MLS_E_NULL, "mls_stage_set_params: null argument");
  PTensor t[6];
  param_tensors(s, t);
  for (int l = 0; l < s->c.max_layers; l++)
    for (auto& e : t) {
      const char* p = (const char*)src + (size_t(l) * s->layer_params + e.off) * s->es;
      if (e.tid == MLS_P_WGU && s->fuse_gu)
        HIP_TRY(mls::gu_permute(p, e.cols, s->param(l, e.ioff), e.ld, e.rows, s->c.ffn, true, s->st));
      else
        HIP_TRY(copy2d(s, s->param(l, e.ioff), e.ld, p, e.cols, e.rows, e.cols));
    }
  if (int rc = refresh_transposed(s)) return rc;
  HIP_TRY(hipStreamSynchronize(s->st));
  return MLS_OK;
}

int mls_stage_inflight(const mls_stage* s) { return s ? s->count : fail(MLS_E_NULL, "null handle"); }

int mls_stage_reset(mls_stage* s) {
  if (!s) return fail(MLS_E_NULL, "null handle");
  s->head = 0;
  s->count = 0;
  return MLS_OK;
}

int mls_stage_debug_read(mls_stage* s, int32_t id, int32_t layer, int32_t slot, void* dst) {
  if (!s || !dst) return fail(MLS_E_NULL, "mls_stage_debug_read: null argument");
  const int64_t T = s->T, h = s->c.hidden, f = s->c.ffn;
  const void* src = nullptr;
  int64_t cols = 0, ld = 0;
  if (id >= MLS_T_DY) {
    // layer 0 of micro-batch `slot` of the most recent backward call: its workspace entries are still intact,
    // and the gradient w.r.t. the output of layer 0 sits in ping-pong buffer 1
    if (slot < 0 || slot >= (int)s->last_k.size()) return fail(MLS_E_RANGE, "micro-batch index beyond the most recent backward call");
    if (s->last_k[slot] == 0) return fail(MLS_E_RANGE, "that micro-batch ran no layer");
    switch (id) {
      case MLS_T_DY: src = s->g1 + size_t(slot) * s->mb_h; cols = h; ld = s->ld_h; break;
      case MLS_T_DGU: src = s->dgu + size_t(slot) * s->mb_gu; cols = 2 * f; ld = s->ld_gu; break;
      case MLS_T_DH: src = s->dh + size_t(slot) * s->mb_h; cols = h; ld = s->ld_h; break;
      case MLS_T_DQKV: src = s->dqkv + size_t(slot) * s->mb_qkv; cols = s->qkvw; ld = s->ld_qkv; break;
      default: return fail(MLS_E_RANGE, "unknown tensor id");
    }
  } else {
    if (slot < 0 || slot >= s->count) return fail(MLS_E_RANGE, "stash slot out of range");
    const int phys = (s->head + slot) % s->c.max_inflight;
    if (layer < 0 || layer >= s->slot_k[phys]) return fail(MLS_E_RANGE, "layer out of range for this stash entry");
    const char* e = s->slot_layer(phys, layer);
    const LayerStash& L = s->ls;
    if (s->c.recompute && id != MLS_T_X) return fail(MLS_E_RANGE, "with recomputation only MLS_T_X is kept");
    switch (id) {
      case MLS_T_X: src = e + L.x; cols = h; ld = s->ld_h; break;
      case MLS_T_A: src = e + L.a; cols = h; ld = s->ld_h; break;
      case MLS_T_QKV: src = e + L.qkv; cols = s->qkvw; ld = s->ld_qkv; break;
      case MLS_T_O: src = e + L.o; cols = s->qd; ld = s->ld_qd; break;
      case MLS_T_H: src = e + L.h; cols = h; ld = s->ld_h; break;
      case MLS_T_B: src = e + L.b; cols = h; ld = s->ld_h; break;
      case MLS_T_GU: src = e + L.gu; cols = 2 * f; ld = s->ld_gu; break;
      case MLS_T_Z: src = e + L.z; cols = f; ld = s->ld_f; break;
      case MLS_T_LSE:
        HIP_TRY(hipMemcpyAsync(dst, e + L.lse, size_t(s->c.micro_batch) * s->c.n_q_heads * s->c.seq * 4,
                               hipMemcpyDeviceToDevice, s->st));
        HIP_TRY(hipStreamSynchronize(s->st));
        return MLS_OK;
      default: return fail(MLS_E_RANGE, "unknown tensor id");
    }
  }
  if ((id == MLS_T_GU || id == MLS_T_DGU) && s->fuse_gu)  // dst is dense and in the public column order
    HIP_TRY(mls::gu_permute(src, ld, dst, cols, T, s->c.ffn, false, s->st));
  else
    HIP_TRY(copy2d(s, dst, cols, src, ld, T, cols));
  HIP_TRY(hipStreamSynchronize(s->st));
  return MLS_OK;
}

int mls_stage_timing(mls_stage* s, int32_t enable) {
  if (!s) return fail(MLS_E_NULL, "null handle");
  if (enable && s->tm.ev.empty()) {
    s->tm.ev.resize(2 * 4096);
    s->tm.cls.resize(4096);
    for (auto& e : s->tm.ev) HIP_TRY(hipEventCreate(&e));
  }
  if (!enable) HIP_TRY(s->tm.flush());
  s->tm.on = enable != 0;
  return MLS_OK;
}

int mls_stage_timing_read(mls_stage* s, double* ms, int64_t* launches) {
  if (!s || !ms || !launches) return fail(MLS_E_NULL, "mls_stage_timing_read: null argument");
  HIP_TRY(s->tm.flush());
  for (int i = 0; i < CLS_COUNT; i++) {
    ms[i] = s->tm.ms[i];
    launches[i] = s->tm.launches[i];
    s->tm.ms[i] = 0;
    s->tm.launches[i] = 0;
  }
  return MLS_OK;
}

int mls_gemm(int32_t dtype, int32_t mode, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
             const void* R, int64_t M, int64_t N, int64_t K, void* hip_stream) {
  if (!A || !B || !C) return fail(MLS_E_NULL, "mls_gemm: null argument");
  if (dtype != MLS_BF16 && dtype != MLS_FP32) return fail(MLS_E_CONFIG, "mls_gemm: bad dtype");
  if (mode < 0 || mode > 2) return fail(MLS_E_CONFIG, "mls_gemm: mode must be 0, 1 or 2");
  if (M < 0 || N < 0 || K < 0 || M % 8 || N % 8 || K % 8 || M > (1 << 24) || N > (1 << 24) || K > (1 << 24))
    return fail(MLS_E_CONFIG, "mls_gemm: dimensions must be non-negative multiples of 8 below 2^24");
  const int64_t a_len = mode == mls::GEMM_TN ? M : K, b_len = mode == mls::GEMM_NT ? K : N;
  if ((uintptr_t(A) | uintptr_t(B) | uintptr_t(C) | uintptr_t(R)) & 15)
    return fail(MLS_E_CONFIG, "mls_gemm: operands must be 16-byte aligned");
  if (lda == 0) lda = a_len;
  if (ldb == 0) ldb = b_len;
  if (ldc == 0) ldc = N;
  if (lda < a_len || ldb < b_len || ldc < N || lda % 8 || ldb % 8 || ldc % 8)
    return fail(MLS_E_CONFIG, "mls_gemm: a row stride must be a multiple of 8 not below the row length");
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e = dtype == MLS_BF16 ? mls::gemm_bf16(mode, A, B, C, R, (int)M, (int)N, (int)K, lda, ldb, ldc, ldc, st)
                                   : mls::gemm_f32(mode, A, B, C, R, (int)M, (int)N, (int)K, lda, ldb, ldc, ldc, st);
  if (e != hipSuccess) return fail_hip(e, "mls_gemm launch");
  return MLS_OK;
}

}  // extern "C"
