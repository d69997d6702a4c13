// First/last-stage layers (include/mls_ends.h): token embedding gather and its deterministic scatter-add backward;
// final RMSNorm, LM head and mean cross-entropy with the logits gradient formed in place of the logits.  The
// contractions and the RMSNorm are the kernels of the decoder stage; the kernels here are the HBM-bound rest.
#include <hip/hip_runtime.h>

#include <mutex>
#include <string>
#include <vector>

#include "../../include/mls.h"
#include "../../include/mls_ends.h"
#include "common.h"
#include "kernels.h"

namespace {

constexpr int TH = 256;
constexpr int MAX_MB = 16;  // micro-batches one scatter launch covers

// ---- x[t, :] = embed[tokens[t], :] (zero row for an id outside the table); one thread per 8 columns
template <typename T>
__global__ __launch_bounds__(TH) void embed_gather_kernel(const int32_t* __restrict__ tok, const T* __restrict__ E,
                                                          int64_t ld_e, T* __restrict__ x, int64_t total, int h,
                                                          int V) {
  const int64_t id = int64_t(blockIdx.x) * TH + threadIdx.x;
  if (id >= total) return;
  const int cpr = h >> 3;
  const int64_t t = id / cpr;
  const int c = int(id % cpr) * 8;
  const int v = tok[t];
  float val[8];
  if (v >= 0 && v < V) {
    load8(E + int64_t(v) * ld_e + c, val);
  } else {
#pragma unroll
    for (int e = 0; e < 8; e++) val[e] = 0.f;
  }
  store8(x + t * h + c, val);
}

// ---- grads_embed[v, :] += sum of the dX rows at the positions that hold token v, in ascending (micro-batch,
// position) order.  One workgroup per table row: it scans the token ids 256 at a time, shares the match masks
// through LDS and then every thread walks the matches in order for its own columns.  No atomics: each table row
// has one owner, so the result is bitwise reproducible.
struct TokPtrs { const int32_t* p[MAX_MB]; };
template <typename T, int MAXC>
__global__ __launch_bounds__(TH) void embed_scatter_kernel(TokPtrs tp, int n, const T* __restrict__ dX, int Ttok, int h,
                                                           float* __restrict__ gE) {
  __shared__ unsigned long long masks[TH / 64];
  const int v = blockIdx.x, cpr = h >> 3;
  float acc[MAXC][8];
#pragma unroll
  for (int i = 0; i < MAXC; i++)
#pragma unroll
    for (int e = 0; e < 8; e++) acc[i][e] = 0.f;
  bool any = false;
  for (int mb = 0; mb < n; mb++) {
    const int32_t* tok = tp.p[mb];
    for (int base = 0; base < Ttok; base += TH) {
      const int pos = base + threadIdx.x;
      const unsigned long long m = __ballot(pos < Ttok && tok[pos] == v);
      if ((threadIdx.x & 63) == 0) masks[threadIdx.x >> 6] = m;
      __syncthreads();
#pragma unroll
      for (int w = 0; w < TH / 64; w++) {
        unsigned long long mm = masks[w];
        while (mm) {
          const int bit = __ffsll((long long)mm) - 1;
          mm &= mm - 1;
          any = true;
          const T* row = dX + (int64_t(mb) * Ttok + base + w * 64 + bit) * h;
#pragma unroll
          for (int i = 0; i < MAXC; i++) {
            const int c = threadIdx.x + i * TH;
            if (c < cpr) {
              float d[8];
              load8(row + c * 8, d);
#pragma unroll
              for (int e = 0; e < 8; e++) acc[i][e] += d[e];
            }
          }
        }
      }
      __syncthreads();
    }
  }
  if (!any) return;
#pragma unroll
  for (int i = 0; i < MAXC; i++) {
    const int c = threadIdx.x + i * TH;
    if (c < cpr) {
      float g[8];
      float* p = gE + int64_t(v) * h + c * 8;
      load8(p, g);
#pragma unroll
      for (int e = 0; e < 8; e++) g[e] += acc[i][e];
      store8(p, g);
    }
  }
}

// ---- cross-entropy of one row of logits per workgroup, and its gradient in place:
//   pass 1 (from HBM): running maximum and sum of exponentials per thread, merged across the workgroup;
//   pass 2 (the row is 64 KB or so: from L2): logits <- scale * (exp(logit - lse) - [column == target]).
// An ignored target (outside [0, V)) gives loss 0 and a zero row.
template <typename T>
__global__ __launch_bounds__(TH) void ce_kernel(T* __restrict__ logits, int64_t ld, const int32_t* __restrict__ targets,
                                                int V, float scale, float* __restrict__ row_loss) {
  __shared__ float sm[TH / 64], ss[TH / 64];
  __shared__ float s_lse;
  const int64_t t = blockIdx.x;
  T* row = logits + t * ld;
  const int tgt = targets[t];
  const bool valid = tgt >= 0 && tgt < V;
  const int cpr = V >> 3;
  float m = -INFINITY, s = 0.f;
  for (int c = threadIdx.x; c < cpr; c += TH) {
    float x[8];
    load8(row + c * 8, x);
    float cm = x[0];
#pragma unroll
    for (int e = 1; e < 8; e++) cm = fmaxf(cm, x[e]);
    const float nm = fmaxf(m, cm);
    float add = 0.f;
#pragma unroll
    for (int e = 0; e < 8; e++) add += __expf(x[e] - nm);
    s = s * __expf(m - nm) + add;  // exp(-inf) = 0 on the first chunk
    m = nm;
  }
  // merge (m, s) pairs: lanes, then wavefronts
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float om = __shfl_xor(m, o, 64), os = __shfl_xor(s, o, 64);
    const float nm = fmaxf(m, om);
    s = (m == -INFINITY ? 0.f : s * __expf(m - nm)) + (om == -INFINITY ? 0.f : os * __expf(om - nm));
    m = nm;
  }
  if ((threadIdx.x & 63) == 0) {
    sm[threadIdx.x >> 6] = m;
    ss[threadIdx.x >> 6] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = sm[0], S = ss[0];
#pragma unroll
    for (int w = 1; w < TH / 64; w++) {
      const float nm = fmaxf(M, sm[w]);
      S = (M == -INFINITY ? 0.f : S * __expf(M - nm)) + (sm[w] == -INFINITY ? 0.f : ss[w] * __expf(sm[w] - nm));
      M = nm;
    }
    const float lse = M + logf(S);
    s_lse = lse;
    row_loss[t] = valid ? lse - to_f32(row[tgt]) : 0.f;  // read before pass 2 overwrites the row
  }
  __syncthreads();
  const float lse = s_lse;
  for (int c = threadIdx.x; c < cpr; c += TH) {
    float x[8], g[8];
    load8(row + c * 8, x);
#pragma unroll
    for (int e = 0; e < 8; e++) g[e] = valid ? scale * (__expf(x[e] - lse) - (c * 8 + e == tgt ? 1.f : 0.f)) : 0.f;
    store8(row + c * 8, g);
  }
}

// ---- out[0] = (sum of v[0..n)) / n, one workgroup, fixed summation tree
__global__ __launch_bounds__(1024) void mean_kernel(const float* __restrict__ v, int n, float* __restrict__ out) {
  __shared__ float red[16];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 1024) s += v[i];
  s = block_sum(s, red);
  if (threadIdx.x == 0) out[0] = s / (float)n;
}

inline int blocks_for(int64_t n) { return int((n + TH - 1) / TH); }
size_t align256(size_t v) { return (v + 255) & ~size_t(255); }
int64_t padded(int64_t n) { return n % 256 == 0 ? n + 64 : n; }

}  // namespace

// ---- Scratch of mls_head_forward_static: the per-token loss terms between the cross-entropy kernel and the mean.
// One array per GPU (every device that loads this code object holds its own copy until the process ends).  In host
// code the array's name is only a handle for hipGetSymbolAddress; the device address is looked up once per device,
// with that device current, and kernels get that address as an argument.
constexpr int STATIC_TOKENS = 65536;  // 256 KiB
static __device__ __align__(256) float scratch[STATIC_TOKENS];
namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
float* g_scratch_ptr[MAX_DEVICES] = {};
// device address of `scratch` on the current device (looked up on first use there)
hipError_t scratch_address(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    if ((e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch))) != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace

struct mls_ends {
  mls_ends_config c;
  int dt, es, T;
  hipStream_t st;
  int64_t ld_h, ld_v;
  size_t off_e, off_g, off_w, n_params;  // public offsets (= layout of grads)
  char *embed = nullptr, *gamma = nullptr, *wlm = nullptr;  // internal: embed [V, ld_h], gamma [h], w_lm [h, ld_v]
  // bf16 storage: w_lm transposed, [V, ld_h], for the forward product (both operands stored along the contraction
  // index is the fastest form of the bf16 GEMM); rewritten whenever the parameters are set
  char* wlm_t = nullptr;
  int32_t* tok = nullptr;  // [max_inflight, T]
  int e_head = 0, e_count = 0;
  // head stash, one entry per kept micro-batch
  char *y = nullptr, *nrm = nullptr, *dlog = nullptr;
  float* r = nullptr;
  size_t mb_h = 0, mb_v = 0;
  int h_head = 0, h_count = 0;
  // workspace
  char* dn = nullptr;
  float *partial = nullptr, *row_loss = nullptr;
};

namespace {

int fail(int code, const std::string& msg) { return mls::set_error(code, msg.c_str()); }
int fail_hip(hipError_t e, const char* what) {
  return fail(e == hipErrorOutOfMemory ? MLS_E_NOMEM : MLS_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) return fail_hip(e_, #expr);   \
  } while (0)

hipError_t copy2d(const mls_ends* s, void* dst, int64_t ld_dst, const void* src, int64_t ld_src, int64_t rows,
                  int64_t cols) {
  return hipMemcpy2DAsync(dst, size_t(ld_dst) * s->es, src, size_t(ld_src) * s->es, size_t(cols) * s->es, size_t(rows),
                          hipMemcpyDeviceToDevice, s->st);
}

hipError_t gemm(const mls_ends* s, int mode, const void* A, const void* B, void* C, int M, int N, int K, int64_t lda,
                int64_t ldb, int64_t ldc) {
  return s->dt == mls::DT_BF16 ? mls::gemm_bf16(mode, A, B, C, nullptr, M, N, K, lda, ldb, ldc, 0, s->st)
                               : mls::gemm_f32(mode, A, B, C, nullptr, M, N, K, lda, ldb, ldc, 0, s->st);
}

void release(mls_ends* s) {
  void* p[] = {s->embed, s->gamma, s->wlm, s->wlm_t, s->tok, s->y, s->nrm, s->dlog, s->r, s->dn, s->partial, s->row_loss};
  for (void* q : p)
    if (q) (void)hipFree(q);
  delete s;
}

// the three parameter tensors: public offset, internal pointer, rows, cols, internal row stride, generator id
struct PT { size_t off; char* ptr; int64_t rows, cols, ld; uint32_t tid; double scale, offset; };
void param_tensors(const mls_ends* s, PT (&t)[3]) {
  const int64_t h = s->c.hidden, V = s->c.vocab;
  t[0] = {s->off_e, s->embed, V, h, s->ld_h, 6, 0.02, 0.0};
  t[1] = {s->off_g, s->gamma, 1, h, h, 7, 0.02, 1.0};
  t[2] = {s->off_w, s->wlm, h, V, s->ld_v, 8, 0.02, 0.0};
}

}  // namespace

extern "C" {

int mls_ends_init(const mls_ends_config* cfg, uint64_t seed, void* hip_stream, mls_ends** out) {
  if (!cfg || !out) return fail(MLS_E_NULL, "mls_ends_init: null argument");
  *out = nullptr;
  const mls_ends_config& c = *cfg;
  if (c.dtype != MLS_BF16 && c.dtype != MLS_FP32) return fail(MLS_E_CONFIG, "dtype must be MLS_BF16 or MLS_FP32");
  if (c.hidden < 8 || c.hidden % 8 || c.hidden > 16384) return fail(MLS_E_CONFIG, "hidden must be a multiple of 8 in [8, 16384]");
  if (c.vocab < 8 || c.vocab % 8) return fail(MLS_E_CONFIG, "vocab must be a positive multiple of 8");
  if (c.seq < 1 || c.micro_batch < 1 || c.max_inflight < 1) return fail(MLS_E_CONFIG, "seq, micro_batch and max_inflight must be positive");
  if (!(c.rms_eps >= 0.f)) return fail(MLS_E_CONFIG, "rms_eps >= 0 required");
  const int64_t T = int64_t(c.seq) * c.micro_batch;
  if (T > (1 << 24) || c.vocab > (1 << 24) || T * int64_t(c.vocab) > (int64_t(1) << 40))
    return fail(MLS_E_CONFIG, "tokens per micro-batch or vocabulary too large");
  mls_ends* s = new mls_ends();
  s->c = c;
  s->dt = c.dtype == MLS_BF16 ? mls::DT_BF16 : mls::DT_FP32;
  s->es = c.dtype == MLS_BF16 ? 2 : 4;
  s->T = int(T);
  s->st = (hipStream_t)hip_stream;
  s->ld_h = padded(c.hidden);
  s->ld_v = padded(c.vocab);
  const size_t h = c.hidden, V = c.vocab;
  s->off_e = 0;
  s->off_g = V * h;
  s->off_w = s->off_g + h;
  s->n_params = s->off_w + h * V;
  s->mb_h = align256(size_t(T) * s->ld_h * s->es);
  s->mb_v = align256(size_t(T) * s->ld_v * s->es);
  const size_t nmb = c.max_inflight;
  auto alloc = [&](void** p, size_t bytes) { return hipMalloc(p, bytes ? bytes : 256); };
  hipError_t e = hipSuccess;
  if ((e = alloc((void**)&s->embed, V * s->ld_h * s->es)) != hipSuccess ||
      (e = alloc((void**)&s->gamma, h * s->es)) != hipSuccess ||
      (e = alloc((void**)&s->wlm, h * s->ld_v * s->es)) != hipSuccess ||
      (s->dt == mls::DT_BF16 && (e = alloc((void**)&s->wlm_t, V * s->ld_h * s->es)) != hipSuccess) ||
      (e = alloc((void**)&s->tok, nmb * T * 4)) != hipSuccess ||
      (e = alloc((void**)&s->y, nmb * s->mb_h)) != hipSuccess ||
      (e = alloc((void**)&s->nrm, nmb * s->mb_h)) != hipSuccess ||
      (e = alloc((void**)&s->dlog, nmb * s->mb_v)) != hipSuccess ||
      (e = alloc((void**)&s->r, nmb * T * 4)) != hipSuccess ||
      (e = alloc((void**)&s->dn, s->mb_h)) != hipSuccess ||
      (e = alloc((void**)&s->partial, size_t(mls::rmsnorm_bwd_blocks(s->T)) * h * 4)) != hipSuccess ||
      (e = alloc((void**)&s->row_loss, T * 4)) != hipSuccess) {
    release(s);
    return fail_hip(e, "hipMalloc");
  }
  PT t[3];
  param_tensors(s, t);
  for (auto& q : t)
    if ((e = mls::fill_normal(s->dt, q.ptr, q.rows, q.cols, q.ld, seed, q.tid, 0, q.scale, q.offset, s->st)) != hipSuccess) {
      release(s);
      return fail_hip(e, "weight generator");
    }
  if (s->wlm_t && (e = mls::transpose_bf16(s->wlm, s->ld_v, s->wlm_t, s->ld_h, c.hidden, c.vocab, s->st)) != hipSuccess) {
    release(s);
    return fail_hip(e, "transpose_bf16");
  }
  if ((e = hipStreamSynchronize(s->st)) != hipSuccess) {
    release(s);
    return fail_hip(e, "hipStreamSynchronize");
  }
  float* sp = nullptr;  // set-up of mls_head_forward_static on this device
  if ((e = scratch_address(&sp)) != hipSuccess) {
    release(s);
    return fail_hip(e, "hipGetSymbolAddress(scratch)");
  }
  *out = s;
  return MLS_OK;
}

void mls_ends_free(mls_ends* s) {
  if (!s) return;
  (void)hipStreamSynchronize(s->st);
  release(s);
}

int mls_embed_forward(mls_ends* s, const int32_t* tokens, void* x) {
  if (!s || !tokens || !x) return fail(MLS_E_NULL, "mls_embed_forward: null argument");
  if ((uintptr_t(tokens) & 3) || (uintptr_t(x) & 15)) return fail(MLS_E_CONFIG, "mls_embed_forward: x must be 16-byte aligned");
  if (s->e_count >= s->c.max_inflight) return fail(MLS_E_STASH, "embedding stash full: max_inflight micro-batches already forwarded");
  const int slot = (s->e_head + s->e_count) % s->c.max_inflight;
  HIP_TRY(hipMemcpyAsync(s->tok + size_t(slot) * s->T, tokens, size_t(s->T) * 4, hipMemcpyDeviceToDevice, s->st));
  const int64_t total = int64_t(s->T) * (s->c.hidden >> 3);
  if (s->dt == mls::DT_BF16)
    hipLaunchKernelGGL(embed_gather_kernel<bf16_t>, dim3(blocks_for(total)), dim3(TH), 0, s->st, tokens,
                       (const bf16_t*)s->embed, s->ld_h, (bf16_t*)x, total, s->c.hidden, s->c.vocab);
  else
    hipLaunchKernelGGL(embed_gather_kernel<float>, dim3(blocks_for(total)), dim3(TH), 0, s->st, tokens,
                       (const float*)s->embed, s->ld_h, (float*)x, total, s->c.hidden, s->c.vocab);
  HIP_TRY(hipGetLastError());
  s->e_count++;
  return MLS_OK;
}

int mls_embed_backward(mls_ends* s, const void* dX, float* grads, int32_t n) {
  if (!s) return fail(MLS_E_NULL, "mls_embed_backward: null handle");
  if (n < 0) return fail(MLS_E_RANGE, "n_microbatches must be >= 0");
  if (n == 0) return MLS_OK;
  if (!dX || !grads) return fail(MLS_E_NULL, "mls_embed_backward: null argument");
  if ((uintptr_t(dX) | uintptr_t(grads)) & 15) return fail(MLS_E_CONFIG, "mls_embed_backward: dX and grads must be 16-byte aligned");
  if (n > s->e_count) return fail(MLS_E_STASH, "n_microbatches exceeds the kept embedding micro-batches");
  const int h = s->c.hidden, cpr = h >> 3;
  const size_t act = size_t(s->T) * h * s->es;
  for (int i0 = 0; i0 < n; i0 += MAX_MB) {
    const int m = n - i0 < MAX_MB ? n - i0 : MAX_MB;
    TokPtrs tp = {};
    for (int i = 0; i < m; i++) tp.p[i] = s->tok + size_t((s->e_head + i0 + i) % s->c.max_inflight) * s->T;
    const char* dx = (const char*)dX + size_t(i0) * act;
    float* gE = grads + s->off_e;
#define SCATTER(TY, C)                                                                                              \
  hipLaunchKernelGGL((embed_scatter_kernel<TY, C>), dim3(s->c.vocab), dim3(TH), 0, s->st, tp, m, (const TY*)dx, s->T, h, gE)
    const int mc = cpr <= 2 * TH ? 2 : cpr <= 4 * TH ? 4 : 8;
    if (s->dt == mls::DT_BF16) {
      if (mc == 2) SCATTER(bf16_t, 2); else if (mc == 4) SCATTER(bf16_t, 4); else SCATTER(bf16_t, 8);
    } else {
      if (mc == 2) SCATTER(float, 2); else if (mc == 4) SCATTER(float, 4); else SCATTER(float, 8);
    }
#undef SCATTER
    HIP_TRY(hipGetLastError());
  }
  s->e_head = (s->e_head + n) % s->c.max_inflight;
  s->e_count -= n;
  return MLS_OK;
}

// row_loss: T floats of scratch for the per-token loss terms (every one is written before the mean reads it)
static int head_forward(mls_ends* s, const void* y, const int32_t* targets, float loss_weight, float* loss, float* row_loss) {
  if (s->h_count >= s->c.max_inflight) return fail(MLS_E_STASH, "head stash full: max_inflight micro-batches already forwarded");
  const int slot = (s->h_head + s->h_count) % s->c.max_inflight;
  const int T = s->T, h = s->c.hidden, V = s->c.vocab;
  char* ys = s->y + size_t(slot) * s->mb_h;
  char* nr = s->nrm + size_t(slot) * s->mb_h;
  char* dl = s->dlog + size_t(slot) * s->mb_v;
  float* r = s->r + size_t(slot) * T;
  HIP_TRY(copy2d(s, ys, s->ld_h, y, h, T, h));
  HIP_TRY(mls::rmsnorm_fwd(s->dt, ys, s->ld_h, s->gamma, nr, s->ld_h, r, T, h, s->c.rms_eps, s->st));
  if (s->wlm_t) HIP_TRY(gemm(s, mls::GEMM_NT, nr, s->wlm_t, dl, T, V, h, s->ld_h, s->ld_h, s->ld_v));
  else HIP_TRY(gemm(s, mls::GEMM_NN, nr, s->wlm, dl, T, V, h, s->ld_h, s->ld_v, s->ld_v));
  const float scale = loss_weight / (float)T;
  if (s->dt == mls::DT_BF16)
    hipLaunchKernelGGL(ce_kernel<bf16_t>, dim3(T), dim3(TH), 0, s->st, (bf16_t*)dl, s->ld_v, targets, V, scale, row_loss);
  else
    hipLaunchKernelGGL(ce_kernel<float>, dim3(T), dim3(TH), 0, s->st, (float*)dl, s->ld_v, targets, V, scale, row_loss);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(1024), 0, s->st, row_loss, T, loss);
  HIP_TRY(hipGetLastError());
  s->h_count++;
  return MLS_OK;
}

int mls_head_forward(mls_ends* s, const void* y, const int32_t* targets, float loss_weight, float* loss) {
  if (!s || !y || !targets || !loss) return fail(MLS_E_NULL, "mls_head_forward: null argument");
  if (uintptr_t(y) & 15) return fail(MLS_E_CONFIG, "mls_head_forward: y must be 16-byte aligned");
  return head_forward(s, y, targets, loss_weight, loss, s->row_loss);
}

int mls_head_forward_static(mls_ends* s, const void* y, const int32_t* targets, float loss_weight, float* loss) {
  if (!s || !y || !targets || !loss) return fail(MLS_E_NULL, "mls_head_forward_static: null argument");
  if (uintptr_t(y) & 15) return fail(MLS_E_CONFIG, "mls_head_forward_static: y must be 16-byte aligned");
  if (s->T > STATIC_TOKENS)
    return fail(MLS_E_RANGE, "mls_head_forward_static: more than 65536 tokens per micro-batch (the static scratch holds 65536 loss terms)");
  float* sp = nullptr;
  if (hipError_t e = scratch_address(&sp)) return fail_hip(e, "hipGetSymbolAddress(scratch)");
  return head_forward(s, y, targets, loss_weight, loss, sp);
}

int mls_head_backward(mls_ends* s, float* grads, int32_t n, void* dY) {
  if (!s) return fail(MLS_E_NULL, "mls_head_backward: null handle");
  if (n < 0) return fail(MLS_E_RANGE, "n_microbatches must be >= 0");
  if (n == 0) return MLS_OK;
  if (!grads || !dY) return fail(MLS_E_NULL, "mls_head_backward: null argument");
  if ((uintptr_t(dY) | uintptr_t(grads)) & 15) return fail(MLS_E_CONFIG, "mls_head_backward: dY and grads must be 16-byte aligned");
  if (n > s->h_count) return fail(MLS_E_STASH, "n_microbatches exceeds the kept head micro-batches");
  const int T = s->T, h = s->c.hidden, V = s->c.vocab;
  const size_t act = size_t(T) * h * s->es;
  std::vector<const void*> an, bd;
  for (int i = 0; i < n; i++) {
    const int slot = (s->h_head + i) % s->c.max_inflight;
    const char* ys = s->y + size_t(slot) * s->mb_h;
    const char* nr = s->nrm + size_t(slot) * s->mb_h;
    const char* dl = s->dlog + size_t(slot) * s->mb_v;
    const float* r = s->r + size_t(slot) * T;
    // d nrm = dlogits w_lm^T; then the RMSNorm backward straight into the caller's dY
    HIP_TRY(gemm(s, mls::GEMM_NT, dl, s->wlm, s->dn, T, h, V, s->ld_v, s->ld_v, s->ld_h));
    HIP_TRY(mls::rmsnorm_bwd(s->dt, s->dn, s->ld_h, ys, s->ld_h, s->gamma, r, nullptr, 0, (char*)dY + size_t(i) * act, h,
                             grads + s->off_g, s->partial, T, h, s->st));
    an.push_back(nr);
    bd.push_back(dl);
  }
  // grads_w_lm += sum_i nrm_i^T dlogits_i: one contraction over all micro-batches where the DMA path can
  float* gw = grads + s->off_w;
  if (s->dt == mls::DT_BF16 && mls::gemm_tn_segments_ok(T, s->ld_h, s->ld_v)) {
    for (int i = 0; i < n; i += 16)
      HIP_TRY(mls::gemm_bf16_tn_segments(an.data() + i, bd.data() + i, n - i < 16 ? n - i : 16, gw, h, V, T, s->ld_h, s->ld_v, V, s->st));
  } else {
    for (int i = 0; i < n; i++) HIP_TRY(gemm(s, mls::GEMM_TN, an[i], bd[i], gw, h, V, T, s->ld_h, s->ld_v, V));
  }
  s->h_head = (s->h_head + n) % s->c.max_inflight;
  s->h_count -= n;
  return MLS_OK;
}

size_t mls_ends_grad_elems(const mls_ends* s) { return s ? s->n_params : 0; }

int mls_ends_param_layout(const mls_ends* s, int32_t which, size_t* offset, size_t* rows, size_t* cols) {
  if (!s || !offset || !rows || !cols) return fail(MLS_E_NULL, "mls_ends_param_layout: null argument");
  const size_t h = s->c.hidden, V = s->c.vocab;
  switch (which) {
    case MLS_PE_EMBED: *offset = s->off_e; *rows = V; *cols = h; break;
    case MLS_PE_GAMMA_F: *offset = s->off_g; *rows = 1; *cols = h; break;
    case MLS_PE_WLM: *offset = s->off_w; *rows = h; *cols = V; break;
    default: return fail(MLS_E_RANGE, "unknown parameter id");
  }
  return MLS_OK;
}

int mls_ends_get_params(mls_ends* s, void* dst) {
  if (!s || !dst) return fail(MLS_E_NULL, "mls_ends_get_params: null argument");
  PT t[3];
  param_tensors(s, t);
  for (auto& q : t) HIP_TRY(copy2d(s, (char*)dst + q.off * s->es, q.cols, q.ptr, q.ld, q.rows, q.cols));
  HIP_TRY(hipStreamSynchronize(s->st));
  return MLS_OK;
}

int mls_ends_set_params(mls_ends* s, const void* src) {
  if (!s || !src) return fail(MLS_E_NULL, "mls_ends_set_params: null argument");
  PT t[3];
  param_tensors(s, t);
  for (auto& q : t) HIP_TRY(copy2d(s, q.ptr, q.ld, (const char*)src + q.off * s->es, q.cols, q.rows, q.cols));
  if (s->wlm_t) HIP_TRY(mls::transpose_bf16(s->wlm, s->ld_v, s->wlm_t, s->ld_h, s->c.hidden, s->c.vocab, s->st));
  HIP_TRY(hipStreamSynchronize(s->st));
  return MLS_OK;
}

int mls_ends_inflight(const mls_ends* s, int32_t* embed, int32_t* head) {
  if (!s) return fail(MLS_E_NULL, "null handle");
  if (embed) *embed = s->e_count;
  if (head) *head = s->h_count;
  return MLS_OK;
}

int mls_ends_debug_dlogits(mls_ends* s, int32_t slot, void* dst) {
  if (!s || !dst) return fail(MLS_E_NULL, "mls_ends_debug_dlogits: null argument");
  if (slot < 0 || slot >= s->h_count) return fail(MLS_E_RANGE, "head stash slot out of range");
  const int phys = (s->h_head + slot) % s->c.max_inflight;
  HIP_TRY(copy2d(s, dst, s->c.vocab, s->dlog + size_t(phys) * s->mb_v, s->ld_v, s->T, s->c.vocab));
  HIP_TRY(hipStreamSynchronize(s->st));
  return MLS_OK;
}

}  // extern "C"
