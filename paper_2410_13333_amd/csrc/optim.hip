// Optimizer step (AdamW on fp32 master weights) and the straggling-rate probe; C ABI in include/mls_optim.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <string>

#include "../../include/mls.h"
#include "../../include/mls_optim.h"
#include "common.h"
#include "kernels.h"

namespace {

constexpr int TH = 256;

// master <- storage-type parameters; moments <- 0 (8 elements per thread)
template <typename T>
__global__ __launch_bounds__(TH) void optim_init_kernel(const T* __restrict__ p, float* __restrict__ w, float* __restrict__ m,
                                                        float* __restrict__ v, size_t n8) {
  const size_t i = size_t(blockIdx.x) * TH + threadIdx.x;
  if (i >= n8) return;
  float x[8], z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  load8(p + i * 8, x);
  store8(w + i * 8, x);
  store8(m + i * 8, z);
  store8(v + i * 8, z);
}

// One AdamW step over 8 parameters per thread.  c1 = 1 / (1 - beta1^t), c2 = 1 / (1 - beta2^t).
template <typename T>
__global__ __launch_bounds__(TH) void adamw_kernel(float* __restrict__ w, float* __restrict__ m, float* __restrict__ v,
                                                   const float* __restrict__ g, T* __restrict__ out, size_t n8, float gs,
                                                   float lr, float b1, float b2, float eps, float wd, float c1, float c2) {
  const size_t i = size_t(blockIdx.x) * TH + threadIdx.x;
  if (i >= n8) return;
  float wv[8], mv[8], vv[8], gv[8];
  load8(w + i * 8, wv);
  load8(m + i * 8, mv);
  load8(v + i * 8, vv);
  load8(g + i * 8, gv);
#pragma unroll
  for (int e = 0; e < 8; e++) {
    const float gr = gs * gv[e];
    mv[e] = b1 * mv[e] + (1.f - b1) * gr;
    vv[e] = b2 * vv[e] + (1.f - b2) * gr * gr;
    wv[e] -= lr * ((mv[e] * c1) / (sqrtf(vv[e] * c2) + eps) + wd * wv[e]);
  }
  store8(w + i * 8, wv);
  store8(m + i * 8, mv);
  store8(v + i * 8, vv);
  store8(out + i * 8, wv);
}

int fail(int code, const std::string& msg) { return mls::set_error(code, msg.c_str()); }
int fail_hip(hipError_t e, const char* what) {
  return fail(e == hipErrorOutOfMemory ? MLS_E_NOMEM : MLS_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) return fail_hip(e_, #expr);   \
  } while (0)

}  // namespace

struct mls_optim {
  size_t n = 0;
  int dt = 0;
  hipStream_t st = nullptr;
  float *w = nullptr, *m = nullptr, *v = nullptr;
  int64_t t = 0;
};

struct mls_probe {
  double tau_ref = 0, threshold = 0, prev = 0, last_rate = 0, last_tau = 0;
  bool have_prev = false, pending = false, have_last = false;
  int last_shift = 0;
  int64_t units = 0;
  hipStream_t st = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
};

namespace {

void release(mls_optim* o) {
  for (float* p : {o->w, o->m, o->v})
    if (p) (void)hipFree(p);
  delete o;
}

// the shift rule on a new rate
void judge(mls_probe* p, double rate, double tau) {
  p->last_shift = p->have_prev && std::fabs(rate - p->prev) / p->prev > p->threshold ? 1 : 0;
  p->prev = rate;
  p->have_prev = true;
  p->last_rate = rate;
  p->last_tau = tau;
  p->have_last = true;
}

}  // namespace

extern "C" {

int mls_optim_init(size_t n, const void* params, int32_t dtype, void* hip_stream, mls_optim** out) {
  if (!params || !out) return fail(MLS_E_NULL, "mls_optim_init: null argument");
  *out = nullptr;
  if (dtype != MLS_BF16 && dtype != MLS_FP32) return fail(MLS_E_CONFIG, "dtype must be MLS_BF16 or MLS_FP32");
  if (n == 0 || n % 8) return fail(MLS_E_CONFIG, "the parameter count must be a positive multiple of 8");
  if (uintptr_t(params) & 15) return fail(MLS_E_CONFIG, "mls_optim_init: params must be 16-byte aligned");
  mls_optim* o = new mls_optim();
  o->n = n;
  o->dt = dtype == MLS_BF16 ? mls::DT_BF16 : mls::DT_FP32;
  o->st = (hipStream_t)hip_stream;
  hipError_t e;
  if ((e = hipMalloc((void**)&o->w, n * 4)) != hipSuccess || (e = hipMalloc((void**)&o->m, n * 4)) != hipSuccess ||
      (e = hipMalloc((void**)&o->v, n * 4)) != hipSuccess) {
    release(o);
    return fail_hip(e, "hipMalloc");
  }
  const size_t n8 = n / 8;
  const unsigned blocks = unsigned((n8 + TH - 1) / TH);
  if (o->dt == mls::DT_BF16)
    hipLaunchKernelGGL(optim_init_kernel<bf16_t>, dim3(blocks), dim3(TH), 0, o->st, (const bf16_t*)params, o->w, o->m, o->v, n8);
  else
    hipLaunchKernelGGL(optim_init_kernel<float>, dim3(blocks), dim3(TH), 0, o->st, (const float*)params, o->w, o->m, o->v, n8);
  if ((e = hipGetLastError()) != hipSuccess || (e = hipStreamSynchronize(o->st)) != hipSuccess) {
    release(o);
    return fail_hip(e, "optimizer state initialisation");
  }
  *out = o;
  return MLS_OK;
}

void mls_optim_free(mls_optim* o) {
  if (!o) return;
  (void)hipStreamSynchronize(o->st);
  release(o);
}

int mls_optim_step(mls_optim* o, const float* grads, const mls_adamw* hp, float grad_scale, void* params_out) {
  if (!o || !grads || !hp || !params_out) return fail(MLS_E_NULL, "mls_optim_step: null argument");
  if ((uintptr_t(grads) | uintptr_t(params_out)) & 15) return fail(MLS_E_CONFIG, "mls_optim_step: grads and params_out must be 16-byte aligned");
  if (!(hp->lr >= 0.f) || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) ||
      !(hp->eps >= 0.f) || !(hp->weight_decay >= 0.f))
    return fail(MLS_E_CONFIG, "mls_optim_step: need lr, eps, weight_decay >= 0 and betas in [0, 1)");
  o->t++;
  const float c1 = float(1.0 / (1.0 - std::pow((double)hp->beta1, (double)o->t)));
  const float c2 = float(1.0 / (1.0 - std::pow((double)hp->beta2, (double)o->t)));
  const size_t n8 = o->n / 8;
  const unsigned blocks = unsigned((n8 + TH - 1) / TH);
  if (o->dt == mls::DT_BF16)
    hipLaunchKernelGGL(adamw_kernel<bf16_t>, dim3(blocks), dim3(TH), 0, o->st, o->w, o->m, o->v, grads, (bf16_t*)params_out, n8,
                       grad_scale, hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, c1, c2);
  else
    hipLaunchKernelGGL(adamw_kernel<float>, dim3(blocks), dim3(TH), 0, o->st, o->w, o->m, o->v, grads, (float*)params_out, n8,
                       grad_scale, hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, c1, c2);
  HIP_TRY(hipGetLastError());
  return MLS_OK;
}

int64_t mls_optim_steps(const mls_optim* o) { return o ? o->t : 0; }

int mls_optim_read(mls_optim* o, int32_t which, float* dst) {
  if (!o || !dst) return fail(MLS_E_NULL, "mls_optim_read: null argument");
  if (which < 0 || which > 2) return fail(MLS_E_RANGE, "mls_optim_read: which must be 0 (weights), 1 or 2 (moments)");
  const float* src = which == 0 ? o->w : which == 1 ? o->m : o->v;
  HIP_TRY(hipMemcpyAsync(dst, src, o->n * 4, hipMemcpyDeviceToDevice, o->st));
  HIP_TRY(hipStreamSynchronize(o->st));
  return MLS_OK;
}

int mls_probe_init(double tau_ref_ms, double threshold, void* hip_stream, mls_probe** out) {
  if (!out) return fail(MLS_E_NULL, "mls_probe_init: null argument");
  *out = nullptr;
  if (!(tau_ref_ms > 0) || !(threshold >= 0)) return fail(MLS_E_CONFIG, "mls_probe_init: need tau_ref_ms > 0 and threshold >= 0");
  mls_probe* p = new mls_probe();
  p->tau_ref = tau_ref_ms;
  p->threshold = threshold;
  p->st = (hipStream_t)hip_stream;  // the events are created by the first mls_probe_begin: replaying needs no GPU
  *out = p;
  return MLS_OK;
}

void mls_probe_free(mls_probe* p) {
  if (!p) return;
  if (p->e0) (void)hipEventDestroy(p->e0);
  if (p->e1) (void)hipEventDestroy(p->e1);
  delete p;
}

int mls_probe_begin(mls_probe* p) {
  if (!p) return fail(MLS_E_NULL, "mls_probe_begin: null handle");
  if (!p->e0) HIP_TRY(hipEventCreate(&p->e0));
  if (!p->e1) HIP_TRY(hipEventCreate(&p->e1));
  HIP_TRY(hipEventRecord(p->e0, p->st));
  return MLS_OK;
}

int mls_probe_end(mls_probe* p, int32_t layers, int32_t microbatches) {
  if (!p) return fail(MLS_E_NULL, "mls_probe_end: null handle");
  if (layers < 0 || microbatches < 0) return fail(MLS_E_RANGE, "mls_probe_end: negative count");
  if (!p->e1) return fail(MLS_E_RANGE, "mls_probe_end without mls_probe_begin");
  HIP_TRY(hipEventRecord(p->e1, p->st));
  p->units = int64_t(layers) * microbatches;
  p->pending = true;
  return MLS_OK;
}

int mls_probe_read(mls_probe* p, double* rate, double* tau_ms, int32_t* shift) {
  if (!p) return fail(MLS_E_NULL, "mls_probe_read: null handle");
  if (p->pending) {
    if (p->units == 0) return fail(MLS_E_RANGE, "mls_probe_read: the bracketed step held no work (layers x micro-batches = 0)");
    HIP_TRY(hipEventSynchronize(p->e1));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, p->e0, p->e1));
    const double tau = double(ms) / double(p->units);
    judge(p, tau / p->tau_ref, tau);
    p->pending = false;
  }
  if (!p->have_last) return fail(MLS_E_RANGE, "mls_probe_read: no step has been bracketed");
  if (rate) *rate = p->last_rate;
  if (tau_ms) *tau_ms = p->last_tau;
  if (shift) *shift = p->last_shift;
  return MLS_OK;
}

int mls_probe_feed(mls_probe* p, double elapsed_ms, int32_t layers, int32_t microbatches, double* rate, int32_t* shift) {
  if (!p) return fail(MLS_E_NULL, "mls_probe_feed: null handle");
  const int64_t units = int64_t(layers) * microbatches;
  if (layers < 0 || microbatches < 0 || units == 0 || !(elapsed_ms >= 0))
    return fail(MLS_E_RANGE, "mls_probe_feed: need layers x micro-batches > 0 and elapsed_ms >= 0");
  const double tau = elapsed_ms / double(units);
  judge(p, tau / p->tau_ref, tau);
  if (rate) *rate = p->last_rate;
  if (shift) *shift = p->last_shift;
  return MLS_OK;
}

}  // extern "C"
