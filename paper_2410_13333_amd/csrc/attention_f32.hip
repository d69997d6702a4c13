// fp32 causal attention for the all-fp32 validation mode (tiny shapes): one thread per query row (forward,
// dQ) or per key row (dK, dV), online softmax in the forward, scalar loops, no atomics.  Also holds the
// delta_i = sum_c dO[i,c]*O[i,c] kernel that both storage types share.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int DMAX = 128;

__global__ __launch_bounds__(64) void attn_fwd_f32_kernel(const float* __restrict__ qkv, int64_t ld,
                                                          float* __restrict__ o, int64_t ldo, float* __restrict__ lse,
                                                          int b, int S, int nq, int nkv, int d) {
  const int64_t id = int64_t(blockIdx.x) * 64 + threadIdx.x;
  if (id >= int64_t(b) * nq * S) return;
  const int i = int(id % S), hq = int((id / S) % nq), bi = int(id / (int64_t(S) * nq));
  const int hk = hq / (nq / nkv);
  const float* q = qkv + (int64_t(bi) * S + i) * ld + hq * d;
  const float* kb = qkv + int64_t(bi) * S * ld + int64_t(nq + hk) * d;
  const float* vb = kb + int64_t(nkv) * d;
  const float scale = rsqrtf((float)d);
  float qr[DMAX], acc[DMAX];
#pragma unroll
  for (int c = 0; c < DMAX; c++) { qr[c] = c < d ? q[c] : 0.f; acc[c] = 0.f; }
  float m = -INFINITY, l = 0.f;
  for (int j = 0; j <= i; j++) {
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < DMAX; c++) if (c < d) s += qr[c] * kb[j * ld + c];
    s *= scale;
    const float mn = fmaxf(m, s), corr = __expf(m - mn), p = __expf(s - mn);
    l = l * corr + p;
#pragma unroll
    for (int c = 0; c < DMAX; c++) if (c < d) acc[c] = acc[c] * corr + p * vb[j * ld + c];
    m = mn;
  }
  float* orow = o + (int64_t(bi) * S + i) * ldo + hq * d;
#pragma unroll
  for (int c = 0; c < DMAX; c++) if (c < d) orow[c] = acc[c] / l;
  lse[(int64_t(bi) * nq + hq) * S + i] = m + __logf(l);
}

template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(const T* __restrict__ o, int64_t ldo,
                                                         const T* __restrict__ d_o, int64_t ldd,
                                                         float* __restrict__ delta, int b, int S, int nq, int d) {
  // 16 lanes per (token, head) row of d <= 128 elements, 8 elements per lane: four rows per wavefront
  const int64_t w = (int64_t(blockIdx.x) * 256 + threadIdx.x) >> 4;
  const int c = (threadIdx.x & 15) * 8;
  const bool live = w < int64_t(b) * S * nq;
  const int hq = live ? int(w % nq) : 0;
  const int64_t t = live ? w / nq : 0;
  float s = 0.f;
  if (live && c < d) {
    float a[8], g[8];
    load8(o + t * ldo + hq * d + c, a);
    load8(d_o + t * ldd + hq * d + c, g);
#pragma unroll
    for (int e = 0; e < 8; e++) s += a[e] * g[e];
  }
#pragma unroll
  for (int m = 8; m > 0; m >>= 1) s += __shfl_xor(s, m, 64);
  if (live && c == 0) delta[(int64_t(t / S) * nq + hq) * S + (t % S)] = s;
}

__global__ __launch_bounds__(64) void attn_dq_f32_kernel(const float* __restrict__ qkv, int64_t ld,
                                                         const float* __restrict__ lse, const float* __restrict__ d_o,
                                                         int64_t ldd, const float* __restrict__ delta,
                                                         float* __restrict__ dqkv, int64_t ldg, int b, int S, int nq,
                                                         int nkv, int d) {
  const int64_t id = int64_t(blockIdx.x) * 64 + threadIdx.x;
  if (id >= int64_t(b) * nq * S) return;
  const int i = int(id % S), hq = int((id / S) % nq), bi = int(id / (int64_t(S) * nq));
  const int hk = hq / (nq / nkv);
  const float* q = qkv + (int64_t(bi) * S + i) * ld + hq * d;
  const float* kb = qkv + int64_t(bi) * S * ld + int64_t(nq + hk) * d;
  const float* vb = kb + int64_t(nkv) * d;
  const float* dor = d_o + (int64_t(bi) * S + i) * ldd + hq * d;
  const float scale = rsqrtf((float)d);
  const float L = lse[(int64_t(bi) * nq + hq) * S + i], D = delta[(int64_t(bi) * nq + hq) * S + i];
  float qr[DMAX], dr[DMAX], acc[DMAX];
#pragma unroll
  for (int c = 0; c < DMAX; c++) { qr[c] = c < d ? q[c] : 0.f; dr[c] = c < d ? dor[c] : 0.f; acc[c] = 0.f; }
  for (int j = 0; j <= i; j++) {
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int c = 0; c < DMAX; c++) if (c < d) { s += qr[c] * kb[j * ld + c]; dp += dr[c] * vb[j * ld + c]; }
    const float p = __expf(s * scale - L);
    const float ds = p * (dp - D) * scale;
#pragma unroll
    for (int c = 0; c < DMAX; c++) if (c < d) acc[c] += ds * kb[j * ld + c];
  }
  float* out = dqkv + (int64_t(bi) * S + i) * ldg + hq * d;
#pragma unroll
  for (int c = 0; c < DMAX; c++) if (c < d) out[c] = acc[c];
}

__global__ __launch_bounds__(64) void attn_dkv_f32_kernel(const float* __restrict__ qkv, int64_t ld,
                                                          const float* __restrict__ lse, const float* __restrict__ d_o,
                                                          int64_t ldd, const float* __restrict__ delta,
                                                          float* __restrict__ dqkv, int64_t ldg, int b, int S, int nq,
                                                          int nkv, int d) {
  const int64_t id = int64_t(blockIdx.x) * 64 + threadIdx.x;
  if (id >= int64_t(b) * nkv * S) return;
  const int j = int(id % S), hk = int((id / S) % nkv), bi = int(id / (int64_t(S) * nkv));
  const int grp = nq / nkv;
  const float* kr_ = qkv + (int64_t(bi) * S + j) * ld + int64_t(nq + hk) * d;
  const float* vr_ = kr_ + int64_t(nkv) * d;
  const float scale = rsqrtf((float)d);
  float kr[DMAX], vr[DMAX], dk[DMAX], dv[DMAX];
#pragma unroll
  for (int c = 0; c < DMAX; c++) { kr[c] = c < d ? kr_[c] : 0.f; vr[c] = c < d ? vr_[c] : 0.f; dk[c] = 0.f; dv[c] = 0.f; }
  for (int hq = hk * grp; hq < (hk + 1) * grp; hq++) {
    for (int i = j; i < S; i++) {
      const float* q = qkv + (int64_t(bi) * S + i) * ld + hq * d;
      const float* dor = d_o + (int64_t(bi) * S + i) * ldd + hq * d;
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int c = 0; c < DMAX; c++) if (c < d) { s += q[c] * kr[c]; dp += dor[c] * vr[c]; }
      const int64_t si = (int64_t(bi) * nq + hq) * S + i;
      const float p = __expf(s * scale - lse[si]);
      const float ds = p * (dp - delta[si]) * scale;
#pragma unroll
      for (int c = 0; c < DMAX; c++) if (c < d) { dv[c] += p * dor[c]; dk[c] += ds * q[c]; }
    }
  }
  float* ok = dqkv + (int64_t(bi) * S + j) * ldg + int64_t(nq + hk) * d;
  float* ov = ok + int64_t(nkv) * d;
#pragma unroll
  for (int c = 0; c < DMAX; c++) if (c < d) { ok[c] = dk[c]; ov[c] = dv[c]; }
}

}  // namespace

namespace mls {

hipError_t attn_delta(int dt, const void* o, int64_t ld_o, const void* d_o, int64_t ld_do, float* delta, int b, int S,
                      int nq, int d, hipStream_t st) {
  const int64_t waves = int64_t(b) * S * nq;
  if (waves == 0) return hipSuccess;
  const int blocks = int((waves * 16 + 255) / 256);  // 16 lanes per row
  if (dt == DT_BF16)
    hipLaunchKernelGGL(attn_delta_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t*)o, ld_o,
                       (const bf16_t*)d_o, ld_do, delta, b, S, nq, d);
  else
    hipLaunchKernelGGL(attn_delta_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)o, ld_o,
                       (const float*)d_o, ld_do, delta, b, S, nq, d);
  return hipGetLastError();
}

hipError_t attn_fwd_f32(const void* qkv, int64_t ld_qkv, void* o, int64_t ld_o, float* lse, int b, int S, int nq, int nkv,
                        int d, hipStream_t st) {
  const int64_t n = int64_t(b) * nq * S;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(attn_fwd_f32_kernel, dim3(int((n + 63) / 64)), dim3(64), 0, st, (const float*)qkv, ld_qkv, (float*)o,
                     ld_o, lse, b, S, nq, nkv, d);
  return hipGetLastError();
}

hipError_t attn_bwd_f32(const void* qkv, int64_t ld_qkv, const void* o, int64_t ld_o, const float* lse, const void* d_o,
                        int64_t ld_do, void* dqkv, int64_t ld_dqkv, float* delta, int b, int S, int nq, int nkv, int d,
                        hipStream_t st) {
  const int64_t n = int64_t(b) * nq * S, nk = int64_t(b) * nkv * S;
  if (n == 0) return hipSuccess;
  hipError_t e = attn_delta(DT_FP32, o, ld_o, d_o, ld_do, delta, b, S, nq, d, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_dq_f32_kernel, dim3(int((n + 63) / 64)), dim3(64), 0, st, (const float*)qkv, ld_qkv, lse,
                     (const float*)d_o, ld_do, delta, (float*)dqkv, ld_dqkv, b, S, nq, nkv, d);
  hipLaunchKernelGGL(attn_dkv_f32_kernel, dim3(int((nk + 63) / 64)), dim3(64), 0, st, (const float*)qkv, ld_qkv, lse,
                     (const float*)d_o, ld_do, delta, (float*)dqkv, ld_dqkv, b, S, nq, nkv, d);
  return hipGetLastError();
}

}  // namespace mls
