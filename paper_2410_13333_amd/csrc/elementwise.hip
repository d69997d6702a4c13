// HBM-bound kernels of the decoder layer: RMSNorm forward/backward (with the residual-gradient add fused),
// rotary embedding, SwiGLU forward/backward, and the weight generator.  All use 16-byte accesses, fp32
// arithmetic and wavefront (64-lane) reductions; each tensor is read once and written once.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int EW_THREADS = 256;
// NORM_MAXC = 16-byte chunks per thread a row may span (template argument MAXC of the norm kernels):
// hidden <= MAXC * 8 * 256; instantiated for 2, 4 and 8 so that narrow rows do not pay for wide ones in registers

// ---------------------------------------------------------------- RMSNorm forward: one workgroup per row
template <typename T, int NORM_MAXC>
__global__ __launch_bounds__(EW_THREADS) void rmsnorm_fwd_kernel(const T* __restrict__ x, int64_t ldx,
                                                                 const T* __restrict__ gamma, T* __restrict__ a,
                                                                 int64_t lda, float* __restrict__ rstd, int h,
                                                                 float eps) {
  __shared__ float red[EW_THREADS / 64];
  const int64_t row = blockIdx.x;
  const T* xr = x + row * ldx;
  const int nchunk = h >> 3;
  float v[NORM_MAXC][8];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < NORM_MAXC; i++) {
    const int c = threadIdx.x + i * EW_THREADS;
    if (c < nchunk) {
      load8(xr + c * 8, v[i]);
#pragma unroll
      for (int e = 0; e < 8; e++) ss += v[i][e] * v[i][e];
    }
  }
  const float r = rsqrtf(block_sum(ss, red) / (float)h + eps);
  if (threadIdx.x == 0) rstd[row] = r;
#pragma unroll
  for (int i = 0; i < NORM_MAXC; i++) {
    const int c = threadIdx.x + i * EW_THREADS;
    if (c < nchunk) {
      float g[8], o[8];
      load8(gamma + c * 8, g);
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] = v[i][e] * r * g[e];
      store8(a + row * lda + c * 8, o);
    }
  }
}

// eight consecutive bf16 elements as they lie in memory (16 bytes), converted on demand
template <typename T>
struct Raw8;
template <>
struct Raw8<bf16_t> {
  uint4 v;
  __device__ __forceinline__ void load(const bf16_t* p) { v = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void get(float (&o)[8]) const {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
// ---------------------------------------------------------------- RMSNorm backward
// Workgroup w handles rows w, w + gridDim.x, ...; it keeps its share of the column sums for dgamma in
// registers and writes them to partial[w][:], which a second kernel adds up in a fixed order.
template <typename T, int NORM_MAXC>
__global__ __launch_bounds__(EW_THREADS) void rmsnorm_bwd_kernel(const T* __restrict__ da, int64_t ld_da,
                                                                 const T* __restrict__ x, int64_t ldx,
                                                                 const T* __restrict__ gamma,
                                                                 const float* __restrict__ rstd, const T* dres,
                                                                 int64_t ld_dres, T* dx, int64_t ld_dx,
                                                                 float* __restrict__ partial, int rows, int h,
                                                                 bool acc_partial) {
  __shared__ float red[EW_THREADS / 64];
  const int nchunk = h >> 3;
  float g[NORM_MAXC][8], dg[NORM_MAXC][8];
#pragma unroll
  for (int i = 0; i < NORM_MAXC; i++) {
    const int c = threadIdx.x + i * EW_THREADS;
#pragma unroll
    for (int e = 0; e < 8; e++) dg[i][e] = 0.f;
    if (c < nchunk) load8(gamma + c * 8, g[i]);
  }
  // bf16 rows of up to 8192 elements are software-pipelined: the (unconverted) operands of the workgroup's next
  // row are requested before the current row is reduced, so that two rows per workgroup are in flight.  Wider or
  // fp32 rows would not fit the registers that way and take the plain loop.
  if constexpr (sizeof(T) == 2 && NORM_MAXC <= 4) {
    Raw8<T> rx[NORM_MAXC], rda[NORM_MAXC], rres[NORM_MAXC];
    auto request = [&](int64_t row) {
#pragma unroll
      for (int i = 0; i < NORM_MAXC; i++) {
        const int c = threadIdx.x + i * EW_THREADS;
        if (c < nchunk) {
          rx[i].load(x + row * ldx + c * 8);
          rda[i].load(da + row * ld_da + c * 8);
          if (dres) rres[i].load(dres + row * ld_dres + c * 8);
        }
      }
    };
    if (blockIdx.x < rows) request(blockIdx.x);
    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
      const float r = rstd[row];
      float n[NORM_MAXC][8], dn[NORM_MAXC][8], res[NORM_MAXC][8];
      float dot = 0.f;
#pragma unroll
      for (int i = 0; i < NORM_MAXC; i++) {
        const int c = threadIdx.x + i * EW_THREADS;
        if (c < nchunk) {
          float xv[8], dav[8];
          rx[i].get(xv);
          rda[i].get(dav);
          if (dres) {
            rres[i].get(res[i]);
          } else {
#pragma unroll
            for (int e = 0; e < 8; e++) res[i][e] = 0.f;
          }
#pragma unroll
          for (int e = 0; e < 8; e++) {
            n[i][e] = xv[e] * r;
            dn[i][e] = dav[e] * g[i][e];
            dg[i][e] += dav[e] * n[i][e];
            dot += dn[i][e] * n[i][e];
          }
        }
      }
      if (row + gridDim.x < rows) request(row + gridDim.x);
      const float mean = block_sum(dot, red) / (float)h;
#pragma unroll
      for (int i = 0; i < NORM_MAXC; i++) {
        const int c = threadIdx.x + i * EW_THREADS;
        if (c < nchunk) {
          float o[8];
#pragma unroll
          for (int e = 0; e < 8; e++) o[e] = res[i][e] + r * (dn[i][e] - n[i][e] * mean);
          store8(dx + row * ld_dx + c * 8, o);
        }
      }
    }
  } else {
    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
      const float r = rstd[row];
      float n[NORM_MAXC][8], dn[NORM_MAXC][8];
      float dot = 0.f;
#pragma unroll
      for (int i = 0; i < NORM_MAXC; i++) {
        const int c = threadIdx.x + i * EW_THREADS;
        if (c < nchunk) {
          float xv[8], dav[8];
          load8(x + row * ldx + c * 8, xv);
          load8(da + row * ld_da + c * 8, dav);
#pragma unroll
          for (int e = 0; e < 8; e++) {
            n[i][e] = xv[e] * r;
            dn[i][e] = dav[e] * g[i][e];
            dg[i][e] += dav[e] * n[i][e];
            dot += dn[i][e] * n[i][e];
          }
        }
      }
      float res[NORM_MAXC][8];  // requested before the reduction so that their latency overlaps it
#pragma unroll
      for (int i = 0; i < NORM_MAXC; i++) {
        const int c = threadIdx.x + i * EW_THREADS;
        if (c < nchunk) {
          if (dres) {
            load8(dres + row * ld_dres + c * 8, res[i]);
          } else {
#pragma unroll
            for (int e = 0; e < 8; e++) res[i][e] = 0.f;
          }
        }
      }
      const float mean = block_sum(dot, red) / (float)h;
#pragma unroll
      for (int i = 0; i < NORM_MAXC; i++) {
        const int c = threadIdx.x + i * EW_THREADS;
        if (c < nchunk) {
          float o[8];
#pragma unroll
          for (int e = 0; e < 8; e++) o[e] = res[i][e] + r * (dn[i][e] - n[i][e] * mean);
          store8(dx + row * ld_dx + c * 8, o);
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NORM_MAXC; i++) {
    const int c = threadIdx.x + i * EW_THREADS;
    if (c < nchunk) {
      float* p = partial + int64_t(blockIdx.x) * h + c * 8;
      if (acc_partial) {  // on top of what earlier calls left (same workgroup, same rows' share: a fixed order)
        float prev[8];
        load8(p, prev);
#pragma unroll
        for (int e = 0; e < 8; e++) dg[i][e] += prev[e];
      }
      store8(p, dg[i]);
    }
  }
}

// out[c] += sum_b partial[b][c]: 16 columns per workgroup, 16 row groups per column, fixed summation order
__global__ __launch_bounds__(256) void colsum_add_kernel(const float* __restrict__ partial, float* __restrict__ out,
                                                         int nblocks, int h, bool overwrite) {
  __shared__ float red[16][17];
  const int cl = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cl;
  float s = 0.f;
  if (c < h)
    for (int b = grp; b < nblocks; b += 16) s += partial[int64_t(b) * h + c];
  red[grp][cl] = s;
  __syncthreads();
  if (grp == 0 && c < h) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < 16; g++) t += red[g][cl];
    out[c] = overwrite ? t : out[c] + t;
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float4* __restrict__ p, size_t n4) {
  const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
  if (i < n4) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// ---------------------------------------------------------------- rotary embedding, in place
// One thread rotates 8 pairs (i .. i+7, i+d/2 .. i+d/2+7) of one head of one token.
template <typename T>
__global__ __launch_bounds__(EW_THREADS) void rope_kernel(T* __restrict__ u, const float* __restrict__ cos_tab,
                                                          const float* __restrict__ sin_tab, int64_t total, int S,
                                                          int n_heads, int d, int64_t ld, float sign) {
  const int64_t id = int64_t(blockIdx.x) * EW_THREADS + threadIdx.x;
  if (id >= total) return;
  const int cph = d >> 4;  // chunks of 8 pairs per head
  const int c = int(id % cph);
  const int head = int((id / cph) % n_heads);
  const int64_t t = id / (int64_t(cph) * n_heads);
  const int pos = int(t % S);
  T* p = u + t * ld + head * d + c * 8;
  float a[8], b[8], cs[8], sn[8], oa[8], ob[8];
  load8(p, a);
  load8(p + (d >> 1), b);
  load8(cos_tab + int64_t(pos) * (d >> 1) + c * 8, cs);
  load8(sin_tab + int64_t(pos) * (d >> 1) + c * 8, sn);
#pragma unroll
  for (int e = 0; e < 8; e++) {
    const float s = sign * sn[e];
    oa[e] = a[e] * cs[e] - b[e] * s;
    ob[e] = a[e] * s + b[e] * cs[e];
  }
  store8(p, oa);
  store8(p + (d >> 1), ob);
}

// ---------------------------------------------------------------- SwiGLU

template <typename T>
__global__ __launch_bounds__(EW_THREADS) void swiglu_fwd_kernel(const T* __restrict__ gu, int64_t ld_gu,
                                                                T* __restrict__ z, int64_t ld_z, int64_t total,
                                                                int f) {
  const int64_t id = int64_t(blockIdx.x) * EW_THREADS + threadIdx.x;
  if (id >= total) return;
  const int cpr = f >> 3;
  const int64_t t = id / cpr;
  const int c = int(id % cpr);
  float g[8], u[8], o[8];
  load8(gu + t * ld_gu + c * 8, g);
  load8(gu + t * ld_gu + f + c * 8, u);
#pragma unroll
  for (int e = 0; e < 8; e++) o[e] = g[e] * sigmoidf_(g[e]) * u[e];
  store8(z + t * ld_z + c * 8, o);
}

// IL: gu and dgu are in the interleaved gate/up column order (32 gates, their 32 ups, ...), else [gates | ups]
template <typename T, bool IL>
__global__ __launch_bounds__(EW_THREADS) void swiglu_bwd_kernel(const T* __restrict__ dz, int64_t ld_dz,
                                                                const T* __restrict__ gu, int64_t ld_gu,
                                                                T* __restrict__ dgu, int64_t ld_dgu, int64_t total,
                                                                int f) {
  const int64_t id = int64_t(blockIdx.x) * EW_THREADS + threadIdx.x;
  if (id >= total) return;
  const int cpr = f >> 3;
  const int64_t t = id / cpr;
  const int c = int(id % cpr) * 8;
  const int cg = IL ? (c >> 5) * 64 + (c & 31) : c, cu = IL ? cg + 32 : f + c;
  float g[8], u[8], d[8], og[8], ou[8];
  load8(gu + t * ld_gu + cg, g);
  load8(gu + t * ld_gu + cu, u);
  load8(dz + t * ld_dz + c, d);
#pragma unroll
  for (int e = 0; e < 8; e++) {
    const float s = sigmoidf_(g[e]);
    og[e] = d[e] * u[e] * s * (1.f + g[e] * (1.f - s));
    ou[e] = d[e] * g[e] * s;
  }
  store8(dgu + t * ld_dgu + cg, og);
  store8(dgu + t * ld_dgu + cu, ou);
}

// ---------------------------------------------------------------- weight generator (counter-based, fp64 Box-Muller)
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
// fp64 -> bf16 bits, one round-to-nearest-even (normal range)
__device__ __forceinline__ uint16_t f64_to_bf16_bits(double v) {
  const uint64_t u = (uint64_t)__double_as_longlong(v);
  const uint32_t sign = uint32_t(u >> 63) << 15;
  const int exp = int((u >> 52) & 0x7ff);
  if (exp == 0) return (uint16_t)sign;
  const uint64_t man = u & ((1ull << 52) - 1);
  uint32_t keep = (uint32_t(exp - 1023 + 127) << 7) | uint32_t(man >> 45);
  const uint64_t rem = man & ((1ull << 45) - 1), half = 1ull << 44;
  if (rem > half || (rem == half && (keep & 1))) keep += 1;
  return (uint16_t)(sign | keep);
}
__device__ __forceinline__ void put(bf16_t* p, double v) { *reinterpret_cast<uint16_t*>(p) = f64_to_bf16_bits(v); }
__device__ __forceinline__ void put(float* p, double v) { *p = (float)v; }

template <typename T>
__global__ __launch_bounds__(EW_THREADS) void fill_normal_kernel(T* __restrict__ out, int64_t n, int64_t cols,
                                                                 int64_t ld, uint64_t stream, double scale,
                                                                 double offset, int gu_f) {
  const int64_t i = int64_t(blockIdx.x) * EW_THREADS + threadIdx.x;  // flat index in the dense (public) layout
  if (i >= n) return;
  const uint64_t c = stream + 2ull * (uint64_t)i;
  const uint64_t r1 = mix64(c), r2 = mix64(c + 1);
  const double u1 = ((double)(r1 >> 11) + 1.0) * 0x1p-53;
  const double u2 = (double)(r2 >> 11) * 0x1p-53;
  const double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
  const int64_t col = i % cols;  // gu_f > 0: the tensor is stored in the interleaved gate/up column order
  put(out + (i / cols) * ld + (gu_f > 0 ? gu_interleaved_col(int(col), gu_f) : col), offset + scale * z);
}

// dst <- src with the columns of a [rows, 2f] matrix moved between the public and the interleaved gate/up order
// (8 columns per thread; blocks of 32 columns move as a whole)
__global__ __launch_bounds__(EW_THREADS) void gu_permute_kernel(const bf16_t* __restrict__ src, int64_t ld_src,
                                                                bf16_t* __restrict__ dst, int64_t ld_dst,
                                                                int64_t total, int f, bool to_interleaved) {
  const int64_t id = int64_t(blockIdx.x) * EW_THREADS + threadIdx.x;
  if (id >= total) return;
  const int cpr = f >> 2;  // 16-byte chunks per row of 2f columns
  const int64_t t = id / cpr;
  const int c = int(id % cpr) * 8, ci = gu_interleaved_col(c, f);
  const uint4 v = *reinterpret_cast<const uint4*>(src + t * ld_src + (to_interleaved ? c : ci));
  *reinterpret_cast<uint4*>(dst + t * ld_dst + (to_interleaved ? ci : c)) = v;
}

// dst[c][r] = src[r][c] for a rows x cols bf16 matrix (rows, cols multiples of 8): 64 x 64 tiles through LDS, padded
// against bank conflicts; 256 threads, each moves 16 elements
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16_t* __restrict__ src, int64_t ld_src,
                                                             bf16_t* __restrict__ dst, int64_t ld_dst, int rows, int cols) {
  __shared__ bf16_t tile[64][66];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < 16; i++) {
    const int r = ty + i * 4;
    if (r0 + r < rows && c0 + tx < cols) tile[r][tx] = src[int64_t(r0 + r) * ld_src + c0 + tx];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; i++) {
    const int c = ty + i * 4;
    if (c0 + c < cols && r0 + tx < rows) dst[int64_t(c0 + c) * ld_dst + r0 + tx] = tile[tx][c];
  }
}

inline int blocks_for(int64_t n) { return int((n + EW_THREADS - 1) / EW_THREADS); }

}  // namespace

namespace mls {

hipError_t rmsnorm_fwd(int dt, const void* x, int64_t ldx, const void* gamma, void* a, int64_t lda, float* r, int T,
                       int h, float eps, hipStream_t st) {
  if (T == 0) return hipSuccess;
#define FWD(TY, C)                                                                                             \
  hipLaunchKernelGGL((rmsnorm_fwd_kernel<TY, C>), dim3(T), dim3(EW_THREADS), 0, st, (const TY*)x, ldx,             \
                     (const TY*)gamma, (TY*)a, lda, r, h, eps)
  const int mc = h <= 4096 ? 2 : h <= 8192 ? 4 : 8;
  if (dt == DT_BF16) {
    if (mc == 2) FWD(bf16_t, 2); else if (mc == 4) FWD(bf16_t, 4); else FWD(bf16_t, 8);
  } else {
    if (mc == 2) FWD(float, 2); else if (mc == 4) FWD(float, 4); else FWD(float, 8);
  }
#undef FWD
  return hipGetLastError();
}

int rmsnorm_bwd_blocks(int T) { return T < 512 ? (T > 0 ? T : 1) : 512; }

hipError_t rmsnorm_bwd(int dt, const void* da, int64_t ld_da, const void* x, int64_t ldx, const void* gamma,
                       const float* r, const void* dres, int64_t ld_dres, void* dx, int64_t ld_dx, float* dgamma,
                       float* partial, int T, int h, hipStream_t st, bool overwrite, bool acc_partial, bool reduce) {
  if (T == 0) return hipSuccess;
  const int nb = rmsnorm_bwd_blocks(T);
#define BWD(TY, C)                                                                                               \
  hipLaunchKernelGGL((rmsnorm_bwd_kernel<TY, C>), dim3(nb), dim3(EW_THREADS), 0, st, (const TY*)da, ld_da,            \
                     (const TY*)x, ldx, (const TY*)gamma, r, (const TY*)dres, ld_dres, (TY*)dx, ld_dx, partial, T, h, acc_partial)
  const int mc = h <= 4096 ? 2 : h <= 8192 ? 4 : 8;
  if (dt == DT_BF16) {
    if (mc == 2) BWD(bf16_t, 2); else if (mc == 4) BWD(bf16_t, 4); else BWD(bf16_t, 8);
  } else {
    if (mc == 2) BWD(float, 2); else if (mc == 4) BWD(float, 4); else BWD(float, 8);
  }
#undef BWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !reduce) return e;
  hipLaunchKernelGGL(colsum_add_kernel, dim3((h + 15) / 16), dim3(256), 0, st, partial, dgamma, nb, h, overwrite);
  return hipGetLastError();
}

// n floats (a multiple of 4, 16-byte aligned) <- 0, as a kernel (safe to record into a HIP graph)
hipError_t fill_zero_f32(float* p, size_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  if (n % 4 || (uintptr_t(p) & 15)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(unsigned((n / 4 + 255) / 256)), dim3(256), 0, st, reinterpret_cast<float4*>(p), n / 4);
  return hipGetLastError();
}

hipError_t rope_inplace(int dt, void* u, const float* cos_tab, const float* sin_tab, int T, int S, int n_heads, int d,
                        int64_t ld, float sign, hipStream_t st) {
  const int64_t total = int64_t(T) * n_heads * (d >> 4);
  if (total == 0) return hipSuccess;
  if (dt == DT_BF16)
    hipLaunchKernelGGL(rope_kernel<bf16_t>, dim3(blocks_for(total)), dim3(EW_THREADS), 0, st, (bf16_t*)u, cos_tab,
                       sin_tab, total, S, n_heads, d, ld, sign);
  else
    hipLaunchKernelGGL(rope_kernel<float>, dim3(blocks_for(total)), dim3(EW_THREADS), 0, st, (float*)u, cos_tab,
                       sin_tab, total, S, n_heads, d, ld, sign);
  return hipGetLastError();
}

hipError_t swiglu_fwd(int dt, const void* gu, int64_t ld_gu, void* z, int64_t ld_z, int T, int f, hipStream_t st) {
  const int64_t total = int64_t(T) * (f >> 3);
  if (total == 0) return hipSuccess;
  if (dt == DT_BF16)
    hipLaunchKernelGGL(swiglu_fwd_kernel<bf16_t>, dim3(blocks_for(total)), dim3(EW_THREADS), 0, st, (const bf16_t*)gu,
                       ld_gu, (bf16_t*)z, ld_z, total, f);
  else
    hipLaunchKernelGGL(swiglu_fwd_kernel<float>, dim3(blocks_for(total)), dim3(EW_THREADS), 0, st, (const float*)gu,
                       ld_gu, (float*)z, ld_z, total, f);
  return hipGetLastError();
}

hipError_t swiglu_bwd(int dt, const void* dz, int64_t ld_dz, const void* gu, int64_t ld_gu, void* dgu, int64_t ld_dgu,
                      int T, int f, hipStream_t st, bool interleaved) {
  const int64_t total = int64_t(T) * (f >> 3);
  if (total == 0) return hipSuccess;
  if (interleaved && (dt != DT_BF16 || f % 32)) return hipErrorInvalidValue;
  if (interleaved)
    hipLaunchKernelGGL((swiglu_bwd_kernel<bf16_t, true>), dim3(blocks_for(total)), dim3(EW_THREADS), 0, st,
                       (const bf16_t*)dz, ld_dz, (const bf16_t*)gu, ld_gu, (bf16_t*)dgu, ld_dgu, total, f);
  else if (dt == DT_BF16)
    hipLaunchKernelGGL((swiglu_bwd_kernel<bf16_t, false>), dim3(blocks_for(total)), dim3(EW_THREADS), 0, st,
                       (const bf16_t*)dz, ld_dz, (const bf16_t*)gu, ld_gu, (bf16_t*)dgu, ld_dgu, total, f);
  else
    hipLaunchKernelGGL((swiglu_bwd_kernel<float, false>), dim3(blocks_for(total)), dim3(EW_THREADS), 0, st,
                       (const float*)dz, ld_dz, (const float*)gu, ld_gu, (float*)dgu, ld_dgu, total, f);
  return hipGetLastError();
}

hipError_t gu_permute(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t rows, int f,
                      bool to_interleaved, hipStream_t st) {
  const int64_t total = rows * (f >> 2);
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL(gu_permute_kernel, dim3(blocks_for(total)), dim3(EW_THREADS), 0, st, (const bf16_t*)src, ld_src,
                     (bf16_t*)dst, ld_dst, total, f, to_interleaved);
  return hipGetLastError();
}

hipError_t transpose_bf16(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int rows, int cols, hipStream_t st) {
  if (rows == 0 || cols == 0) return hipSuccess;
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3((cols + 63) / 64, (rows + 63) / 64), dim3(256), 0, st, (const bf16_t*)src,
                     ld_src, (bf16_t*)dst, ld_dst, rows, cols);
  return hipGetLastError();
}

hipError_t fill_normal(int dt, void* out, int64_t rows, int64_t cols, int64_t ld, uint64_t seed, uint32_t tensor,
                       uint32_t layer, double scale, double offset, hipStream_t st, int gu_f) {
  const int64_t n = rows * cols;
  if (n == 0) return hipSuccess;
  auto mixh = [](uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  };
  const uint64_t stream = mixh(mixh(seed) ^ ((uint64_t(tensor) << 32) | layer));
  if (dt == DT_BF16)
    hipLaunchKernelGGL(fill_normal_kernel<bf16_t>, dim3(blocks_for(n)), dim3(EW_THREADS), 0, st, (bf16_t*)out, n, cols,
                       ld, stream, scale, offset, gu_f);
  else
    hipLaunchKernelGGL(fill_normal_kernel<float>, dim3(blocks_for(n)), dim3(EW_THREADS), 0, st, (float*)out, n, cols, ld,
                       stream, scale, offset, gu_f);
  return hipGetLastError();
}

}  // namespace mls
