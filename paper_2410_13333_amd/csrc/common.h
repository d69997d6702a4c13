// Shared device helpers of the decoder-stage library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define MLS_LDS __attribute__((address_space(3)))

// ---- 8-element (one 16-byte bf16 chunk / two 16-byte fp32 chunks) loads and stores, values as fp32
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
  uint4 raw = *reinterpret_cast<const uint4*>(p);
  uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; i++) {
    v[2 * i] = __uint_as_float(w[i] << 16);
    v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 t = {(bf16_t)lo, (bf16_t)hi};  // round-to-nearest-even (v_cvt_pk_bf16_f32)
  return __builtin_bit_cast(uint32_t, t);
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
  uint4 raw;
  raw.x = pack_bf16x2(v[0], v[1]); raw.y = pack_bf16x2(v[2], v[3]);
  raw.z = pack_bf16x2(v[4], v[5]); raw.w = pack_bf16x2(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = raw;
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
  reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
}
// ---- 4-element bf16 (8-byte) loads and stores
__device__ __forceinline__ void load4(const bf16_t* p, float (&v)[4]) {
  const uint2 raw = *reinterpret_cast<const uint2*>(p);
  v[0] = __uint_as_float(raw.x << 16);
  v[1] = __uint_as_float(raw.x & 0xffff0000u);
  v[2] = __uint_as_float(raw.y << 16);
  v[3] = __uint_as_float(raw.y & 0xffff0000u);
}
__device__ __forceinline__ void store4(bf16_t* p, const float (&v)[4]) {
  uint2 raw;
  raw.x = pack_bf16x2(v[0], v[1]);
  raw.y = pack_bf16x2(v[2], v[3]);
  *reinterpret_cast<uint2*>(p) = raw;
}
__device__ __forceinline__ float round_bf16(float v) { return (float)(bf16_t)v; }
__device__ __forceinline__ float sigmoidf_(float g) { return 1.f / (1.f + __expf(-g)); }

// ---- gate/up column order.  Public: [gate 0..f) | up 0..f)].  Interleaved (internal, used when the SwiGLU is fused
// into the contractions around it; needs f % 32 == 0): 32 gate columns, then the 32 up columns of the same indices,
// and so on, so that a lane of the contraction's epilogue holds a gate and its up.
__host__ __device__ __forceinline__ int gu_public_col(int n, int f) { return ((n >> 5) & 1) * f + (n >> 6) * 32 + (n & 31); }
__host__ __device__ __forceinline__ int gu_interleaved_col(int c, int f) {
  const int w = c >= f, r = c - w * f;
  return (r >> 5) * 64 + w * 32 + (r & 31);
}

__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ void from_f32(bf16_t& d, float v) { d = (bf16_t)v; }
__device__ __forceinline__ void from_f32(float& d, float v) { d = v; }

// ---- reductions: 64-lane wavefront, then up to 16 wavefronts through LDS
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// sum over the whole workgroup; `red` is an LDS array of >= blockDim.x/64 floats; all threads get the result
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();  // protects `red` against the previous use
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; i++) t += red[i];
  return t;
}
