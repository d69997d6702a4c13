// fp32 GEMM for the all-fp32 validation mode of the stage (tiny shapes only): a plain LDS-tiled FMA kernel,
// 64x64x16 tiles, 4x4 outputs per thread.  Same three modes and epilogues as the bf16 kernel.
#include "common.h"
#include "kernels.h"

namespace {

constexpr int FB = 64, FK = 16;

// A(m,k) = A[m*sam + k*sak], B(k,n) = B[k*sbk + n*sbn]
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                       float* C, const float* R, int M, int N, int K, int64_t sam,
                                                       int64_t sak, int64_t sbk, int64_t sbn, int64_t ldc,
                                                       int64_t ldr, int accumulate) {
  __shared__ float As[FK][FB + 1], Bs[FK][FB + 1];
  const int m0 = blockIdx.y * FB, n0 = blockIdx.x * FB;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += FK) {
    for (int i = threadIdx.x; i < FB * FK; i += 256) {
      // consecutive threads walk the memory-contiguous index of each operand
      int am, ak, bk, bn;
      if (sak == 1) { ak = i % FK; am = i / FK; } else { am = i % FB; ak = i / FB; }
      if (sbn == 1) { bn = i % FB; bk = i / FB; } else { bk = i % FK; bn = i / FK; }
      As[ak][am] = (m0 + am < M && k0 + ak < K) ? A[(m0 + am) * sam + (k0 + ak) * sak] : 0.f;
      Bs[bk][bn] = (n0 + bn < N && k0 + bk < K) ? B[(k0 + bk) * sbk + (n0 + bn) * sbn] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < FK; k++) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int row = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
      if (row < M && col < N) {
        const int64_t off = int64_t(row) * ldc + col;
        float v = acc[i][j];
        if (accumulate) v += C[off];
        else if (R) v += R[int64_t(row) * ldr + col];
        C[off] = v;
      }
    }
}

}  // namespace

namespace mls {

hipError_t gemm_f32(int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K, int64_t lda,
                    int64_t ldb, int64_t ldc, int64_t ldr, hipStream_t st) {
  if (M == 0 || N == 0) return hipSuccess;
  int64_t sam, sak, sbk, sbn;
  int acc = 0;
  switch (mode) {
    case GEMM_NN: sam = lda; sak = 1; sbk = ldb; sbn = 1; break;
    case GEMM_NT: sam = lda; sak = 1; sbk = 1; sbn = ldb; break;
    case GEMM_TN: sam = 1; sak = lda; sbk = ldb; sbn = 1; acc = 1; break;
    default: return hipErrorInvalidValue;
  }
  dim3 grid((N + FB - 1) / FB, (M + FB - 1) / FB);
  hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, (const float*)A, (const float*)B, (float*)C,
                     (const float*)R, M, N, K, sam, sak, sbk, sbn, ldc, ldr, acc);
  return hipGetLastError();
}

}  // namespace mls
