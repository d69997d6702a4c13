// Host-side launchers of the HIP kernels of the decoder-stage library.  Every launcher enqueues on `st`,
// never synchronises and returns the launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mls {

enum { GEMM_NN = 0, GEMM_NT = 1, GEMM_TN = 2 };
enum { DT_BF16 = 0, DT_FP32 = 1 };

// ---- contractions (gemm_bf16.hip, gemm_f32.hip); modes as documented at mls_gemm; leading dims in elements
// (ldr: row stride of the residual R, ignored when R is null)
hipError_t gemm_bf16(int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K, int64_t lda,
                     int64_t ldb, int64_t ldc, int64_t ldr, hipStream_t st);
// the two implementations behind gemm_bf16: LDS-DMA main path and the register-staged fallback for operands
// too large for 31-bit buffer offsets
bool gemm_bf16_dma_ok(int mode, int M, int N, int K, int64_t lda, int64_t ldb);
hipError_t gemm_bf16_dma(int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K,
                         int64_t lda, int64_t ldb, int64_t ldc, int64_t ldr, hipStream_t st);
// weight gradient of several micro-batches in one launch: C[M,N] += sum_i A_i[kseg,M]^T * B_i[kseg,N], C fp32,
// at most 16 pieces, all with the same strides; true if the operands fit the DMA path's 31-bit offsets
bool gemm_tn_segments_ok(int kseg, int64_t lda, int64_t ldb);
hipError_t gemm_bf16_tn_segments(const void* const* A, const void* const* B, int nseg, void* C, int M, int N, int kseg,
                                 int64_t lda, int64_t ldb, int64_t ldc, hipStream_t st);
hipError_t gemm_f32(int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K, int64_t lda,
                    int64_t ldb, int64_t ldc, int64_t ldr, hipStream_t st);

// ---- row-wise and elementwise kernels (elementwise.hip); dt selects the storage type; every matrix argument is
// followed by its row stride in elements (all row strides are multiples of 8)
// a = x * r * gamma, r[t] = rsqrt(mean(x^2) + eps) saved as fp32
hipError_t rmsnorm_fwd(int dt, const void* x, int64_t ldx, const void* gamma, void* a, int64_t lda, float* r, int T,
                       int h, float eps, hipStream_t st);
// dx = dres + r*(dn - n*mean(dn*n)), dn = da*gamma, n = x*r;  dgamma += sum_t da*n (two-stage, deterministic).
// partial: workspace of rmsnorm_bwd_blocks(T) * h floats.
int rmsnorm_bwd_blocks(int T);
hipError_t rmsnorm_bwd(int dt, const void* da, int64_t ld_da, const void* x, int64_t ldx, const void* gamma,
                       const float* r, const void* dres, int64_t ld_dres, void* dx, int64_t ld_dx, float* dgamma,
                       float* partial, int T, int h, hipStream_t st);
// rotate the pairs (i, i+d/2) of the first n_heads heads of every row of u [T, ld] by sign*angle(t % S, i)
hipError_t rope_inplace(int dt, void* u, const float* cos_tab, const float* sin_tab, int T, int S, int n_heads, int d,
                        int64_t ld, float sign, hipStream_t st);
hipError_t swiglu_fwd(int dt, const void* gu, int64_t ld_gu, void* z, int64_t ld_z, int T, int f, hipStream_t st);
hipError_t swiglu_bwd(int dt, const void* dz, int64_t ld_dz, const void* gu, int64_t ld_gu, void* dgu, int64_t ld_dgu,
                      int T, int f, hipStream_t st);
// weights from the counter-based generator: element (r, c) of a rows x cols tensor stored with row stride ld is
// offset + scale*z(seed, tensor, layer, r*cols + c), rounded once
hipError_t fill_normal(int dt, void* out, int64_t rows, int64_t cols, int64_t ld, uint64_t seed, uint32_t tensor,
                       uint32_t layer, double scale, double offset, hipStream_t st);

// ---- attention (attention_bf16.hip, attention_f32.hip).  qkv: [T, q_dim + 2 kv_dim] rows = q heads | k heads | v heads
// (rotary already applied); o: [T, q_dim]; lse: natural-log softmax denominators [b, n_q, S] fp32.
hipError_t attn_fwd(int dt, const void* qkv, int64_t ld_qkv, void* o, int64_t ld_o, float* lse, int b, int S, int nq,
                    int nkv, int d, hipStream_t st);
// dqkv has the column layout of qkv; delta: workspace [b, n_q, S] fp32 (row sums of do*o)
hipError_t attn_bwd(int dt, const void* qkv, int64_t ld_qkv, const void* o, int64_t ld_o, const float* lse,
                    const void* d_o, int64_t ld_do, void* dqkv, int64_t ld_dqkv, float* delta, int b, int S, int nq,
                    int nkv, int d, hipStream_t st);

// pieces behind the two dispatchers above
hipError_t attn_delta(int dt, const void* o, int64_t ld_o, const void* d_o, int64_t ld_do, float* delta, int b, int S,
                      int nq, int d, hipStream_t st);
hipError_t attn_fwd_f32(const void* qkv, int64_t ld_qkv, void* o, int64_t ld_o, float* lse, int b, int S, int nq, int nkv,
                        int d, hipStream_t st);
hipError_t attn_bwd_f32(const void* qkv, int64_t ld_qkv, const void* o, int64_t ld_o, const float* lse, const void* d_o,
                        int64_t ld_do, void* dqkv, int64_t ld_dqkv, float* delta, int b, int S, int nq, int nkv, int d,
                        hipStream_t st);
hipError_t attn_fwd_bf16(const void* qkv, int64_t ld_qkv, void* o, int64_t ld_o, float* lse, int b, int S, int nq, int nkv,
                         int d, hipStream_t st);
hipError_t attn_bwd_bf16(const void* qkv, int64_t ld_qkv, const void* o, int64_t ld_o, const float* lse, const void* d_o,
                         int64_t ld_do, void* dqkv, int64_t ld_dqkv, float* delta, int b, int S, int nq, int nkv, int d,
                         hipStream_t st);

}  // namespace mls
