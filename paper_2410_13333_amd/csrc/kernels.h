// Host-side launchers of the HIP kernels of the decoder-stage library.  Every launcher enqueues on `st`,
// never synchronises and returns the launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace mls {

enum { GEMM_NN = 0, GEMM_NT = 1, GEMM_TN = 2 };
enum { DT_BF16 = 0, DT_FP32 = 1 };

// records `msg` as the calling thread's mls_last_error text and returns `code` (stage.hip)
int set_error(int code, const char* msg);

// Raises a kernel's dynamic-LDS limit, once per device (the attribute belongs to the function on the current
// device).  `done` is the launcher's own bit mask of devices already served; racing threads at worst set it twice.
inline hipError_t raise_lds_limit(const void* kern, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = uint64_t(1) << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

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
// gu_f > 0: the N = 2 gu_f columns of the B pieces are in the interleaved gate/up order and C is in the public one
// overwrite: C = instead of C += (the fp32 gradient is then not read)
hipError_t gemm_bf16_tn_segments(const void* const* A, const void* const* B, int nseg, void* C, int M, int N, int kseg,
                                 int64_t lda, int64_t ldb, int64_t ldc, hipStream_t st, int gu_f = 0,
                                 bool overwrite = false);
// the 256x256 tiles of a problem on the 16x16x32 form of the matrix instruction (gemm_bf16_m16.hip); K % 32 == 0
// (% 64 for NN and NT)
bool gemm_m16_ok(int mode, int K);
hipError_t gemm_m16(int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K, int64_t lda,
                    int64_t ldb, int64_t ldc, int64_t ldr, uint32_t ab, uint32_t bb, hipStream_t st);
hipError_t gemm_m16_swiglu(const void* A, const void* W, void* GU, void* Z, int M, int N, int K, int64_t lda, int64_t ldw,
                           int64_t ldgu, int64_t ldz, uint32_t ab, uint32_t bb, hipStream_t st, bool w_nk);
hipError_t gemm_m16_rope(const void* A, const void* W, void* C, int M, int N, int K, int64_t lda, int64_t ldw, int64_t ldc,
                         uint32_t ab, uint32_t bb, const float* cos_tab, const float* sin_tab, int seq, int rot_cols,
                         int head_dim, hipStream_t st, bool w_nk);
hipError_t gemm_m16_tn_segments(const void* const* A, const void* const* B, int nseg, void* C, int M, int N, int kseg,
                                int64_t lda, int64_t ldb, int64_t ldc, uint32_t ab, uint32_t bb, hipStream_t st, int gu_f,
                                bool overwrite);
hipError_t fill_zero_f32(float* p, size_t n, hipStream_t st);
// SwiGLU fused into the gate/up contraction (bf16, f % 32 == 0, DMA path).  Interleaved gate/up column order:
// 32 gate columns, the 32 up columns of the same indices, and so on (gu_interleaved_col in common.h).
//   GU[M, 2f] = A[M,K] W[K, 2f] (W and GU interleaved), Z[M, f] = silu(gate) * up
// w_nk: W is given transposed, [2f][K] (rows in the interleaved order) with row stride ldw.
bool gemm_swiglu_ok(int M, int f, int K, int64_t lda, int64_t ldw, bool w_nk = false);
hipError_t gemm_bf16_swiglu(const void* A, const void* W, void* GU, void* Z, int M, int f, int K, int64_t lda,
                            int64_t ldw, int64_t ldgu, int64_t ldz, hipStream_t st, bool w_nk = false);
// The rotary embedding fused into the q|k|v projection (bf16, DMA path): C[M, N] = A[M,K] W[K,N] rounded to bf16, then
// every head vector (head_dim = 64 or 128 columns) in the columns below rot_cols rotated by the angle of its row's
// position row % seq, pairs (i, i + head_dim/2); cos_tab, sin_tab: [seq][head_dim/2] fp32.
// w_nk: W is given transposed, [N][K] with row stride ldw.
bool gemm_rope_ok(int M, int N, int K, int64_t lda, int64_t ldw, int seq, int rot_cols, int head_dim, bool w_nk = false);
hipError_t gemm_bf16_rope(const void* A, const void* W, void* C, int M, int N, int K, int64_t lda, int64_t ldw, int64_t ldc,
                          const float* cos_tab, const float* sin_tab, int seq, int rot_cols, int head_dim, hipStream_t st,
                          bool w_nk = false);
hipError_t gemm_f32(int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K, int64_t lda,
                    int64_t ldb, int64_t ldc, int64_t ldr, hipStream_t st);

// ---- row-wise and elementwise kernels (elementwise.hip); dt selects the storage type; every matrix argument is
// followed by its row stride in elements (all row strides are multiples of 8)
// a = x * r * gamma, r[t] = rsqrt(mean(x^2) + eps) saved as fp32
hipError_t rmsnorm_fwd(int dt, const void* x, int64_t ldx, const void* gamma, void* a, int64_t lda, float* r, int T,
                       int h, float eps, hipStream_t st);
// dx = dres + r*(dn - n*mean(dn*n)), dn = da*gamma, n = x*r;  dgamma += sum_t da*n (two-stage, deterministic).
// partial: workspace of rmsnorm_bwd_blocks(T) * h floats.  dres may be null (no residual branch: dx without it).
// overwrite: dgamma = instead of +=.  A sequence of calls over several micro-batches may share one column
// reduction: acc_partial adds this call's row-block sums to those already in `partial` (same T), and only the
// call with `reduce` adds the columns of `partial` into dgamma (dgamma and overwrite are ignored otherwise).
int rmsnorm_bwd_blocks(int T);
hipError_t rmsnorm_bwd(int dt, const void* da, int64_t ld_da, const void* x, int64_t ldx, const void* gamma,
                       const float* r, const void* dres, int64_t ld_dres, void* dx, int64_t ld_dx, float* dgamma,
                       float* partial, int T, int h, hipStream_t st, bool overwrite = false, bool acc_partial = false,
                       bool reduce = true);
// rotate the pairs (i, i+d/2) of the first n_heads heads of every row of u [T, ld] by sign*angle(t % S, i)
hipError_t rope_inplace(int dt, void* u, const float* cos_tab, const float* sin_tab, int T, int S, int n_heads, int d,
                        int64_t ld, float sign, hipStream_t st);
hipError_t swiglu_fwd(int dt, const void* gu, int64_t ld_gu, void* z, int64_t ld_z, int T, int f, hipStream_t st);
hipError_t swiglu_bwd(int dt, const void* dz, int64_t ld_dz, const void* gu, int64_t ld_gu, void* dgu, int64_t ld_dgu,
                      int T, int f, hipStream_t st, bool interleaved = false);  // interleaved: gu, dgu in that order
// weights from the counter-based generator: element (r, c) of a rows x cols tensor stored with row stride ld is
// offset + scale*z(seed, tensor, layer, r*cols + c), rounded once
hipError_t fill_normal(int dt, void* out, int64_t rows, int64_t cols, int64_t ld, uint64_t seed, uint32_t tensor,
                       uint32_t layer, double scale, double offset, hipStream_t st, int gu_f = 0);
// dst[c][r] = src[r][c], bf16, rows x cols (used for the transposed weight copies of the data-gradient contractions)
hipError_t transpose_bf16(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int rows, int cols, hipStream_t st);
// gu_f > 0 above: a [rows, 2 gu_f] gate/up tensor is written in the interleaved column order.  gu_permute moves a
// bf16 [rows, 2f] matrix between the public and the interleaved column order.
hipError_t gu_permute(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t rows, int f,
                      bool to_interleaved, hipStream_t st);

// ---- attention (attention_bf16.hip, attention_f32.hip).  qkv: [T, q_dim + 2 kv_dim] rows = q heads | k heads | v heads
// (rotary already applied); o: [T, q_dim]; lse: natural-log softmax denominators [b, n_q, S] fp32.
hipError_t attn_fwd(int dt, const void* qkv, int64_t ld_qkv, void* o, int64_t ld_o, float* lse, int b, int S, int nq,
                    int nkv, int d, hipStream_t st);
// dqkv has the column layout of qkv; delta: workspace [b, n_q, S] fp32 (row sums of do*o); part: workspace of
// attn_bwd_scratch_floats() floats, or null.  With few KV heads the dK / dV kernels share the query heads of a
// group out over several workgroups, which leave fp32 partial sums in `part` for a fixed-order reduction; without
// the workspace one workgroup walks the whole group.  cos_tab, sin_tab ([S][d/2] fp32, bf16 storage only): the q and
// k parts of dqkv come out turned back by the rotary angle of their position, i.e. as gradients w.r.t. the
// projection's output; without them they are gradients w.r.t. the rotated q and k.
size_t attn_bwd_scratch_floats(int dt, int b, int S, int nq, int nkv, int d);
hipError_t attn_bwd(int dt, const void* qkv, int64_t ld_qkv, const void* o, int64_t ld_o, const float* lse,
                    const void* d_o, int64_t ld_do, void* dqkv, int64_t ld_dqkv, float* delta, int b, int S, int nq,
                    int nkv, int d, hipStream_t st, float* part = nullptr, const float* cos_tab = nullptr,
                    const float* sin_tab = nullptr);

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
                         hipStream_t st, float* part, const float* cos_tab, const float* sin_tab);

}  // namespace mls
