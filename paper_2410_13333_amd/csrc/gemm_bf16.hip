// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// One kernel template serves the three contraction shapes of a decoder layer:
//   NN  C[M,N]  = A[M,K] * B[K,N] (+ R)      forward projections, residual add in the epilogue
//   NT  C[M,N]  = A[M,K] * B[N,K]^T          data gradients (B is the weight in its [in,out] layout)
//   TN  C[M,N] += A[K,M]^T * B[K,N]  (fp32)  weight gradients; the fp32 read-modify-write of the
//                                            epilogue IS the accumulation over micro-batches
// An operand whose contraction index is contiguous in memory is staged in LDS as [row][k] and read with
// ds_read_b128; an operand whose contraction index is strided is staged as [k][col] exactly as it lies in
// memory and read with ds_read_b64_tr_b16, which hands each lane four k-consecutive values of one column,
// so no transposed copy of any tensor ever exists in HBM.
#include "common.h"
#include "kernels.h"

namespace {

enum { EPI_BF16 = 0, EPI_F32_ACC = 1 };

template <int BM, int BN, int BK, int WGM, int WGN, bool ATR, bool BTR>
struct Geo {
  static constexpr int NT = WGM * WGN * 64;
  static constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
  // LDS row lengths in elements.  [row][k] tiles: +8 elements (16 B) so that 16 rows read by a ds_read_b128
  // start in 16 distinct 4-bank groups.  [k][col] tiles: +32 elements (64 B) so that the 4 k-rows a
  // transposing read touches fall into distinct banks.
  static constexpr int A_ROWS = ATR ? BK : BM, A_COLS = ATR ? BM : BK, A_LD = A_COLS + (ATR ? 32 : 8);
  static constexpr int B_ROWS = BTR ? BK : BN, B_COLS = BTR ? BN : BK, B_LD = B_COLS + (BTR ? 32 : 8);
  static constexpr int A_ELEMS = A_ROWS * A_LD, B_ELEMS = B_ROWS * B_LD;
  static constexpr int STAGE = A_ELEMS + B_ELEMS;
  static constexpr int NA = A_ROWS * A_COLS / 8 / NT, NB = B_ROWS * B_COLS / 8 / NT;
  static constexpr size_t LDS_BYTES = size_t(2) * STAGE * sizeof(bf16_t);
  static_assert(A_ROWS * A_COLS / 8 % NT == 0 && B_ROWS * B_COLS / 8 % NT == 0, "tile must split evenly");
};

// global -> registers: tile of ROWS x COLS elements at (row0, col0) of a row-major matrix with `rows` x `cols`
// valid elements; chunks outside are zero.
template <int ROWS, int COLS, int NT, int N>
__device__ __forceinline__ void tile_load(const bf16_t* __restrict__ g, int64_t ld, int row0, int col0, int rows,
                                          int cols, uint4 (&r)[N]) {
  constexpr int CPR = COLS / 8;
#pragma unroll
  for (int i = 0; i < N; i++) {
    const int id = threadIdx.x + i * NT;
    const int rr = row0 + id / CPR, cc = col0 + (id % CPR) * 8;
    if (rr < rows && cc < cols)
      r[i] = *reinterpret_cast<const uint4*>(g + int64_t(rr) * ld + cc);
    else
      r[i] = make_uint4(0, 0, 0, 0);
  }
}
template <int ROWS, int COLS, int LD, int NT, int N>
__device__ __forceinline__ void tile_store(bf16_t* lds, const uint4 (&r)[N]) {
  constexpr int CPR = COLS / 8;
#pragma unroll
  for (int i = 0; i < N; i++) {
    const int id = threadIdx.x + i * NT;
    *reinterpret_cast<uint4*>(lds + (id / CPR) * LD + (id % CPR) * 8) = r[i];
  }
}

// MFMA operand fragment of 32 rows (or columns) x 16 k-values: lane l holds row l%32, k = (l/32)*8 .. +7.
template <int LD>
__device__ __forceinline__ bf16x8 frag_rowk(const bf16_t* tile, int row_base, int kk, int lane) {
  const uint4 v = *reinterpret_cast<const uint4*>(tile + (row_base + (lane & 31)) * LD + kk * 16 + (lane >> 5) * 8);
  return __builtin_bit_cast(bf16x8, v);
}
// Same fragment out of a [k][col] tile.  A transposing read serves 16 lanes: lane 4r+c passes the address of
// (k0 + r, col0 + 4c) and receives k0..k0+3 of column col0 + (lane%16).
template <int LD>
__device__ __forceinline__ bf16x8 frag_kcol(const bf16_t* tile, int col_base, int kk, int lane) {
  const int kr = kk * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
  const int col = col_base + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  const bf16_t* p = tile + kr * LD + col;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLS_LDS s16x4*)(p));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLS_LDS s16x4*)(p + 4 * LD));
  s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

template <int BM, int BN, int BK, int WGM, int WGN, bool ATR, bool BTR, int EPI>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_kernel(const bf16_t* __restrict__ A,
                                                                   const bf16_t* __restrict__ B, void* __restrict__ Cv,
                                                                   const bf16_t* __restrict__ R, int M, int N, int K,
                                                                   int64_t lda, int64_t ldb, int64_t ldc, int64_t ldr,
                                                                   int tiles_m, int tiles_n) {
  using G = Geo<BM, BN, BK, WGM, WGN, ATR, BTR>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD one contiguous run of tiles (M fastest)
  // so that the tiles sharing a B panel also share an L2.
  const int nwg = gridDim.x, pid = blockIdx.x;
  const int xcd = pid & 7, q = nwg >> 3, rem = nwg & 7;
  const int tile = xcd * q + (xcd < rem ? xcd : rem) + (pid >> 3);
  const int m0 = (tile % tiles_m) * BM, n0 = (tile / tiles_m) * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave % WGM) * (BM / WGM), wn = (wave / WGM) * (BN / WGN);

  f32x16 acc[G::TM][G::TN];
#pragma unroll
  for (int i = 0; i < G::TM; i++)
#pragma unroll
    for (int j = 0; j < G::TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  uint4 ra[G::NA], rb[G::NB];
  auto gload = [&](int k0) {
    if (ATR) tile_load<G::A_ROWS, G::A_COLS, G::NT>(A, lda, k0, m0, K, M, ra);
    else     tile_load<G::A_ROWS, G::A_COLS, G::NT>(A, lda, m0, k0, M, K, ra);
    if (BTR) tile_load<G::B_ROWS, G::B_COLS, G::NT>(B, ldb, k0, n0, K, N, rb);
    else     tile_load<G::B_ROWS, G::B_COLS, G::NT>(B, ldb, n0, k0, N, K, rb);
  };
  auto lstore = [&](int buf) {
    bf16_t* sa = smem + buf * G::STAGE;
    tile_store<G::A_ROWS, G::A_COLS, G::A_LD, G::NT>(sa, ra);
    tile_store<G::B_ROWS, G::B_COLS, G::B_LD, G::NT>(sa + G::A_ELEMS, rb);
  };

  const int nk = (K + BK - 1) / BK;
  gload(0);
  lstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; kt++) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nk;
    if (more) gload((kt + 1) * BK);
    const bf16_t* sa = smem + cur * G::STAGE;
    const bf16_t* sb = sa + G::A_ELEMS;
#pragma unroll
    for (int kk = 0; kk < BK / 16; kk++) {
      bf16x8 af[G::TM], bfr[G::TN];
#pragma unroll
      for (int i = 0; i < G::TM; i++)
        af[i] = ATR ? frag_kcol<G::A_LD>(sa, wm + i * 32, kk, lane) : frag_rowk<G::A_LD>(sa, wm + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < G::TN; j++)
        bfr[j] = BTR ? frag_kcol<G::B_LD>(sb, wn + j * 32, kk, lane) : frag_rowk<G::B_LD>(sb, wn + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < G::TM; i++)
#pragma unroll
        for (int j = 0; j < G::TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) lstore(cur ^ 1);
    __syncthreads();
  }

  // Epilogue.  Accumulator element (g*4 + r) of lane l is C[row = (l/32)*4 + 8g + r][col = l%32] of its 32x32 tile.
#pragma unroll
  for (int i = 0; i < G::TM; i++)
#pragma unroll
    for (int j = 0; j < G::TN; j++) {
      const int col = n0 + wn + j * 32 + (lane & 31);
      if (col >= N) continue;
#pragma unroll
      for (int g = 0; g < 4; g++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int row = m0 + wm + i * 32 + (lane >> 5) * 4 + 8 * g + r;
          if (row >= M) continue;
          const int64_t off = int64_t(row) * ldc + col;
          float v = acc[i][j][g * 4 + r];
          if (EPI == EPI_BF16) {
            if (R) v += to_f32(R[int64_t(row) * ldr + col]);
            reinterpret_cast<bf16_t*>(Cv)[off] = (bf16_t)v;
          } else {
            float* C = reinterpret_cast<float*>(Cv);
            C[off] += v;
          }
        }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN, bool ATR, bool BTR, int EPI>
hipError_t launch(const bf16_t* A, const bf16_t* B, void* C, const bf16_t* R, int M, int N, int K, int64_t lda,
                  int64_t ldb, int64_t ldc, int64_t ldr, hipStream_t st) {
  using G = Geo<BM, BN, BK, WGM, WGN, ATR, BTR>;
  auto kern = gemm_bf16_kernel<BM, BN, BK, WGM, WGN, ATR, BTR, EPI>;
  static std::atomic<uint64_t> lds_raised{0};
  if (hipError_t e = mls::raise_lds_limit(reinterpret_cast<const void*>(kern), (int)G::LDS_BYTES, lds_raised)) return e;
  const int tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tm * tn), dim3(G::NT), G::LDS_BYTES, st, A, B, C, R, M, N, K, lda, ldb, ldc, ldr, tm, tn);
  return hipGetLastError();
}

template <bool ATR, bool BTR, int EPI>
hipError_t dispatch(const bf16_t* A, const bf16_t* B, void* C, const bf16_t* R, int M, int N, int K, int64_t lda,
                    int64_t ldb, int64_t ldc, int64_t ldr, hipStream_t st) {
  const int64_t big_tiles = int64_t((M + 255) / 256) * ((N + 255) / 256);
  if (big_tiles >= 192) return launch<256, 256, 32, 2, 2, ATR, BTR, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, ldr, st);
  return launch<128, 128, 32, 2, 2, ATR, BTR, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, ldr, st);
}

}  // namespace

namespace mls {

hipError_t gemm_bf16(int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K, int64_t lda,
                     int64_t ldb, int64_t ldc, int64_t ldr, hipStream_t st) {
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* b = static_cast<const bf16_t*>(B);
  const bf16_t* r = static_cast<const bf16_t*>(R);
  if (M == 0 || N == 0) return hipSuccess;
  if (gemm_bf16_dma_ok(mode, M, N, K, lda, ldb)) return gemm_bf16_dma(mode, A, B, C, R, M, N, K, lda, ldb, ldc, ldr, st);
  switch (mode) {
    case GEMM_NN: return dispatch<false, true, EPI_BF16>(a, b, C, r, M, N, K, lda, ldb, ldc, ldr, st);
    case GEMM_NT: return dispatch<false, false, EPI_BF16>(a, b, C, r, M, N, K, lda, ldb, ldc, ldr, st);
    case GEMM_TN: return dispatch<true, true, EPI_F32_ACC>(a, b, C, r, M, N, K, lda, ldb, ldc, ldr, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace mls
