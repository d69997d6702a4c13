// bf16 GEMM, main path: tiles go from global memory straight into LDS (buffer_load_dwordx4 ... lds), so the
// main loop holds no staging registers and no LDS stores; out-of-range rows and columns are zero-filled by
// the buffer range check instead of branches.  Same three modes and epilogues as gemm_bf16.hip.
//
// LDS tiles are unpadded (the DMA writes 64 lanes x 16 B contiguously) and XOR-swizzled on the global-address
// side so that both fragment read patterns are bank-conflict free:
//   [row][k] tiles (contraction index contiguous in memory), read with ds_read_b128:
//        16-byte chunk c of row r lives in slot c ^ ((r / rows_per_256B) % chunks_per_row)
//   [k][col] tiles (contraction index strided in memory), read with ds_read_b64_tr_b16:
//        16-byte chunk c of k-row r lives in chunk c ^ ((r & 3) << 2)   (moves 64-byte blocks)
// The pipeline keeps NS tile stages in LDS with ONE workgroup barrier per k-step: the loads of tile kt+NS-1 are
// issued right after the barrier that publishes tile kt and retires the reads of tile kt-1.  In the skewed
// form (NS >= 3) that barrier already publishes tile kt+1, whose first fragments are then fetched during the
// last substep of tile kt, so no LDS latency is exposed behind the barrier.
// The LDS-DMA instructions are inline asm because the compiler would otherwise wait for all of them
// (vmcnt(0)) before every LDS read; the waits are placed by hand.
// A workgroup is NW wavefronts, 2 along M by NW/2 along N: 4 (one per SIMD, 128x128 of a 256x256 tile each, all
// accumulators in AGPRs) or 8 (two per SIMD, 128x64 each, under 256 registers, so that one wavefront issues MFMAs
// while the other waits at the barrier or for its fragments).  bf16 epilogues leave through an LDS staging pass
// that turns the accumulator layout into whole-row 16-byte accesses.
#include <cstdlib>
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;
// EPI_ROPE: the head vectors in columns below rot_cols are rotated by the rotary angle of their row's position
// (row % seq), pairs (i, i + head_dim/2), in fp32 on the accumulators, and rounded to bf16 once; the remaining
// columns (v) are stored as they are.
// Epilogues.  EPI_BF16: C = acc (+ R), bf16.  EPI_F32_ACC: C += acc, fp32 (C = acc when `ldx` != 0); with `xf` > 0
// the columns are the gate/up-interleaved order and are written to their public places (see gu_public_col).  EPI_SWIGLU: N = 2f
// interleaved columns [gate | up]; C receives both (bf16) and X[row][f] their SwiGLU product.  (The SwiGLU backward
// as an epilogue of the dZ contraction was measured slower than a separate kernel: the epilogue's extra reads are
// fully exposed with one workgroup per CU.)
enum { EPI_BF16 = 0, EPI_F32_ACC = 1, EPI_SWIGLU = 2, EPI_ROPE = 3 };
enum { PIPE_PLAIN = 0, PIPE_SKEW = 1 };

__device__ __forceinline__ void dma16(i32x4 rsrc, uint32_t voff, uint32_t lds_byte) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_byte), "v"(voff), "s"(rsrc)
               : "memory");
}
// orders this wave's LDS accesses before the call against those after it (the wave exchanges data with itself)
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ i32x4 make_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)p;
  i32x4 r;
  r[0] = (int)(uint32_t)a;
  r[1] = (int)((uint32_t)(a >> 32) & 0xffffu);  // stride 0: raw buffer, byte offsets
  r[2] = (int)bytes;
  r[3] = 0x00020000;
  return r;
}

constexpr uint32_t OOB = 0x80000000u;  // beyond any num_records accepted by the launcher

// Segmented contraction (weight gradients over several micro-batches in one launch): the contraction index runs
// over nseg pieces of kseg rows each; piece i has its own operand base pointers, all pieces share the strides.
constexpr int MAX_SEGS = 16;
struct SegArgs {
  const bf16_t* a[MAX_SEGS];
  const bf16_t* b[MAX_SEGS];
  int nseg, kseg;
};
// rotary tables [seq][head_dim/2] fp32 and the column range they apply to (EPI_ROPE)
struct RopeArgs {
  const float* cos_tab;
  const float* sin_tab;
  int seq, rot_cols, head_dim;
};

// ---- [row][k] tile: ROWS x BK elements, BK*2 bytes per row
template <int ROWS, int BK, int NW = 4>
struct RowTile {
  static constexpr int RB = BK * 2, CPR = RB / 16, RPB = 256 / RB;  // row bytes, chunks per row, rows per 256 B
  static constexpr int BYTES = ROWS * RB, RPI = 1024 / RB;          // rows per DMA instruction
  static constexpr int NI = ROWS / RPI / NW;                        // DMA instructions per wave
  static_assert(RB == 64 || RB == 128, "BK must be 32 or 64");
  uint32_t goff[NI];  // byte offset of this lane's chunk at k-tile 0 (OOB if the row is out of range)
  int kcol[NI];       // its first k index inside a tile
  __device__ __forceinline__ void init(int row0, int nrows, int64_t ld, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NI; i++) {
      const int r = (wave * NI + i) * RPI + lane / CPR;
      const int c = (lane % CPR) ^ ((r / RPB) % CPR);  // logical chunk stored in this lane's slot
      kcol[i] = c * 8;
      goff[i] = row0 + r < nrows ? uint32_t((int64_t(row0 + r) * ld + c * 8) * 2) : OOB;
    }
  }
  // byte offset of DMA instruction i for the tile starting at k0 (columns at or beyond K are out of range)
  __device__ __forceinline__ uint32_t voff(int i, int k0, int K, int64_t) const {
    return k0 + kcol[i] < K ? goff[i] + uint32_t(k0) * 2 : OOB;
  }
  // MFMA operand: lane l = row rbase + l%32, k = kk*16 + (l/32)*8 .. +7
  static __device__ __forceinline__ bf16x8 frag(const unsigned char* t, int rbase, int kk, int lane) {
    const int r = rbase + (lane & 31), c = kk * 2 + (lane >> 5);
    const uint4 v = *reinterpret_cast<const uint4*>(t + r * RB + ((c ^ ((r / RPB) % CPR)) << 4));
    return __builtin_bit_cast(bf16x8, v);
  }
};

// ---- [k][col] tile: BK x COLS elements, COLS*2 bytes per k-row
template <int COLS, int BK, int NW = 4>
struct ColTile {
  static constexpr int CB = COLS * 2, CPR = CB / 16;
  static constexpr int BYTES = BK * CB, RPI = 1024 / CB;
  static constexpr int NI = BK / RPI / NW;
  static_assert(CPR >= 16, "tile must be at least 128 columns wide");
  uint32_t goff[NI];  // byte offset at k-tile 0 (OOB if the column is out of range)
  __device__ __forceinline__ void init(int col0, int ncols, int64_t ld, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NI; i++) {
      const int r = (wave * NI + i) * RPI + lane / CPR;
      const int c = (lane % CPR) ^ ((r & 3) << 2);
      goff[i] = col0 + c * 8 < ncols ? uint32_t((int64_t(r) * ld + col0 + c * 8) * 2) : OOB;
    }
  }
  // k-rows beyond K lie beyond the end of the matrix and are zero-filled by the range check
  __device__ __forceinline__ uint32_t voff(int i, int k0, int, int64_t ld) const {
    return goff[i] < OOB ? goff[i] + uint32_t(int64_t(k0) * ld * 2) : OOB;
  }
  // MFMA operand: lane l = column cbase + l%32, k = kk*16 + (l/32)*8 .. +7.  A transposing read serves 16
  // lanes: lane 4r+c passes the address of (k0 + r, col0 + 4c) and receives k0..k0+3 of column col0 + lane%16.
  static __device__ __forceinline__ bf16x8 frag(const unsigned char* t, int cbase, int kk, int lane) {
    const int kr = kk * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
    const int col = cbase + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
    const int sw = (kr & 3) << 2;
    const unsigned char* p = t + kr * CB + (((col >> 3) ^ sw) << 4) + (col & 7) * 2;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLS_LDS s16x4*)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLS_LDS s16x4*)(p + 4 * CB));
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
};

template <int BM, int BN, int BK, int NS, bool ATR, bool BTR, int EPI, int PIPE, bool SEG, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_dma_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                       void* __restrict__ Cv, const bf16_t* __restrict__ R, int M,
                                                       int N, int K, int64_t lda, int64_t ldb, int64_t ldc,
                                                       int64_t ldr, uint32_t a_bytes, uint32_t b_bytes, int tiles_m,
                                                       int col0, void* __restrict__ Xv, int64_t ldx, int xf,
                                                       SegArgs segs, RopeArgs rope) {
  using AT_R = RowTile<BM, BK, NW>;
  using AT_C = ColTile<BM, BK, NW>;
  using BT_R = RowTile<BN, BK, NW>;
  using BT_C = ColTile<BN, BK, NW>;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  // NW wavefronts: 2 along M, NW/2 along N (4: one per SIMD, 128x128 each at 256x256; 8: two per SIMD, 128x64 each)
  constexpr int WN = NW / 2;
  constexpr int TM = BM / 64, TN = BN / WN / 32, KS = BK / 16;
  constexpr int LPT = (ATR ? AT_C::NI : AT_R::NI) + (BTR ? BT_C::NI : BT_R::NI);  // DMA loads per wave per tile
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int nwg = gridDim.x, pid = blockIdx.x;
  const int xcd = pid & 7, q = nwg >> 3, rem = nwg & 7;
  const int tile = xcd * q + (xcd < rem ? xcd : rem) + (pid >> 3);
  // inside its run an XCD walks groups of GM tile rows, N fastest within a group, so that the ~32 tiles it has in
  // flight form a squarish patch and share both A and B panels in its L2
  constexpr int GM = 4;
  const int gm = GM < tiles_m ? GM : tiles_m;
  const int per_group = gm * (nwg / tiles_m), grp = tile / per_group, first_m = grp * gm;
  const int gsz = min(tiles_m - first_m, gm), in_grp = tile - grp * per_group;
  const int m0 = (first_m + in_grp % gsz) * BM, n0 = (in_grp / gsz) * BN;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave & 1) * (BM / 2), wn = (wave >> 1) * (BN / WN);

  // prefetch cursor: the k-tile the next DMA instructions fetch (piece pf_seg, first row pf_k0)
  i32x4 ra = make_rsrc(SEG ? segs.a[0] : A, a_bytes), rb = make_rsrc(SEG ? segs.b[0] : B, b_bytes);
  int pf_seg = 0, pf_k0 = 0;
  const int kpiece = SEG ? segs.kseg : K;
  auto advance = [&]() {
    pf_k0 += BK;
    if (SEG && pf_k0 >= kpiece) {
      pf_k0 = 0;
      pf_seg++;
      const int i = pf_seg < segs.nseg ? pf_seg : segs.nseg - 1;
      ra = make_rsrc(segs.a[i], a_bytes);
      rb = make_rsrc(segs.b[i], b_bytes);
    }
  };
  AT_R atr;
  AT_C atc;
  BT_R btr;
  BT_C btc;
  if (ATR) atc.init(m0, M, lda, wave, lane); else atr.init(m0, M, lda, wave, lane);
  if (BTR) btc.init(n0, N, ldb, wave, lane); else btr.init(n0, N, ldb, wave, lane);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(MLS_LDS unsigned char*)smem;
  const uint32_t a_wave = lds0 + wave * (A_BYTES / NW), b_wave = lds0 + A_BYTES + wave * (B_BYTES / NW);
  constexpr int NIA = ATR ? AT_C::NI : AT_R::NI;
  // DMA instruction d (0 .. LPT-1) of this wave for k-tile kt into `stage`: the first NIA belong to A
  // (`live` false: the tile does not exist; the load is sent out of range and only zero-fills a dead stage, which
  // keeps the number of loads per k-step, and with it the vmcnt bookkeeping, constant and the loop branch-free)
  auto fire = [&](int d, int stage, bool live) {
    const int k0 = pf_k0;
    if (d < NIA) {
      const uint32_t v = ATR ? atc.voff(d, k0, kpiece, lda) : atr.voff(d, k0, kpiece, lda);
      dma16(ra, live ? v : OOB, a_wave + stage * STAGE + d * 1024);
    } else {
      const uint32_t v = BTR ? btc.voff(d - NIA, k0, kpiece, ldb) : btr.voff(d - NIA, k0, kpiece, ldb);
      dma16(rb, live ? v : OOB, b_wave + stage * STAGE + (d - NIA) * 1024);
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  const int nk = (SEG ? segs.nseg : 1) * ((kpiece + BK - 1) / BK);
  // Paired A tiles (forward projections: A is [row][k], 32 deep, i.e. 64 bytes of a row per k-tile).  Two consecutive
  // k-tiles share their 128-byte lines; requested one iteration apart, the second request misses the CU's L1 again
  // (48 KiB of lines pass through it per iteration) and every line of A comes from L2 twice.  Here the A tiles of
  // an even / odd pair are requested back to back in one iteration (the L1 merges them: one L2 request per line),
  // into a ring of 5 stages of their own; the B tiles keep their ring of NS = 4 and are requested every iteration.
  constexpr bool PAIRA = !ATR && BTR && BK == 32 && PIPE == PIPE_SKEW && !SEG && NS == 4;
  constexpr int RA = 5;  // stages of the A ring
  if (!PAIRA) {
#pragma unroll
    for (int s = 0; s < NS - 1; s++) {
#pragma unroll
      for (int d = 0; d < LPT; d++) fire(d, s, s < nk);
      advance();
    }
  }

  // LDS reads per 16-wide k-substep and the MFMA : read interleave the scheduler is asked for
  constexpr int NR = (ATR ? 2 : 1) * TM + (BTR ? 2 : 1) * TN, NMFMA = TM * TN;
  constexpr int DPK = (LPT + KS - 1) / KS;  // DMA instructions fired per k-substep
  bf16x8 af[2][TM], bfr[2][TN];
  auto lfrag = [&](const unsigned char* sa, int kk, int buf) {
    const unsigned char* sb = sa + A_BYTES;
#pragma unroll
    for (int i = 0; i < TM; i++)
      af[buf][i] = ATR ? AT_C::frag(sa, wm + i * 32, kk, lane) : AT_R::frag(sa, wm + i * 32, kk, lane);
#pragma unroll
    for (int j = 0; j < TN; j++)
      bfr[buf][j] = BTR ? BT_C::frag(sb, wn + j * 32, kk, lane) : BT_R::frag(sb, wn + j * 32, kk, lane);
  };
  // one 16-wide k-substep; DMA instructions [d0, d1) of the prefetched tile go out between the rows of the MFMA
  // block (operands swapped: the lane ends up with 4 consecutive columns of one row)
  auto mfma_block = [&](int kk, int pstage, bool prefetch, int d0, int d1) {
    const int per = (d1 - d0 + TM - 1) / TM;
#pragma unroll
    for (int i = 0; i < TM; i++) {
#pragma unroll
      for (int d = d0 + ((i + TM / 2) % TM) * per; d < d0 + ((i + TM / 2) % TM + 1) * per && d < d1; d++)
        fire(d, pstage, prefetch);
#pragma unroll
      for (int j = 0; j < TN; j++)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
    }
  };
  auto interleave_hint = [&]() {  // spread the LDS reads just issued over the first half of the MFMAs
    if (NMFMA >= 8) {
#pragma unroll
      for (int g = 0; g < NMFMA / 2; g++) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // 1 MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, NR / (NMFMA / 2), 0);  // its share of the DS reads
      }
    }
  };
  if constexpr (PAIRA) {
    constexpr int NIB = BT_C::NI;
    const uint32_t a_ring = lds0 + wave * (A_BYTES / NW), b_ring = lds0 + RA * A_BYTES + wave * (B_BYTES / NW);
    // DMA instruction d of this wave for k-tile t (t >= nk: sent out of range, zero-fills a dead stage)
    auto fire_a = [&](int d, int t, int st) {
      dma16(ra, t < nk ? atr.voff(d, t * BK, K, lda) : OOB, a_ring + st * A_BYTES + d * 1024);
    };
    auto fire_b = [&](int d, int t, int st) {
      dma16(rb, t < nk ? btc.voff(d, t * BK, K, ldb) : OOB, b_ring + st * B_BYTES + d * 1024);
    };
    auto lfrag2 = [&](int sta, int stb, int kk, int buf) {
      const unsigned char* sa = smem + sta * A_BYTES;
      const unsigned char* sb = smem + RA * A_BYTES + stb * B_BYTES;
#pragma unroll
      for (int i = 0; i < TM; i++) af[buf][i] = AT_R::frag(sa, wm + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; j++) bfr[buf][j] = BT_C::frag(sb, wn + j * 32, kk, lane);
    };
    // prologue, in this order: A0 B0 A1 B1 A2 B2 A3
#pragma unroll
    for (int t = 0; t < 4; t++) {
#pragma unroll
      for (int d = 0; d < NIA; d++) fire_a(d, t, t);
      if (t < 3) {
#pragma unroll
        for (int d = 0; d < NIB; d++) fire_b(d, t, t);
      }
    }
    wait_vmcnt<2 * (NIA + NIB) + NIA>();  // tile 0 has landed
    __syncthreads();
    lfrag2(0, 0, 0, 0);
    int sa_cur = 0, sb_cur = 0;  // ring positions of tile kt
    // one k-tile; ODD iterations request B(kt+3), A(kt+3), A(kt+4), even ones only B(kt+3)
    auto iteration = [&](int kt, auto ODD) {
      constexpr bool odd = decltype(ODD)::value;
      // this wave's part of tile kt+1 has landed: behind it in the queue are, for an even kt, B(kt+2) A(kt+2) A(kt+3),
      // for an odd kt, A(kt+2) B(kt+2)
      if (odd) wait_vmcnt<NIA + NIB>(); else wait_vmcnt<2 * NIA + NIB>();
      __syncthreads();  // ... everyone's has; the reads of tile kt-1 are retired
      const int sa_n = sa_cur + 1 == RA ? 0 : sa_cur + 1, sb_n = sb_cur + 1 == NS ? 0 : sb_cur + 1;
      const int sb3 = sb_cur == 0 ? NS - 1 : sb_cur - 1;                  // (kt + 3) % 4 == (kt - 1) % 4
      const int sa3 = sa_cur + 3 >= RA ? sa_cur + 3 - RA : sa_cur + 3;    // (kt + 3) % 5
      const int sa4 = sa_cur == 0 ? RA - 1 : sa_cur - 1;                  // (kt + 4) % 5 == (kt - 1) % 5
      constexpr int NF = odd ? NIB + 2 * NIA : NIB, SLOTS = KS * TM;
      auto fire_n = [&](int n) {  // the n-th request of this iteration
        if (n < NIB) fire_b(n, kt + 3, sb3);
        else if (n < NIB + NIA) fire_a(n - NIB, kt + 3, sa3);
        else fire_a(n - NIB - NIA, kt + 4, sa4);
      };
#pragma unroll
      for (int kk = 0; kk < KS; kk++) {
        __builtin_amdgcn_sched_barrier(0);
        if (kk + 1 < KS) lfrag2(sa_cur, sb_cur, kk + 1, (kk + 1) & 1); else lfrag2(sa_n, sb_n, 0, 0);
#pragma unroll
        for (int i = 0; i < TM; i++) {
          const int slot = kk * TM + i;
#pragma unroll
          for (int n = slot * NF / SLOTS; n < (slot + 1) * NF / SLOTS; n++) fire_n(n);
#pragma unroll
          for (int j = 0; j < TN; j++)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
        }
        interleave_hint();
      }
      sa_cur = sa_n;
      sb_cur = sb_n;
    };
    for (int kt = 0; kt < nk; kt += 2) {
      iteration(kt, std::false_type{});
      if (kt + 1 < nk) iteration(kt + 1, std::true_type{});
    }
  } else
  if (PIPE == PIPE_SKEW) {
    int stage = 0;
    // Skewed pipeline (needs NS >= 3 and an even number of substeps): the barrier at the top of iteration kt
    // publishes tile kt+1, so the first fragments of tile kt+1 are fetched during the last substep of tile kt
    // and no LDS latency is exposed behind the barrier.
    static_assert(PIPE != PIPE_SKEW || (NS >= 3 && KS % 2 == 0), "skewed pipeline needs 3 stages");
    wait_vmcnt<(NS - 2) * LPT>();
    __syncthreads();
    lfrag(smem, 0, 0);
    for (int kt = 0; kt < nk; kt++) {
      wait_vmcnt<(NS >= 3 ? NS - 3 : 0) * LPT>();  // this wave's part of tile kt+1 has landed
      __syncthreads();                             // ... everyone's has; the reads of tile kt-1 are retired
      const bool prefetch = kt + NS - 1 < nk;
      const int pstage = stage == 0 ? NS - 1 : stage - 1, nstage = stage + 1 == NS ? 0 : stage + 1;
      const unsigned char* sa = smem + stage * STAGE;
#pragma unroll
      for (int kk = 0; kk < KS; kk++) {
        __builtin_amdgcn_sched_barrier(0);
        if (kk + 1 < KS) lfrag(sa, kk + 1, (kk + 1) & 1); else lfrag(smem + nstage * STAGE, 0, 0);
        mfma_block(kk, pstage, prefetch, kk * DPK, (kk + 1) * DPK < LPT ? (kk + 1) * DPK : LPT);
        interleave_hint();
      }
      advance();
      stage = nstage;
    }
  } else {
    int stage = 0;
    for (int kt = 0; kt < nk; kt++) {
      // tile kt has landed once at most the loads of the NS-2 younger tiles are still in flight
      wait_vmcnt<(NS - 2) * LPT>();
      __syncthreads();
      const bool prefetch = kt + NS - 1 < nk;
      const int pstage = stage == 0 ? NS - 1 : stage - 1;
      const unsigned char* sa = smem + stage * STAGE;
      lfrag(sa, 0, 0);
#pragma unroll
      for (int kk = 0; kk < KS; kk++) {
        __builtin_amdgcn_sched_barrier(0);
        if (kk + 1 < KS) lfrag(sa, kk + 1, (kk + 1) & 1);
        // every request for the next tile goes out in the first substep, right behind the barrier that freed its
        // stage: with two stages a request issued later in the k-step has less than a k-step to land
        mfma_block(kk, pstage, prefetch, kk == 0 ? 0 : LPT, LPT);
        if (kk + 1 < KS) interleave_hint();
      }
      advance();
      stage = stage + 1 == NS ? 0 : stage + 1;
    }
  }
  wait_vmcnt<0>();  // nothing of this wave may still be writing LDS when it leaves

  // ---- Epilogue.  Element (g*4 + e) of lane l is C[row l%32][col (l/32)*4 + 8g + e] of its 32x32 tile: a store
  // straight from the accumulators would touch 32 rows with 16 bytes each.  Instead each wave passes its tile, 32
  // rows at a time, through its own 16 KiB of the (now free) LDS and moves whole rows to and from memory (bf16
  // epilogues): lane l
  // handles the 16-byte chunk l % NCH of row l / NCH.  The staging rows are XOR-swizzled by chunk so that both
  // access patterns spread over all banks.  `col0` is the column of the whole problem at which this launch's
  // column 0 sits (a launch may cover a column range).
  __syncthreads();  // every wave has read its last fragments and every DMA has landed
  // (the rotary epilogue packs the staging areas, 4 KiB each, to make room for its exchange buffers)
  unsigned char* ws = smem + wave * (EPI == EPI_ROPE ? 4096 : 64 * 1024 / NW);
  constexpr int CW = BN / WN;                         // columns of a wave tile
  constexpr int RB = CW * 2, NCH = RB / 16;           // bytes and 16-byte chunks per staged row (bf16)
  constexpr int RPI = 64 / NCH, NT = 32 / RPI;        // rows per whole-wave access, accesses per 32 rows
  const int crow = lane / NCH, cch = lane % NCH;      // this lane's row and chunk in a whole-wave access
  const int r32 = lane & 31, hi = lane >> 5;
  const bool col_ok = n0 + wn + cch * 8 < N;        // N is a multiple of 8
  const int ccol = col0 + n0 + wn + cch * 8;        // first column of this lane's chunk, in the whole problem
  // rows of RB < 256 bytes share a 256-byte bank line: the swizzle key is the line, so that the 32 rows of an
  // accumulator-layout access fall on every bank equally often
  constexpr int RPL = RB < 256 ? 256 / RB : 1;
  auto stage_at = [&](int row, int chunk) { return ws + row * RB + ((chunk ^ ((row / RPL) & (NCH - 1))) << 4); };
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int row0 = m0 + wm + i * 32;
    if (EPI == EPI_F32_ACC) {
      // C += acc straight from the accumulator layout (16 bytes per lane, read and written by the same lane);
      // staging this one through LDS measured slower
      const int row = row0 + r32;
      if (row < M) {
#pragma unroll
        for (int q = 0; q < TN * 4; q++) {
          const int j = q >> 2, g = q & 3, col = n0 + wn + j * 32 + hi * 4 + 8 * g;
          if (col >= N) continue;
          float4* c = reinterpret_cast<float4*>(reinterpret_cast<float*>(Cv) + int64_t(row) * ldc +
                                                (xf > 0 ? gu_public_col(col0 + col, xf) : col0 + col));
          float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
          if (ldx == 0) t = *c;  // ldx != 0 in this mode: store, do not accumulate (C is not read)
          t.x += acc[i][j][g * 4]; t.y += acc[i][j][g * 4 + 1]; t.z += acc[i][j][g * 4 + 2]; t.w += acc[i][j][g * 4 + 3];
          *c = t;
        }
      }
    } else {
      if (EPI == EPI_BF16 && R) {  // residual rows -> LDS
#pragma unroll
        for (int t = 0; t < NT; t++) {
          const int lrow = t * RPI + crow, row = row0 + lrow;
          uint4 rr = make_uint4(0, 0, 0, 0);
          if (row < M && col_ok) rr = *reinterpret_cast<const uint4*>(R + int64_t(row) * ldr + ccol);
          *reinterpret_cast<uint4*>(stage_at(lrow, cch)) = rr;
        }
        wave_lds_sync();
      }
      if constexpr (EPI == EPI_ROPE) {
        // Rotation on the fp32 accumulators.  A head of 64 columns is this wave's two 32-column tiles: the partner of
        // a value sits in the same lane, in the other tile.  A head of 128 columns spans this wave's 64 columns and
        // those of the wave next to it along N (wave ^ 2): the waves exchange their fp32 rows through LDS behind the
        // bf16 staging areas (two buffers of 8 KiB per wave, alternating with the 32-row block so that one workgroup
        // barrier per block suffices; 16-byte chunks XOR-swizzled by row).  The table entries are requested before
        // the exchange so that their latency passes behind the barrier.
        const bool wide = rope.head_dim == 128;
        const bool rot = col0 + n0 + wn < rope.rot_cols;  // whole heads: uniform over the wave
        const int d2 = rope.head_dim >> 1;
        unsigned char* fx = smem + 32 * 1024 + (i & 1) * NW * 8192;
        auto fx_at = [&](int w, int chunk) { return fx + w * 8192 + r32 * 256 + ((chunk ^ (r32 & 15)) << 4); };
        float4 cs[TN][4], sn[TN][4];
        if (rot) {
          const int row = row0 + r32;
          const int64_t at = int64_t((row < M ? row : 0) % rope.seq) * d2 + hi * 4;
#pragma unroll
          for (int j = 0; j < (wide ? TN : 1); j++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
              cs[j][g] = *reinterpret_cast<const float4*>(rope.cos_tab + at + j * 32 + 8 * g);
              sn[j][g] = *reinterpret_cast<const float4*>(rope.sin_tab + at + j * 32 + 8 * g);
            }
        }
        if (wide) {
          if (rot) {
#pragma unroll
            for (int q = 0; q < TN * 4; q++) {
              const int j = q >> 2, g = q & 3;
              *reinterpret_cast<float4*>(fx_at(wave, j * 8 + 2 * g + hi)) =
                  make_float4(acc[i][j][g * 4], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]);
            }
          }
          __syncthreads();
        }
        if (rot) {
          const bool first = !((wave >> 1) & 1);  // wide: this wave holds the first halves of its pairs
#pragma unroll
          for (int g = 0; g < 4; g++) {
            if (wide) {
#pragma unroll
              for (int j = 0; j < TN; j++) {
                const float4 pv = *reinterpret_cast<const float4*>(fx_at(wave ^ 2, j * 8 + 2 * g + hi));
                const float pp[4] = {pv.x, pv.y, pv.z, pv.w};
                const float c[4] = {cs[j][g].x, cs[j][g].y, cs[j][g].z, cs[j][g].w};
                const float sv[4] = {sn[j][g].x, sn[j][g].y, sn[j][g].z, sn[j][g].w};
#pragma unroll
                for (int e = 0; e < 4; e++) {
                  const float own = acc[i][j][g * 4 + e];
                  // first half: u1 c - u2 s with u1 own, u2 partner; second half: u1 s + u2 c with u1 partner, u2 own
                  acc[i][j][g * 4 + e] = first ? own * c[e] - pp[e] * sv[e] : pp[e] * sv[e] + own * c[e];
                }
              }
            } else {
              const float c[4] = {cs[0][g].x, cs[0][g].y, cs[0][g].z, cs[0][g].w};
              const float sv[4] = {sn[0][g].x, sn[0][g].y, sn[0][g].z, sn[0][g].w};
#pragma unroll
              for (int e = 0; e < 4; e++) {
                const float u1 = acc[i][0][g * 4 + e], u2 = acc[i][1][g * 4 + e];
                acc[i][0][g * 4 + e] = u1 * c[e] - u2 * sv[e];
                acc[i][1][g * 4 + e] = u1 * sv[e] + u2 * c[e];
              }
            }
          }
        }
      }
      // combine in the accumulator layout, in place
      constexpr int ZRB = CW, ZNCH = ZRB / 16, ZRPL = ZRB < 256 ? 256 / ZRB : 1;  // SwiGLU product: half as many columns, staged behind the 8 KiB
      unsigned char* wz = ws + 32 * RB;
#pragma unroll
      for (int q = 0; q < TN * 4; q++) {
        const int j = q >> 2, g = q & 3;
        unsigned char* p = stage_at(r32, 4 * j + g) + hi * 8;
        float v[4] = {acc[i][j][g * 4], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]};
        if (EPI == EPI_BF16 && R) {
          const uint2 rr = *reinterpret_cast<const uint2*>(p);
          v[0] += __uint_as_float(rr.x << 16);
          v[1] += __uint_as_float(rr.x & 0xffff0000u);
          v[2] += __uint_as_float(rr.y << 16);
          v[3] += __uint_as_float(rr.y & 0xffff0000u);
        }
        uint2 o;
        o.x = pack_bf16x2(v[0], v[1]);
        o.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>(p) = o;
        if (EPI == EPI_SWIGLU && !(j & 1)) {
          // 32-column blocks alternate gate, up: tile j (even) holds the gates of the ups in tile j + 1.  The
          // product is formed from the fp32 accumulators and rounded once.
          float z[4];
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const float gr = v[e], ur = acc[i][j | 1][g * 4 + e];
            z[e] = gr * sigmoidf_(gr) * ur;
          }
          uint2 zo;
          zo.x = pack_bf16x2(z[0], z[1]);
          zo.y = pack_bf16x2(z[2], z[3]);
          const int zc = 4 * (j >> 1) + g;
          *reinterpret_cast<uint2*>(wz + r32 * ZRB + ((zc ^ ((r32 / ZRPL) & (ZNCH - 1))) << 4) + hi * 8) = zo;
        }
      }
      wave_lds_sync();
#pragma unroll
      for (int t = 0; t < NT; t++) {
        const int lrow = t * RPI + crow, row = row0 + lrow;
        const uint4 o = *reinterpret_cast<const uint4*>(stage_at(lrow, cch));
        if (row < M && col_ok) *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(Cv) + int64_t(row) * ldc + ccol) = o;
      }
      if (EPI == EPI_SWIGLU) {
        constexpr int ZRPI = 64 / ZNCH, ZNT = 32 / ZRPI;
        const int zrow = lane / ZNCH, zch = lane % ZNCH;
        const int zcol = ((col0 + n0 + wn) >> 1) + zch * 8;  // product column of this lane's chunk
        const bool z_ok = n0 + wn + zch * 16 < N;
#pragma unroll
        for (int t = 0; t < ZNT; t++) {
          const int lrow = t * ZRPI + zrow, row = row0 + lrow;
          const uint4 o = *reinterpret_cast<const uint4*>(wz + lrow * ZRB + ((zch ^ ((lrow / ZRPL) & (ZNCH - 1))) << 4));
          if (row < M && z_ok) *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(Xv) + int64_t(row) * ldx + zcol) = o;
        }
      }
      wave_lds_sync();
    }
  }
}

template <int BM, int BN, int BK, int NS, bool ATR, bool BTR, int EPI, int PIPE = PIPE_PLAIN, bool SEG = false, int NW = 4>
hipError_t launch(const bf16_t* A, const bf16_t* B, void* C, const bf16_t* R, int M, int N, int K, int64_t lda,
                  int64_t ldb, int64_t ldc, int64_t ldr, uint32_t a_bytes, uint32_t b_bytes, hipStream_t st,
                  const SegArgs* segs = nullptr, int col0 = 0, void* X = nullptr, int64_t ldx = 0, int xf = 0,
                  const RopeArgs* rope = nullptr) {
  // (the forward form keeps its A tiles in a ring of 5 stages beside the NS stages of B: see PAIRA in the kernel)
  constexpr bool PAIRA = !ATR && BTR && BK == 32 && PIPE == PIPE_SKEW && !SEG && NS == 4;
  constexpr int LDS_PIPE = PAIRA ? (5 * BM + NS * BN) * BK * 2 : NS * (BM + BN) * BK * 2;
  // the rotary epilogue keeps two buffers of 8 KiB of fp32 rows per wavefront behind 32 KiB of bf16 staging areas and
  // pairs the two 32-column tiles of a wavefront
  static_assert(EPI != EPI_ROPE || BN / (NW / 2) == 64, "rotary epilogue: wave tile");
  constexpr int LDS_ROPE = (32 + 16 * NW) * 1024;
  constexpr int LDS = EPI == EPI_ROPE && LDS_ROPE > LDS_PIPE ? LDS_ROPE : LDS_PIPE;
  auto kern = gemm_dma_kernel<BM, BN, BK, NS, ATR, BTR, EPI, PIPE, SEG, NW>;
  SegArgs sa = {};
  if (segs) sa = *segs;
  RopeArgs ra = {};
  if (rope) ra = *rope;
  static std::atomic<uint64_t> lds_raised{0};
  if (hipError_t e = mls::raise_lds_limit(reinterpret_cast<const void*>(kern), LDS, lds_raised)) return e;
  const int tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tm * tn), dim3(NW * 64), LDS, st, A, B, C, R, M, N, K, lda, ldb, ldc, ldr, a_bytes, b_bytes, tm,
                     col0, X, ldx, xf, sa, ra);
  return hipGetLastError();
}

// Tiling plan of one problem.  256x256 tiles (one workgroup per CU) run whole rounds of the 256 CUs; what is left
// over would still cost a full round, so the trailing columns may run as a second launch of smaller tiles instead:
// 256x128 (half the work per workgroup) or 128x128 (a quarter, at about three quarters of the big tile's rate).
// The choice minimises rounds x work per workgroup / relative rate, the rates being measured ones (13B stage: a
// 128x128 tail of 64 tiles' worth takes 0.29 of a round against 0.5 as 256x128 tiles on half the CUs; 7B stage:
// three rounds of 128x128 tiles for 176 tiles' worth are no faster than one round of 256x256).
enum { TAIL_NONE = 0, TAIL_256x128 = 1, TAIL_128x128 = 2 };
struct ColumnPlan {
  int n1;    // leading columns (a multiple of 256, possibly 0) run with 256x256 tiles
  int tail;  // TAIL_*: how the columns from n1 on run (TAIL_NONE: n1 == N, everything is 256x256)
};
ColumnPlan plan_columns(int M, int N) {
  constexpr int CUS = 256;
  const int tm = (M + 255) / 256, tn = (N + 255) / 256;
  const int n1_tiles = int(int64_t(tm) * tn / CUS * CUS / tm);  // whole rounds' worth of tile columns
  const int rest_cols = N - n1_tiles * 256;
  if (rest_cols <= 0) return {N, TAIL_NONE};
  auto rounds = [&](int64_t wgs) { return double((wgs + CUS - 1) / CUS); };
  const double a = rounds(int64_t(tm) * ((rest_cols + 255) / 256));
  const double b = rounds(int64_t(tm) * ((rest_cols + 127) / 128)) * 0.5 / 0.95;
  const double c = rounds(int64_t((M + 127) / 128) * ((rest_cols + 127) / 128)) * 0.25 / 0.75;
  if (a <= b && a <= c) return {N, TAIL_NONE};
  return {n1_tiles * 256, b <= c ? TAIL_256x128 : TAIL_128x128};
}

// Extra operands of the fused epilogues (see the EPI_* list)
struct Extra {
  void* X = nullptr;
  int64_t ldx = 0;
  int xf = 0;
  const RopeArgs* rope = nullptr;
};

// A problem may run as two launches over column ranges; they never offset C, R or X: the kernel adds `col0`, the
// first column of its range, to its epilogue columns
template <bool ATR, bool BTR, int EPI>
hipError_t dispatch(const bf16_t* A, const bf16_t* B, void* C, const bf16_t* R, int M, int N, int K, int64_t lda,
                    int64_t ldb, int64_t ldc, int64_t ldr, uint32_t ab, uint32_t bb, hipStream_t st,
                    const Extra& x = Extra()) {
  // Measured on the 7B stage: with a transposed-read operand (forward, weight gradient) four 32-deep stages in
  // the skewed pipeline win; with two [row][k] operands (data gradient) two 64-deep stages win.  Deeper pipelines
  // and a two-stage loop with its barrier ahead of the last substep all measured within noise of these or slower.
  constexpr int BK = BTR ? 32 : 64, NS = BTR ? 4 : 2, PIPE = BTR ? PIPE_SKEW : PIPE_PLAIN;
  // Wavefronts per 256x256 workgroup, by measurement on the 7B stage: the bf16-epilogue modes run 8 (two per SIMD,
  // 128x64 each: the second wavefront covers the first one's barrier and load waits; forward -5 %, data gradient
  // -3 %), the fp32 read-modify-write mode runs 4 (128x128 each; 8 measured 2.5 % slower there).
  constexpr int NW = EPI != EPI_F32_ACC ? 8 : 4;
  const ColumnPlan cp = plan_columns(M, N);
  // MLS_OLD_GEMM in the environment keeps the 32x32x16 kernels of this file for every tile (for comparisons)
  static const bool use_m16 = getenv("MLS_OLD_GEMM") == nullptr;
  if (cp.n1 > 0 && use_m16 && mls::gemm_m16_ok(ATR ? mls::GEMM_TN : mls::GEMM_NN, K) && (EPI == EPI_SWIGLU || EPI == EPI_ROPE || (x.xf == 0 && x.ldx == 0))) {
    const int mode = ATR ? mls::GEMM_TN : BTR ? mls::GEMM_NN : mls::GEMM_NT;
    hipError_t e;
    if (EPI == EPI_SWIGLU) e = mls::gemm_m16_swiglu(A, B, C, x.X, M, cp.n1, K, lda, ldb, ldc, x.ldx, ab, bb, st, !BTR);
    else if (EPI == EPI_ROPE) e = mls::gemm_m16_rope(A, B, C, M, cp.n1, K, lda, ldb, ldc, ab, bb, x.rope->cos_tab, x.rope->sin_tab,
                                                     x.rope->seq, x.rope->rot_cols, x.rope->head_dim, st, !BTR);
    else e = mls::gemm_m16(mode, A, B, C, R, M, cp.n1, K, lda, ldb, ldc, ldr, ab, bb, st);
    if (e != hipSuccess || cp.tail == TAIL_NONE) return e;
  } else
  if (cp.n1 > 0) {
    hipError_t e = launch<256, 256, BK, NS, ATR, BTR, EPI, PIPE, false, NW>(A, B, C, R, M, cp.n1, K, lda, ldb, ldc, ldr, ab, bb, st,
                                                                           nullptr, 0, x.X, x.ldx, x.xf, x.rope);
    if (e != hipSuccess || cp.tail == TAIL_NONE) return e;
  }
  // the columns of B from n1 on: a pointer offset for [k][n], a row offset for [n][k]
  const int n1 = cp.n1;
  const bf16_t* b2 = BTR ? B + n1 : B + int64_t(n1) * ldb;
  const uint32_t bb2 = BTR ? bb : uint32_t(int64_t(N - n1) * ldb * 2);
  if (cp.tail == TAIL_256x128)
    return launch<256, 128, BK, NS, ATR, BTR, EPI, PIPE>(A, b2, C, R, M, N - n1, K, lda, ldb, ldc, ldr, ab, bb2, st, nullptr, n1,
                                                          x.X, x.ldx, x.xf, x.rope);
  return launch<128, 128, 64, 3, ATR, BTR, EPI>(A, b2, C, R, M, N - n1, K, lda, ldb, ldc, ldr, ab, bb2, st, nullptr, n1, x.X,
                                                 x.ldx, x.xf, x.rope);
}

}  // namespace

namespace mls {

// true if the DMA path can run this problem: every operand (plus one tile of slack) addressable with a
// 31-bit byte offset
bool gemm_bf16_dma_ok(int mode, int M, int N, int K, int64_t lda, int64_t ldb) {
  const int64_t a_rows = mode == GEMM_TN ? K : M, b_rows = mode == GEMM_NT ? N : K;
  const int64_t lim = int64_t(1) << 31;
  return (a_rows + 512) * lda * 2 < lim && (b_rows + 512) * ldb * 2 < lim && K > 0;
}

hipError_t gemm_bf16_dma(int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K,
                         int64_t lda, int64_t ldb, int64_t ldc, int64_t ldr, hipStream_t st) {
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* b = static_cast<const bf16_t*>(B);
  const bf16_t* r = static_cast<const bf16_t*>(R);
  if (M == 0 || N == 0) return hipSuccess;
  const int64_t a_rows = mode == GEMM_TN ? K : M, b_rows = mode == GEMM_NT ? N : K;
  const uint32_t ab = uint32_t(a_rows * lda * 2), bb = uint32_t(b_rows * ldb * 2);
  switch (mode) {
    case GEMM_NN: return dispatch<false, true, EPI_BF16>(a, b, C, r, M, N, K, lda, ldb, ldc, ldr, ab, bb, st);
    case GEMM_NT: return dispatch<false, false, EPI_BF16>(a, b, C, r, M, N, K, lda, ldb, ldc, ldr, ab, bb, st);
    case GEMM_TN: return dispatch<true, true, EPI_F32_ACC>(a, b, C, r, M, N, K, lda, ldb, ldc, ldr, ab, bb, st);
  }
  return hipErrorInvalidValue;
}

bool gemm_tn_segments_ok(int kseg, int64_t lda, int64_t ldb) { return gemm_bf16_dma_ok(GEMM_TN, 8, 8, kseg, lda, ldb); }

// C[M,N] += sum_i A_i[kseg,M]^T * B_i[kseg,N] (fp32 C), the contraction of all pieces accumulated in registers and
// added to C once: the weight gradient of several micro-batches in one launch.  nseg <= 16.
hipError_t gemm_bf16_tn_segments(const void* const* A, const void* const* B, int nseg, void* C, int M, int N, int kseg,
                                 int64_t lda, int64_t ldb, int64_t ldc, hipStream_t st, int gu_f, bool overwrite) {
  if (M == 0 || N == 0 || nseg == 0 || kseg == 0) return hipSuccess;
  if (nseg > MAX_SEGS || (gu_f > 0 && (gu_f % 32 || N != 2 * gu_f))) return hipErrorInvalidValue;
  SegArgs sa = {};
  for (int i = 0; i < nseg; i++) {
    sa.a[i] = static_cast<const bf16_t*>(A[i]);
    sa.b[i] = static_cast<const bf16_t*>(B[i]);
  }
  sa.nseg = nseg;
  sa.kseg = kseg;
  const uint32_t ab = uint32_t(int64_t(kseg) * lda * 2), bb = uint32_t(int64_t(kseg) * ldb * 2);
  const ColumnPlan cp = plan_columns(M, N);
  const int ovw = overwrite ? 1 : 0;
  static const bool use_m16 = getenv("MLS_OLD_GEMM") == nullptr;
  if (cp.n1 > 0 && use_m16 && mls::gemm_m16_ok(mls::GEMM_TN, kseg)) {
    hipError_t e = mls::gemm_m16_tn_segments(A, B, nseg, C, M, cp.n1, kseg, lda, ldb, ldc, ab, bb, st, gu_f, overwrite);
    if (e != hipSuccess || cp.tail == TAIL_NONE) return e;
  } else
  if (cp.n1 > 0) {
    hipError_t e = launch<256, 256, 32, 4, true, true, EPI_F32_ACC, PIPE_SKEW, true>(sa.a[0], sa.b[0], C, nullptr, M, cp.n1, kseg, lda,
                                                                                    ldb, ldc, 0, ab, bb, st, &sa, 0, nullptr, ovw, gu_f);
    if (e != hipSuccess || cp.tail == TAIL_NONE) return e;
  }
  for (int i = 0; i < nseg; i++) sa.b[i] += cp.n1;
  if (cp.tail == TAIL_256x128)
    return launch<256, 128, 32, 4, true, true, EPI_F32_ACC, PIPE_SKEW, true>(sa.a[0], sa.b[0], C, nullptr, M, N - cp.n1, kseg, lda,
                                                                              ldb, ldc, 0, ab, bb, st, &sa, cp.n1, nullptr, ovw, gu_f);
  return launch<128, 128, 64, 3, true, true, EPI_F32_ACC, PIPE_PLAIN, true>(sa.a[0], sa.b[0], C, nullptr, M, N - cp.n1, kseg, lda,
                                                                             ldb, ldc, 0, ab, bb, st, &sa, cp.n1, nullptr, ovw, gu_f);
}

bool gemm_swiglu_ok(int M, int f, int K, int64_t lda, int64_t ldw, bool w_nk) {
  return f > 0 && f % 32 == 0 && gemm_bf16_dma_ok(w_nk ? GEMM_NT : GEMM_NN, M, 2 * f, K, lda, ldw);
}

hipError_t gemm_bf16_swiglu(const void* A, const void* W, void* GU, void* Z, int M, int f, int K, int64_t lda,
                            int64_t ldw, int64_t ldgu, int64_t ldz, hipStream_t st, bool w_nk) {
  if (M == 0 || f == 0) return hipSuccess;
  if (!gemm_swiglu_ok(M, f, K, lda, ldw, w_nk)) return hipErrorInvalidValue;
  Extra x;
  x.X = Z;
  x.ldx = ldz;
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w = static_cast<const bf16_t*>(W);
  const uint32_t ab = uint32_t(int64_t(M) * lda * 2), wb = uint32_t(int64_t(w_nk ? 2 * f : K) * ldw * 2);
  if (w_nk) return dispatch<false, false, EPI_SWIGLU>(a, w, GU, nullptr, M, 2 * f, K, lda, ldw, ldgu, 0, ab, wb, st, x);
  return dispatch<false, true, EPI_SWIGLU>(a, w, GU, nullptr, M, 2 * f, K, lda, ldw, ldgu, 0, ab, wb, st, x);
}

bool gemm_rope_ok(int M, int N, int K, int64_t lda, int64_t ldw, int seq, int rot_cols, int head_dim, bool w_nk) {
  return (head_dim == 64 || head_dim == 128) && seq > 0 && rot_cols >= 0 && rot_cols <= N && rot_cols % head_dim == 0 &&
         N % head_dim == 0 && gemm_bf16_dma_ok(w_nk ? GEMM_NT : GEMM_NN, M, N, K, lda, ldw);
}

hipError_t gemm_bf16_rope(const void* A, const void* W, void* C, int M, int N, int K, int64_t lda, int64_t ldw, int64_t ldc,
                          const float* cos_tab, const float* sin_tab, int seq, int rot_cols, int head_dim, hipStream_t st,
                          bool w_nk) {
  if (M == 0 || N == 0) return hipSuccess;
  if (!cos_tab || !sin_tab || !gemm_rope_ok(M, N, K, lda, ldw, seq, rot_cols, head_dim, w_nk)) return hipErrorInvalidValue;
  const RopeArgs ra = {cos_tab, sin_tab, seq, rot_cols, head_dim};
  Extra x;
  x.rope = &ra;
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w = static_cast<const bf16_t*>(W);
  const uint32_t ab = uint32_t(int64_t(M) * lda * 2), wb = uint32_t(int64_t(w_nk ? N : K) * ldw * 2);
  if (w_nk) return dispatch<false, false, EPI_ROPE>(a, w, C, nullptr, M, N, K, lda, ldw, ldc, 0, ab, wb, st, x);
  return dispatch<false, true, EPI_ROPE>(a, w, C, nullptr, M, N, K, lda, ldw, ldc, 0, ab, wb, st, x);
}

}  // namespace mls
