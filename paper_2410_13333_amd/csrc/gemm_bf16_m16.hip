// bf16 GEMM on v_mfma_f32_16x16x32_bf16: the 256x256 tiles of the three contraction forms of a decoder layer.
//
// Why this instruction: on operands with random mantissas the chip is power-limited, and a stream of 16x16x32
// MFMAs sustains about 14 % more FLOP/s under that limit than a stream of 32x32x16 MFMAs (measured with a loop
// of nothing but MFMAs: 2050 against 1800 TFLOP/s).  The price is twice as many MFMA instructions, 16 cycles
// each, so that a wavefront can hide only about three other instructions behind one of them: the main loop
// below is therefore written out in its issue order (inline asm for the MFMAs, the LDS reads and the
// global->LDS requests; the compiler keeps volatile asm statements in program order).
//
// Shape: 4 wavefronts, one per SIMD, each owns 128x128 of the tile = 8x8 MFMA tiles = 64 accumulators of 4
// registers, all in AGPRs.  k-tiles are 32 deep (one MFMA's depth), NS = 4 stages (16 KiB of A, 16 KiB of B) in LDS, filled by
// buffer_load_dwordx4 ... lds.  The fragments of a whole k-tile (8 of A, 8 of B, 16 bytes per lane each) live in
// registers, in two sets: iteration t issues the MFMAs of tile t from one set while the LDS reads of tile t+1
// fill the other, so no MFMA ever waits for LDS.  One barrier per iteration (after waiting for this wavefront's
// share of tile t+2) frees the stage of tile t+1, which is refilled at once with tile t+NS+1: a tile is requested
// NS-1 = 3 iterations before it is read.
//
// LDS map: the A stages (16 KiB each), then the B stages.  A [k][col] tile has 512-byte k-rows, XOR swizzled on the
// global-address side (swz_kcol).  An operand stored [row][k] is fetched differently: a 32-deep tile would take 64
// bytes of every row, half a cache line, and the other half would be fetched again one k-tile later (the L1 does
// not keep it that long).  Its k-tiles are therefore requested in pairs: one request covers 8 rows x 128 bytes
// (whole lines), and the pair (tiles 2p, 2p+1) lands in two adjacent stages as one [row][64 k] block with 128-byte
// rows, the eight 16-byte chunks of a row permuted by (row >> 1) & 7 so that the fragment reads (plain 16-byte
// reads) of either k-tile are free of bank conflicts.  Request schedules, per wavefront:
//   TN (both [k][col])          8 per iteration (4 of A, 4 of B)
//   NN (A [row][k])             even iterations 12 (the pair of A, 4 of B), odd ones 4 (B)
//   NT (both [row][k])          8 per iteration: the pair of A in even iterations, the pair of B in odd ones; B has a
//                               ring of three pair slots (160 KiB of LDS in all) so that it runs a pair further ahead
//                               (3 does not divide the loop's period of 4: its slot is a run-time offset).
// What was measured on the 7B layer's shapes (TFLOP/s, random operands): pairing A alone lifted NT from 1330 to 1410;
// pairing B as well with all 16 requests in the even iterations fell back to 1375 (bursts stall the in-order issue
// of the wavefront), alternating A and B pairs reached 1460.  NT is now the fastest form (NN 1350, TN 1410), so
// the layer runs its forward products against transposed weight copies.
//
// Restrictions, checked by the launcher: K (and the piece length of a segmented contraction) a multiple of 32, of
// 64 when A is stored [row][k], so that no k-tile is ragged and no pair straddles the end; everything else (ragged
// M and N) is handled by out-of-range requests that zero-fill.  The launcher covers whole 256-column tiles; the
// column remainder of a problem runs on the kernels of gemm_bf16_dma.hip.
#include <type_traits>
#include <utility>

#include "common.h"
#include "kernels.h"

namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;

constexpr int BM = 256, BN = 256, BK = 32, NS = 4, NW = 4;
constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
constexpr int B_OFF = NS * A_BYTES;  // all A stages first, then all B stages
constexpr int LDS_BYTES = NS * (A_BYTES + B_BYTES);
constexpr int LDS_BYTES_NT = LDS_BYTES + 2 * B_BYTES;  // a [row][k] B has a ring of three pairs of stages
constexpr uint32_t OOB = 0x80000000u;
constexpr int MAX_SEGS = 16;

enum { E_BF16 = 0, E_F32 = 1, E_SWIGLU = 2, E_ROPE = 3 };
// The row of MFMAs (of 8) of an iteration before which the barrier sits.  The LDS reads are spread over rows 0..3;
// with the barrier one row later the last reads are back when the wavefront gets there (measured: 5 is 1 % faster
// than 4 for the [k][col] forms, 6 is 2 % slower for all: the requests then crowd into two rows).
constexpr int ROW2 = 5;

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

struct SegArgs {
  const bf16_t* a[MAX_SEGS];
  const bf16_t* b[MAX_SEGS];
  int nseg, kseg;
};
struct RopeArgs {
  const float* cos_tab;
  const float* sin_tab;
  int seq, rot_cols, head_dim;
};

__device__ __forceinline__ i32x4 make_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)p;
  i32x4 r;
  r[0] = (int)(uint32_t)a;
  r[1] = (int)((uint32_t)(a >> 32) & 0xffffu);  // stride 0: raw buffer, byte offsets
  r[2] = (int)bytes;
  r[3] = 0x00020000;
  return r;
}
// 16 bytes per lane from a raw buffer straight into LDS: 64 lanes fill 1 KiB at lds_byte.  soff is a scalar byte
// offset added to the address; it is not part of the range check (voff >= num_records zero-fills).
__device__ __forceinline__ void dma16s(i32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_byte) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(lds_byte), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lgkm0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// C tile (16 columns x 16 rows, transposed product): lane l ends up with C[row l%16][cols 4*(l/16) .. +3]
__device__ __forceinline__ void mfma16(f32x4& c, const i32x4& bfrag, const i32x4& afrag) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(bfrag), "v"(afrag));
}
template <int OFF>
__device__ __forceinline__ void lds_read16(i32x4& f, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f) : "v"(addr), "n"(OFF) : "memory");
}
// transposing read of a [k][col] tile: two 8-byte reads (k-rows kr and kr+4 of the lane's group of eight)
template <int OFF>
__device__ __forceinline__ void lds_read16_tr(i32x4& f, uint32_t addr) {
  i32x2 lo, hi;
  asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
               : "=&v"(lo), "=&v"(hi)
               : "v"(addr), "n"(OFF), "n"(OFF + 4 * BN * 2)
               : "memory");
  f = i32x4{lo[0], lo[1], hi[0], hi[1]};  // (the two halves are allocated as one register quad: no copies)
}

// [k][col] tiles: XOR applied to the 16-byte chunk index (0..31) of k-row kr.  A transposing 8-byte read takes, per
// group of 16 lanes, 32 bytes from each of k-rows kr0 .. kr0+3, and 32 lanes (two groups, k-rows 8 apart) go through
// the 64 banks together; k-rows lie 512 bytes = two bank rounds apart, so the eight 32-byte pieces must be moved to
// eight different places of a round: bits 2, 3 from kr & 3, bit 1 from bit 3 of kr.
__device__ __forceinline__ constexpr int swz_kcol(int kr) { return ((kr & 3) << 2) | (((kr >> 3) & 1) << 1); }

template <bool ATR, bool BTR, int EPI, bool SEG>
__global__ __launch_bounds__(NW * 64) void gemm16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                         void* __restrict__ Cv, const bf16_t* __restrict__ R, int M, int N,
                                                         int K, int64_t lda, int64_t ldb, int64_t ldc, int64_t ldr,
                                                         uint32_t a_bytes, uint32_t b_bytes, int tiles_m, int col0,
                                                         void* __restrict__ Xv, int64_t ldx, int xf, SegArgs segs,
                                                         RopeArgs rope) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  // tile of this workgroup: each XCD gets a contiguous run of tiles, walked in groups of 4 tile rows, N fastest
  const int nwg = gridDim.x, pid = blockIdx.x;
  const int xcd = pid & 7, q8 = nwg >> 3, rem = nwg & 7;
  const int tile = xcd * q8 + (xcd < rem ? xcd : rem) + (pid >> 3);
  const int gm = 4 < tiles_m ? 4 : tiles_m;
  const int per_group = gm * (nwg / tiles_m), grp = tile / per_group, first_m = grp * gm;
  const int gsz = min(tiles_m - first_m, gm), in_grp = tile - grp * per_group;
  const int m0 = (first_m + in_grp % gsz) * BM, n0 = (in_grp / gsz) * BN;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave & 1) * 128, wn = (wave >> 1) * 128;
  const int l16 = lane & 15, g4 = lane >> 4;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(MLS_LDS unsigned char*)smem;

  // ---- requests: 4 per operand per wavefront per k-tile (8 per pair of k-tiles for a [row][k] A); fixed per-lane
  // byte offsets, the k-tile enters as a scalar
  constexpr bool PAIR = !ATR, PAIRB = !BTR;
  static_assert(!((PAIR || PAIRB) && SEG), "segmented contractions are the [k][col] form");
  static_assert(PAIR || !PAIRB, "a [row][k] B comes with a [row][k] A only");
  constexpr int NGA = PAIR ? 8 : 4, NGB = PAIRB ? 8 : 4;
  uint32_t goa[NGA], gob[NGB];
#pragma unroll
  for (int i = 0; i < NGA; i++) {
    if (ATR) {  // [k][col]: k-rows 2q, 2q+1; 32 chunks per k-row
      const int q = wave * 4 + i;
      const int kr = q * 2 + (lane >> 5), c = (lane & 31) ^ swz_kcol(kr);
      goa[i] = m0 + c * 8 < M ? uint32_t((int64_t(kr) * lda + m0 + c * 8) * 2) : OOB;
    } else {    // [row][64 k]: rows 8q .. 8q+7; 8 chunks per row, LDS position p of a row holds chunk p ^ ((row >> 1) & 7)
      const int q = wave * 8 + i;
      const int r = q * 8 + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
      goa[i] = m0 + r < M ? uint32_t((int64_t(m0 + r) * lda + c * 8) * 2) : OOB;
    }
  }
#pragma unroll
  for (int i = 0; i < NGB; i++) {
    if (BTR) {
      const int q = wave * 4 + i;
      const int kr = q * 2 + (lane >> 5), c = (lane & 31) ^ swz_kcol(kr);
      gob[i] = n0 + c * 8 < N ? uint32_t((int64_t(kr) * ldb + n0 + c * 8) * 2) : OOB;
    } else {
      const int q = wave * 8 + i;
      const int r = q * 8 + (lane >> 3), c = (lane & 7) ^ ((r >> 1) & 7);
      gob[i] = n0 + r < N ? uint32_t((int64_t(n0 + r) * ldb + c * 8) * 2) : OOB;
    }
  }
  const int tps = SEG ? segs.kseg / BK : K / BK;            // k-tiles per piece
  const int nk = (SEG ? segs.nseg : 1) * tps;
  const uint32_t ka = ATR ? uint32_t(lda * (BK * 2)) : BK * 2;  // byte step of one k-tile
  const uint32_t kb = BTR ? uint32_t(ldb * (BK * 2)) : BK * 2;
  const i32x4 dead_a = make_rsrc(A, 0), dead_b = make_rsrc(B, 0);
  i32x4 ra = make_rsrc(SEG ? segs.a[0] : A, a_bytes), rb = make_rsrc(SEG ? segs.b[0] : B, b_bytes);
  int rq_tile = 0, rq_seg = 0, rq_in = 0;  // request cursor: next k-tile, its piece and its index inside the piece
  // request D of this wavefront for the cursor's k-tile into `stage`: D = 0..3 of A (unpaired form), 4..7 of B
  auto request = [&](int stage, auto DC) {
    constexpr int d = decltype(DC)::value;
    const bool live = rq_tile < nk;
    if constexpr (d < 4) dma16s(live ? ra : dead_a, goa[d & (NGA - 1)], uint32_t(rq_in) * ka, lds0 + stage * A_BYTES + wave * 4096 + d * 1024);
    else dma16s(live ? rb : dead_b, gob[(d - 4) & (NGB - 1)], uint32_t(rq_in) * kb, lds0 + B_OFF + stage * B_BYTES + wave * 4096 + (d - 4) * 1024);
  };
  // request D of this wavefront for the pair of k-tiles (2 pair, 2 pair + 1) of a [row][k] operand into stages 2 slot,
  // 2 slot + 1: D = 0..7 of A, 8..15 of B
  auto request_pair = [&](int slot, int pair, auto DC) {
    constexpr int d = decltype(DC)::value;
    if constexpr (d < 8)
      dma16s(2 * pair < nk ? ra : dead_a, goa[d & (NGA - 1)], uint32_t(pair) * (4 * BK), lds0 + slot * (2 * A_BYTES) + wave * 8192 + d * 1024);
    else
      dma16s(2 * pair < nk ? rb : dead_b, gob[(d - 8) & (NGB - 1)], uint32_t(pair) * (4 * BK),
             lds0 + B_OFF + slot + wave * 8192 + (d - 8) * 1024);  // (slot: a byte offset here)
  };
#define IC(n) std::integral_constant<int, n>{}
  auto request_b_all = [&](int stage) { request(stage, IC(4)); request(stage, IC(5)); request(stage, IC(6)); request(stage, IC(7)); };
  auto request_a_all = [&](int stage) { request(stage, IC(0)); request(stage, IC(1)); request(stage, IC(2)); request(stage, IC(3)); };
  auto request_pair_all = [&](int slot, int pair) {
    request_pair(slot, pair, IC(0)); request_pair(slot, pair, IC(1)); request_pair(slot, pair, IC(2)); request_pair(slot, pair, IC(3));
    request_pair(slot, pair, IC(4)); request_pair(slot, pair, IC(5)); request_pair(slot, pair, IC(6)); request_pair(slot, pair, IC(7));
  };
  auto request_pairb_all = [&](int slot, int pair) {
    request_pair(slot, pair, IC(8)); request_pair(slot, pair, IC(9)); request_pair(slot, pair, IC(10)); request_pair(slot, pair, IC(11));
    request_pair(slot, pair, IC(12)); request_pair(slot, pair, IC(13)); request_pair(slot, pair, IC(14)); request_pair(slot, pair, IC(15));
  };
  auto advance = [&]() {
    rq_tile++;
    rq_in++;
    if (SEG && rq_in == tps) {
      rq_in = 0;
      rq_seg++;
      const int i = rq_seg < segs.nseg ? rq_seg : segs.nseg - 1;
      ra = make_rsrc(segs.a[i], a_bytes);
      rb = make_rsrc(segs.b[i], b_bytes);
    }
  };

  // ---- fragment addresses: absolute LDS byte addresses for stage 0; stage and fragment index go into the read's
  // immediate offset, so the loop holds no address arithmetic (and the compiler has no reason to recycle a fragment
  // register while an MFMA may still read it).
  // [k][col]: one address per fragment (the swizzle mixes with the fragment index), second half at +4 k-rows.
  // [row][64 k]: one address per k-tile of the pair (the permutation turns the step from one to the other into an
  // XOR), fragment i at +2048 i.
  constexpr int NAA = ATR ? 8 : 2, NBA = BTR ? 8 : 2;
  uint32_t fa_b[NAA], fb_b[NBA];
  if (ATR) {
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const int kr = g4 * 8 + (l16 >> 2), col = wm + i * 16 + (l16 & 3) * 4;
      fa_b[i] = lds0 + kr * (BM * 2) + (((col >> 3) ^ swz_kcol(kr)) << 4) + (col & 7) * 2;
    }
  } else {
#pragma unroll
    for (int hf = 0; hf < 2; hf++) fa_b[hf] = lds0 + (wm + l16) * 128 + (((hf * 4 + g4) ^ ((l16 >> 1) & 7)) << 4);
  }
  if (BTR) {
#pragma unroll
    for (int j = 0; j < 8; j++) {
      const int kr = g4 * 8 + (l16 >> 2), col = wn + j * 16 + (l16 & 3) * 4;
      fb_b[j] = lds0 + B_OFF + kr * (BN * 2) + (((col >> 3) ^ swz_kcol(kr)) << 4) + (col & 7) * 2;
    }
  } else {
#pragma unroll
    for (int hf = 0; hf < 2; hf++) fb_b[hf] = lds0 + B_OFF + (wn + l16) * 128 + (((hf * 4 + g4) ^ ((l16 >> 1) & 7)) << 4);
  }
  i32x4 fa[2][8], fb[2][8];
  // A [row][k] B has a ring of three slots (pairs of stages), one more than A, so that its pairs can be requested a
  // pair further ahead; 3 does not divide the loop's period of 4 iterations, so its slot is a run-time offset: b_slot
  // is that of the pair being read, fb_cur the fragment addresses inside it (updated once per pair).
  uint32_t b_slot = 0, b_free = 0;  // b_free: the slot read before b_slot, free for the next pair
  uint32_t fb_cur[2] = {fb_b[0], fb_b[1]};
  auto next_b_slot = [&]() {
    b_free = b_slot;
    b_slot = b_slot == 4 * B_BYTES ? 0 : b_slot + 2 * B_BYTES;
    fb_cur[0] = fb_b[0] + b_slot;
    fb_cur[1] = fb_b[1] + b_slot;
  };
  // LDS read n (0..15; A fragments first) of the k-tile in stage ST into fragment set SET
  auto rd = [&](auto SETC, auto STC, auto NC) {
    constexpr int set = decltype(SETC)::value, st = decltype(STC)::value, n = decltype(NC)::value;
    if constexpr (n < 8) {
      if constexpr (ATR) lds_read16_tr<st * A_BYTES>(fa[set][n], fa_b[n]);
      else lds_read16<(st >> 1) * (2 * A_BYTES) + n * 2048>(fa[set][n], fa_b[st & 1]);
    } else {
      if constexpr (BTR) lds_read16_tr<st * B_BYTES>(fb[set][n - 8], fb_b[n - 8]);
      else lds_read16<(n - 8) * 2048>(fb[set][n - 8], fb_cur[st & 1]);
    }
  };

  f32x4 c[8][8];
#pragma unroll
  for (int i = 0; i < 8; i++)
#pragma unroll
    for (int j = 0; j < 8; j++) c[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- prologue: tiles 0 .. NS-1 requested; tile 0 read into set 0; tile 1 visible; tile NS requested into stage 0
  // (its B only in the paired form: iteration 0 requests the pair 4, 5)
  if constexpr (PAIRB) {  // B runs one pair further ahead than A
    request_pair_all(0, 0); request_pairb_all(0, 0);
    request_pair_all(1, 1); request_pairb_all(2 * B_BYTES, 1);
    request_pairb_all(4 * B_BYTES, 2);
    rq_tile = rq_in = NS;
    wait_vmcnt<24>();
  } else if constexpr (PAIR) {
    request_pair_all(0, 0);
    request_b_all(0); advance();
    request_b_all(1); advance();
    request_pair_all(1, 1);
    request_b_all(2); advance();
    request_b_all(3); advance();
    wait_vmcnt<20>();
  } else {
#pragma unroll
    for (int s = 0; s < NS; s++) {
      request_a_all(s);
      request_b_all(s);
      advance();
    }
    wait_vmcnt<(NS - 1) * 8>();
  }
  __syncthreads();
  {
#define RD0(n) rd(IC(0), IC(0), IC(n))
    RD0(0); RD0(1); RD0(2); RD0(3); RD0(4); RD0(5); RD0(6); RD0(7);
    RD0(8); RD0(9); RD0(10); RD0(11); RD0(12); RD0(13); RD0(14); RD0(15);
#undef RD0
  }
  wait_vmcnt<(NS - 2) * 8>();  // (both paired: tile 1 came with tile 0)
  wait_lgkm0();
  __syncthreads();
  if constexpr (!PAIR) request_a_all(0);
  if constexpr (!PAIRB) request_b_all(0);
  advance();

  // iteration t (fragment set SET = t % 2): tile t+1 sits in stage ST = (t + 1) % NS
  auto iteration = [&](auto SETC, auto STC) {
    constexpr int set = decltype(SETC)::value, st = decltype(STC)::value;
    if constexpr (PAIRB && (st & 1) == 0) next_b_slot();  // t odd: tile t+1 opens a new pair
    using SN = std::integral_constant<int, set ^ 1>;
    // first half: A fragments 0..3 against all of B, the 16 reads of tile t+1 in between
#define MM(i, j) mfma16(c[i][j], fb[set][j], fa[set][i])
#define RDN(n) rd(SN{}, STC, IC(n))
#define ROW_R(i, r0)                                                           \
  MM(i, 0); MM(i, 1); RDN(r0); MM(i, 2); MM(i, 3); RDN(r0 + 1);                \
  MM(i, 4); MM(i, 5); RDN(r0 + 2); MM(i, 6); MM(i, 7); RDN(r0 + 3);
    ROW_R(0, 0) ROW_R(1, 4) ROW_R(2, 8) ROW_R(3, 12)
#undef ROW_R
    // (the reads are all issued by now; ROW2 - 4 more rows of MFMAs cover the latency of the last ones)
    static_for<(ROW2 - 4) * 8>([&](auto MC) { MM(4 + decltype(MC)::value / 8, decltype(MC)::value % 8); });
    // this wavefront's share of tile t+2 has landed.  Unpaired: the requests of the last two iterations may be in
    // flight.  Paired, t even: tile t+2's A came with the pair of iteration t-2, after which only 4 + 4 requests of B
    // were issued; t odd: tile t+2 came with iteration t-3, followed by 4 + 12 requests.
    // Both paired (A pairs are requested in even iterations, B pairs in odd ones): t even: tile t+2's A came with
    // iteration t-2, its B with t-3, followed by the 8 requests of t-1; t odd: A came with t-3, B with t-4, followed
    // by the requests of t-2 and t-1.
    wait_vmcnt<PAIRB ? ((st & 1) ? 8 : 16) : PAIR ? ((st & 1) ? 8 : 16) : (NS - 2) * 8>();
    wait_lgkm0();                // its reads of tile t+1 are back
    __builtin_amdgcn_s_barrier();
    // second part: the remaining A fragments with the requests spread evenly in between.  Unpaired: 8 for tile
    // t+NS+1 into the stage just freed.  Paired, t even (ST odd): the pair (t+NS, t+NS+1) into stages ST-1, ST (tile t
    // was read in iteration t-1, tile t+1 just now), then B of tile t+NS+1; t odd: B only.  Both paired, t even: the
    // pair of A; t odd: the pair (t+5, t+6) of B into the slot of tiles t-1, t of its ring (read by the last barrier).
    const int pair = (rq_tile - 1) >> 1;
    constexpr bool even = (st & 1) != 0;
    constexpr int nreq = !PAIR ? 8 : PAIRB ? 8 : even ? 12 : 4;
    auto rqn = [&](auto NC) {
      constexpr int n = decltype(NC)::value;
      if constexpr (!PAIR) request(st, IC(n));
      else if constexpr (PAIRB && even) request_pair(st >> 1, pair, IC(n));
      else if constexpr (PAIRB) request_pair(b_free, pair + 1, IC(8 + n));
      else if constexpr (even && n < 8) request_pair(st >> 1, pair, IC(n));
      else if constexpr (even) request(st, IC(n - 4));
      else request(st, IC(4 + n));
    };
    constexpr int slots = (8 - ROW2) * 8;
    static_for<slots>([&](auto MC) {
      constexpr int m = decltype(MC)::value;
      static_for<nreq>([&](auto RC) {
        if constexpr ((decltype(RC)::value * slots) / nreq == m) rqn(RC);
      });
      MM(ROW2 + m / 8, m % 8);
    });
#undef RDN
#undef MM
    advance();
  };
  // in groups of four (one turn of the stage ring): the tiles beyond the last one are zero-filled (descriptor of
  // length zero) and add nothing
  // The compiler does not see MFMAs written as asm and inserts no wait states behind them; whatever it places at
  // the loop exit (copies of accumulators) must find the last MFMA's result written: 16 idle cycles per turn.
  for (int t = 0; t < nk; t += 4) {
    iteration(IC(0), IC(1));
    iteration(IC(1), IC(2));
    iteration(IC(0), IC(3));
    iteration(IC(1), IC(0));
    asm volatile("s_nop 15" ::: "memory");
  }
#undef IC
  wait_vmcnt<0>();
  __syncthreads();

  // ---- epilogue.  Lane l holds, of MFMA tile (i, j): C[row 16 i + l%16][cols 16 j + 4 (l/16) .. +3].
  const int64_t crow0 = m0 + wm, ccol0 = n0 + wn;
  if constexpr (EPI == E_F32) {
    // C (+)= acc in fp32, straight from the accumulator layout (16 bytes per lane); xf > 0: the columns are in the
    // interleaved gate/up order and go to their public places
    float* C = reinterpret_cast<float*>(Cv);
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const int64_t row = crow0 + i * 16 + l16;
      if (row >= M) continue;
#pragma unroll
      for (int j = 0; j < 8; j++) {
        const int col = int(ccol0) + j * 16 + g4 * 4;
        if (col >= N) continue;
        float4* p = reinterpret_cast<float4*>(C + row * ldc + (xf > 0 ? gu_public_col(col0 + col, xf) : col0 + col));
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ldx == 0) t = *p;  // ldx != 0 in this mode: store, do not accumulate
        t.x += c[i][j][0]; t.y += c[i][j][1]; t.z += c[i][j][2]; t.w += c[i][j][3];
        *p = t;
      }
    }
  } else {
    // bf16 output through a per-wavefront staging area (16 rows x 128 columns = 4 KiB, 16-byte chunks XOR-swizzled by
    // row) so that the stores move whole 256-byte rows.  The fused forms work on the fp32 accumulators first:
    //   E_ROPE    a head (64 or 128 columns) lies inside the wavefront's 128 columns, so both values of a rotary pair
    //             (i, i + head_dim/2) sit in the same lane, head_dim/32 MFMA tiles apart: rotate, then round once;
    //   E_SWIGLU  columns come as 32 gates, their 32 ups, ...: the up of a gate sits two MFMA tiles to the right in
    //             the same lane; C gets both, X[row][f] their product silu(gate) * up formed in fp32.
    unsigned char* ws = smem + wave * 8192;
    unsigned char* wz = ws + 4096;
    bf16_t* C = reinterpret_cast<bf16_t*>(Cv);
    // E_ROPE: the rotary table entries of a block of 16 rows (16 positions x head_dim/2 cosines and sines, fp32) come
    // through LDS as well: requested by buffer_load ... lds two blocks ahead into a ring of three slots per wavefront
    // (cos 4 KiB | sin 4 KiB each, behind the staging areas), read back as 16 bytes per lane.  The wavefront is alone
    // on its SIMD here: as plain loads, used right away, the entries cost their full latency in every block (48 us per
    // launch at the 7B shape), and held in registers ahead of time they spill.  A row of a slot keeps its 16-byte
    // chunks XORed with the row index (bank conflicts), applied on the global-address side.
    const bool use_rope = EPI == E_ROPE && col0 + int(ccol0) < rope.rot_cols;  // wave-uniform: whole heads; v is not rotated
    constexpr int RING0 = 32768, RING_SLOT = 8192;
    const uint32_t ring = lds0 + RING0 + wave * (3 * RING_SLOT);
    const unsigned char* ringp = smem + RING0 + wave * (3 * RING_SLOT);
    i32x4 cos_src = {}, sin_src = {};
    int p0 = 0;
    if constexpr (EPI == E_ROPE) {
      const uint32_t tab_bytes = uint32_t(rope.seq) * uint32_t(rope.head_dim / 2) * 4u;
      cos_src = make_rsrc(rope.cos_tab, tab_bytes);
      sin_src = make_rsrc(rope.sin_tab, tab_bytes);
      p0 = int(crow0 % rope.seq);
    }
    // TP = MFMA tiles between the halves of a rotary pair (head_dim / 32); a table row is 64 TP bytes = 4 TP chunks
    auto rope_request = [&](int i, auto TPC) {
      constexpr int TP = decltype(TPC)::value, CPR = 4 * TP, RPI = 16 / TP;  // chunks per row, rows per request
#pragma unroll
      for (int q = 0; q < TP; q++) {
        const int r = q * RPI + lane / CPR;  // row of the block
        int pos = p0 + i * 16 + r;           // its position in the sequence
        if (rope.seq >= 128) pos = pos >= rope.seq ? pos - rope.seq : pos;
        else pos = pos % rope.seq;
        const int sw = TP == 4 ? r : (r >> 1) & 7;
        const uint32_t off = crow0 + i * 16 + r < M ? uint32_t(pos * (64 * TP) + (((lane % CPR) ^ sw) << 4)) : OOB;
        dma16s(cos_src, off, 0, ring + (i % 3) * RING_SLOT + q * 1024);
        dma16s(sin_src, off, 0, ring + (i % 3) * RING_SLOT + 4096 + q * 1024);
      }
    };
    auto rope_request_any = [&](int i) {
      if (rope.head_dim == 128) rope_request(i, std::integral_constant<int, 4>{}); else rope_request(i, std::integral_constant<int, 2>{});
    };
    if constexpr (EPI == E_ROPE) {
      if (use_rope) {
        rope_request_any(0);
        rope_request_any(1);
      }
    }
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const int64_t row = crow0 + i * 16 + l16;
      float v[8][4];
#pragma unroll
      for (int j = 0; j < 8; j++)
#pragma unroll
        for (int e = 0; e < 4; e++) v[j][e] = c[i][j][e];
      if constexpr (EPI == E_BF16) {
        if (R) {
#pragma unroll
          for (int j = 0; j < 8; j++) {
            const int col = int(ccol0) + j * 16 + g4 * 4;
            if (row < M && col < N) {
              float r4[4];
              load4(R + row * ldr + col0 + col, r4);
              v[j][0] += r4[0]; v[j][1] += r4[1]; v[j][2] += r4[2]; v[j][3] += r4[3];
            }
          }
        }
      }
      if constexpr (EPI == E_ROPE) {
        auto rotate = [&](auto TPC) {
          constexpr int TP = decltype(TPC)::value;
          if (i + 2 < 8) rope_request(i + 2, TPC);
          // the requests of block i are older than those of blocks i+1 and i+2 (2 TP each) and than every store in
          // between, which can only make this wait longer than needed
          if (i + 2 < 8) wait_vmcnt<4 * TP>();
          else if (i + 1 < 8) wait_vmcnt<2 * TP>();
          else wait_vmcnt<0>();
          const int sw = TP == 4 ? l16 : (l16 >> 1) & 7;
          const unsigned char* slot = ringp + (i % 3) * RING_SLOT + l16 * (64 * TP);
#pragma unroll
          for (int j = 0; j < 8; j++) {
            if ((j % (2 * TP)) >= TP) continue;  // second halves go with their firsts
            const int jp = j + TP;
            const int ch = ((j % TP) * 4 + g4) ^ sw;  // chunk of features 16 (j % TP) + 4 g4 .. +3
            const float4 cs = *reinterpret_cast<const float4*>(slot + (ch << 4));
            const float4 sn = *reinterpret_cast<const float4*>(slot + 4096 + (ch << 4));
            const float cc[4] = {cs.x, cs.y, cs.z, cs.w}, ss[4] = {sn.x, sn.y, sn.z, sn.w};
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const float u1 = v[j][e], u2 = v[jp][e];
              v[j][e] = u1 * cc[e] - u2 * ss[e];
              v[jp][e] = u1 * ss[e] + u2 * cc[e];
            }
          }
        };
        if (use_rope) {
          if (rope.head_dim == 128) rotate(std::integral_constant<int, 4>{}); else rotate(std::integral_constant<int, 2>{});
        }
      }
#pragma unroll
      for (int j = 0; j < 8; j++) {
        uint2 o;
        o.x = pack_bf16x2(v[j][0], v[j][1]);
        o.y = pack_bf16x2(v[j][2], v[j][3]);
        const int ch = j * 2 + (g4 >> 1);
        *reinterpret_cast<uint2*>(ws + l16 * 256 + ((ch ^ l16) << 4) + (g4 & 1) * 8) = o;
      }
      if constexpr (EPI == E_SWIGLU) {
        // gate tiles 0, 1, 4, 5 with their ups 2, 3, 6, 7 -> product tiles 0..3 (64 columns of X, 128 bytes per row)
#pragma unroll
        for (int zb = 0; zb < 4; zb++) {
          const int jg = (zb >> 1) * 4 + (zb & 1), ju = jg + 2;
          float z[4];
#pragma unroll
          for (int e = 0; e < 4; e++) z[e] = v[jg][e] * sigmoidf_(v[jg][e]) * v[ju][e];
          uint2 o;
          o.x = pack_bf16x2(z[0], z[1]);
          o.y = pack_bf16x2(z[2], z[3]);
          const int ch = zb * 2 + (g4 >> 1);
          *reinterpret_cast<uint2*>(wz + l16 * 128 + ((ch ^ (l16 & 7)) << 4) + (g4 & 1) * 8) = o;
        }
      }
      wave_lds_sync();
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int rr = q * 4 + g4;
        const uint4 o = *reinterpret_cast<const uint4*>(ws + rr * 256 + ((l16 ^ rr) << 4));
        const int64_t grow = crow0 + i * 16 + rr;
        const int gcol = int(ccol0) + l16 * 8;
        if (grow < M && gcol < N) *reinterpret_cast<uint4*>(C + grow * ldc + col0 + gcol) = o;
      }
      if constexpr (EPI == E_SWIGLU) {
        bf16_t* X = reinterpret_cast<bf16_t*>(Xv);
#pragma unroll
        for (int q = 0; q < 2; q++) {
          const int rr = q * 8 + (lane >> 3), chk = lane & 7;
          const uint4 o = *reinterpret_cast<const uint4*>(wz + rr * 128 + ((chk ^ (rr & 7)) << 4));
          const int64_t grow = crow0 + i * 16 + rr;
          const int gcol = int(ccol0) + (chk >> 2) * 64 + (chk & 3) * 8;  // the gate column of this chunk's first product
          const int zcol = ((col0 + int(ccol0)) >> 1) + chk * 8;       // its place among the f products
          if (grow < M && gcol < N) *reinterpret_cast<uint4*>(X + grow * ldx + zcol) = o;
        }
      }
      wave_lds_sync();
    }
  }
}

template <bool ATR, bool BTR, int EPI, bool SEG>
hipError_t launch16(const bf16_t* A, const bf16_t* B, void* C, const bf16_t* R, int M, int N, int K, int64_t lda,
                    int64_t ldb, int64_t ldc, int64_t ldr, uint32_t ab, uint32_t bb, hipStream_t st, const SegArgs* segs,
                    void* X, int64_t ldx, int xf, const RopeArgs* rope) {
  auto kern = gemm16_kernel<ATR, BTR, EPI, SEG>;
  SegArgs sa = {};
  if (segs) sa = *segs;
  RopeArgs rp = {};
  if (rope) rp = *rope;
  static std::atomic<uint64_t> lds_raised{0};
  constexpr int LDS = BTR ? LDS_BYTES : LDS_BYTES_NT;
  if (hipError_t e = mls::raise_lds_limit(reinterpret_cast<const void*>(kern), LDS, lds_raised)) return e;
  const int tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tm * tn), dim3(NW * 64), LDS, st, A, B, C, R, M, N, K, lda, ldb, ldc, ldr, ab, bb, tm, 0, X,
                     ldx, xf, sa, rp);
  return hipGetLastError();
}

}  // namespace

namespace mls {

// k-tiles must be whole; an A stored [row][k] (NN, NT) is fetched in pairs of k-tiles
bool gemm_m16_ok(int mode, int K) { return K > 0 && K % (mode == GEMM_TN ? BK : 2 * BK) == 0; }

// C[M, N] (N a multiple of 256 or the whole problem) in one of the three modes; bf16 C (+ R) for NN and NT, fp32
// C (+)= for TN.  Operand byte lengths as the DMA path takes them.
hipError_t gemm_m16(int mode, const void* A, const void* B, void* C, const void* R, int M, int N, int K, int64_t lda,
                    int64_t ldb, int64_t ldc, int64_t ldr, uint32_t ab, uint32_t bb, hipStream_t st) {
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* b = static_cast<const bf16_t*>(B);
  const bf16_t* r = static_cast<const bf16_t*>(R);
  switch (mode) {
    case GEMM_NN: return launch16<false, true, E_BF16, false>(a, b, C, r, M, N, K, lda, ldb, ldc, ldr, ab, bb, st, nullptr, nullptr, 0, 0, nullptr);
    case GEMM_NT: return launch16<false, false, E_BF16, false>(a, b, C, r, M, N, K, lda, ldb, ldc, ldr, ab, bb, st, nullptr, nullptr, 0, 0, nullptr);
    case GEMM_TN: return launch16<true, true, E_F32, false>(a, b, C, r, M, N, K, lda, ldb, ldc, ldr, ab, bb, st, nullptr, nullptr, 0, 0, nullptr);
  }
  return hipErrorInvalidValue;
}


// GU[M, N = 2f] = A[M,K] W[K, 2f] (interleaved gate/up columns), Z[M, f] = silu(gate) * up; N a multiple of 256 here.
// w_nk: W is given transposed, [2f][K] with row stride ldw.
hipError_t gemm_m16_swiglu(const void* A, const void* W, void* GU, void* Z, int M, int N, int K, int64_t lda, int64_t ldw,
                           int64_t ldgu, int64_t ldz, uint32_t ab, uint32_t bb, hipStream_t st, bool w_nk) {
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w = static_cast<const bf16_t*>(W);
  if (w_nk) return launch16<false, false, E_SWIGLU, false>(a, w, GU, nullptr, M, N, K, lda, ldw, ldgu, 0, ab, bb, st, nullptr, Z, ldz, 0, nullptr);
  return launch16<false, true, E_SWIGLU, false>(a, w, GU, nullptr, M, N, K, lda, ldw, ldgu, 0, ab, bb, st, nullptr, Z, ldz, 0, nullptr);
}
// C[M, N] = A[M,K] W[K,N] with the head vectors in the columns below rot_cols rotated by the angle of their row's
// position.  w_nk: W is given transposed, [N][K] with row stride ldw.
hipError_t gemm_m16_rope(const void* A, const void* W, void* C, int M, int N, int K, int64_t lda, int64_t ldw, int64_t ldc,
                         uint32_t ab, uint32_t bb, const float* cos_tab, const float* sin_tab, int seq, int rot_cols,
                         int head_dim, hipStream_t st, bool w_nk) {
  const RopeArgs ra = {cos_tab, sin_tab, seq, rot_cols, head_dim};
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* w = static_cast<const bf16_t*>(W);
  if (w_nk) return launch16<false, false, E_ROPE, false>(a, w, C, nullptr, M, N, K, lda, ldw, ldc, 0, ab, bb, st, nullptr, nullptr, 0, 0, &ra);
  return launch16<false, true, E_ROPE, false>(a, w, C, nullptr, M, N, K, lda, ldw, ldc, 0, ab, bb, st, nullptr, nullptr, 0, 0, &ra);
}

// C[M, N] (+)= sum_i A_i[kseg, M]^T B_i[kseg, N] in fp32 over nseg <= 16 pieces (kseg a multiple of 32), N a multiple
// of 256 or the whole problem; gu_f > 0: interleaved gate/up columns go to their public places; overwrite: C =.
hipError_t gemm_m16_tn_segments(const void* const* A, const void* const* B, int nseg, void* C, int M, int N, int kseg,
                                int64_t lda, int64_t ldb, int64_t ldc, uint32_t ab, uint32_t bb, hipStream_t st, int gu_f,
                                bool overwrite) {
  if (nseg < 1 || nseg > MAX_SEGS || kseg % BK) return hipErrorInvalidValue;
  SegArgs sa = {};
  for (int i = 0; i < nseg; i++) {
    sa.a[i] = static_cast<const bf16_t*>(A[i]);
    sa.b[i] = static_cast<const bf16_t*>(B[i]);
  }
  sa.nseg = nseg;
  sa.kseg = kseg;
  return launch16<true, true, E_F32, true>(sa.a[0], sa.b[0], C, nullptr, M, N, kseg, lda, ldb, ldc, 0, ab, bb, st, &sa, nullptr,
                                           overwrite ? 1 : 0, gu_f, nullptr);
}

}  // namespace mls
