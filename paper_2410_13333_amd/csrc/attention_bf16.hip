// Causal grouped-query attention for bf16 storage on the gfx950 matrix cores: forward with online softmax,
// backward as three kernels (dQ, which also forms the row sums delta = dO . O; dK; dV) that recompute the
// probabilities from the saved log-sum-exp.
// Nothing of size S x S is ever written; no float atomics, so results are bitwise reproducible.
//
// Register-resident probabilities.  v_mfma_f32_32x32x16_bf16 leaves element (g*4+r) of lane l at
// [row (l/32)*4 + 8g + r][col l%32] of the 32x32 result and expects the B operand as "lane l holds column
// l%32, eight k-values".  All score-like products are therefore computed TRANSPOSED so that the softmax row
// index is the lane's column: a lane then owns all the probabilities of its row that it computed, can turn
// them into a B operand of the next product without leaving its registers, and keeps the running row
// maximum / sum as plain scalars.  The contraction index of that next product is permuted (k-values
// 4g..4g+3 and 8+4g..8+4g+3 per 16-step), which is free because the A operand is fetched with the same
// permutation by ds_read_b64_tr_b16 out of a tile stored [kv][d] just as it lies in memory.
//
// LDS tiles are 64 rows x D columns, unpadded, with an XOR swizzle of the 16-byte chunks that makes both
// access patterns bank-conflict free: ds_read_b128 of 16 consecutive rows at one column chunk, and the
// transposing 8-byte reads of 4 consecutive rows x 64 bytes.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;

// 16 bytes per lane from a raw buffer straight into LDS (64 lanes fill 1 KiB at lds_byte); out-of-range lanes
// are zero-filled.  Inline asm so that the waits are placed by hand (see gemm_bf16_dma.hip).
__device__ __forceinline__ void dma16(i32x4 rsrc, uint32_t voff, uint32_t lds_byte) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_byte), "v"(voff), "s"(rsrc)
               : "memory");
}
__device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ i32x4 make_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)p;
  i32x4 r;
  r[0] = (int)(uint32_t)a;
  r[1] = (int)((uint32_t)(a >> 32) & 0xffffu);
  r[2] = (int)bytes;
  r[3] = 0x00020000;
  return r;
}
constexpr uint32_t OOB = 0x80000000u;

constexpr int AT_THREADS = 256;
constexpr int TR = 64;  // rows of an LDS tile
constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;

// element offset of (row, col) inside a swizzled 64 x D tile
template <int D>
__device__ __forceinline__ int toff(int row, int col) {
  if (D == 128) {
    const int sw = ((row & 3) << 2) | ((row >> 2) & 3);
    return row * 128 + ((((col >> 3) ^ sw)) << 3) + (col & 7);
  } else {
    const int line = row >> 1;
    const int sw = ((line & 1) << 2) | ((line >> 1) & 3);
    return line * 128 + (((((row & 1) << 3) | (col >> 3)) ^ sw) << 3) + (col & 7);
  }
}

template <int D>
struct Tile {
  static constexpr int BYTES = TR * D * 2;
  static constexpr int NI = BYTES / 1024 / 4;  // DMA instructions per wave per tile
  // Per-lane source offsets (bytes, relative to element (row0, col0) of the source matrix) of this wave's DMA
  // instructions: instruction q = wave*NI + i fills LDS bytes [1024 q, 1024 q + 1024) of the tile, and the lane
  // that writes a given 16-byte slot fetches the chunk the swizzle assigns to it.
  uint32_t off[NI];
  __device__ __forceinline__ void init(int64_t ld, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NI; i++) {
      const int q = wave * NI + i;
      int row, chunk;
      if (D == 128) {
        row = q * 4 + (lane >> 4);
        chunk = (lane & 15) ^ (((row & 3) << 2) | ((row >> 2) & 3));
      } else {
        const int line = q * 4 + (lane >> 4);
        const int idx = (lane & 15) ^ (((line & 1) << 2) | ((line >> 1) & 3));
        row = line * 2 + (idx >> 3);
        chunk = idx & 7;
      }
      off[i] = uint32_t((int64_t(row) * ld + chunk * 8) * 2);
    }
  }
  // rows [row0, row0+64) x cols [col0, col0+D) of the matrix behind rsrc (row stride ld) -> tile at LDS byte
  // address `tile`; rows at or beyond the end of the buffer are zero-filled; live = false sends nothing useful
  __device__ __forceinline__ void dma(i32x4 rsrc, int64_t ld, int row0, int col0, uint32_t tile, int wave,
                                      bool live) const {
    const uint32_t base = uint32_t((int64_t(row0) * ld + col0) * 2);
#pragma unroll
    for (int i = 0; i < NI; i++) dma16(rsrc, live ? base + off[i] : OOB, tile + (wave * NI + i) * 1024);
  }
  // A operand, rows = tile rows rt*32 .. +31, k = tile columns kk*16 .. +15
  static __device__ __forceinline__ bf16x8 frag_rows(const bf16_t* t, int rt, int kk, int lane) {
    const uint4 v = *reinterpret_cast<const uint4*>(t + toff<D>(rt * 32 + (lane & 31), kk * 16 + (lane >> 5) * 8));
    return __builtin_bit_cast(bf16x8, v);
  }
  // A operand, rows = tile COLUMNS ct*32 .. +31, k = tile rows of the 16-step `ks` in the permuted order
  // that matches a B operand built from accumulator registers: k-values 4g..4g+3 then 8+4g..8+4g+3, g = lane/32.
  static __device__ __forceinline__ bf16x8 frag_cols(const bf16_t* t, int ct, int ks, int lane) {
    const int row = ks * 16 + (lane >> 5) * 4 + ((lane & 15) >> 2);
    const int col = ct * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLS_LDS s16x4*)(t + toff<D>(row, col)));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLS_LDS s16x4*)(t + toff<D>(row + 8, col)));
    s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
};

// B operand straight from global memory: column l%32 = matrix row row0 + l%32, k = matrix columns kk*16 + (l/32)*8 ..
__device__ __forceinline__ bf16x8 gfrag(const bf16_t* __restrict__ g, int64_t ld, int row, int col, bool valid) {
  uint4 v = make_uint4(0, 0, 0, 0);
  if (valid) v = *reinterpret_cast<const uint4*>(g + int64_t(row) * ld + col);
  return __builtin_bit_cast(bf16x8, v);
}

// two accumulator groups (2s, 2s+1) of a 32x32 result -> B operand of the next product
__device__ __forceinline__ bf16x8 acc_to_b(const f32x16& a, int s) {
  uint4 v;
  v.x = pack_bf16x2(a[8 * s + 0], a[8 * s + 1]);
  v.y = pack_bf16x2(a[8 * s + 2], a[8 * s + 3]);
  v.z = pack_bf16x2(a[8 * s + 4], a[8 * s + 5]);
  v.w = pack_bf16x2(a[8 * s + 6], a[8 * s + 7]);
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int e = 0; e < 16; e++) z[e] = 0.f;
  return z;
}

// N LDS fragment reads feeding N MFMAs, each read issued DEPTH fragments ahead of its use so that the LDS latency
// hides behind the MFMAs in between (left to itself the compiler reads every fragment right before its MFMA and
// waits for it).  read(i) returns fragment i (RPF LDS instructions each), use(i, f) issues the MFMA that takes it.
template <int N, int DEPTH, int RPF, class Read, class Use>
__device__ __forceinline__ void read_ahead(Read&& read, Use&& use) {
  bf16x8 f[N];  // fully unrolled: a fragment's registers are free again once its MFMA has issued
#pragma unroll
  for (int i = 0; i < DEPTH && i < N; i++) f[i] = read(i);
#pragma unroll
  for (int i = 0; i < N; i++) {
    if (i + DEPTH < N) f[i + DEPTH] = read(i + DEPTH);
    use(i, f[i]);
  }
  // the issue order the scheduler is asked for: DEPTH fragments, then MFMA / next fragment alternating
#pragma unroll
  for (int i = 0; i < DEPTH && i < N; i++) __builtin_amdgcn_sched_group_barrier(0x100, RPF, 0);
#pragma unroll
  for (int i = 0; i < N; i++) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (i + DEPTH < N) __builtin_amdgcn_sched_group_barrier(0x100, RPF, 0);
  }
}

// store a transposed 32x32 result (col l%32 = token, rows = feature index) as bf16: 4 consecutive features = 8 bytes
__device__ __forceinline__ void store_t(bf16_t* __restrict__ out, int64_t ld, int token, int col0, const f32x16& a,
                                        float mul, int lane, bool valid) {
  if (!valid) return;
#pragma unroll
  for (int g = 0; g < 4; g++) {
    uint2 v;
    v.x = pack_bf16x2(a[g * 4 + 0] * mul, a[g * 4 + 1] * mul);
    v.y = pack_bf16x2(a[g * 4 + 2] * mul, a[g * 4 + 3] * mul);
    *reinterpret_cast<uint2*>(out + int64_t(token) * ld + col0 + (lane >> 5) * 4 + 8 * g) = v;
  }
}

// The same store for a whole head vector of a gradient w.r.t. rotated q or k, turned back by the rotary angle of
// its position on the way out (the transpose of the forward rotation): with (g1, g2) the halves of the gradient,
// the result is (g1 c + g2 s, g2 c - g1 s).  Feature i of the first half sits in tile i / 32, its partner
// i + D/2 in tile i / 32 + D/64, same register.  cos_tab, sin_tab: [S][D/2] fp32; pos: position in the sequence.
template <int D>
__device__ __forceinline__ void store_t_unrotate(bf16_t* __restrict__ out, int64_t ld, int token, int pos, int col0,
                                                 const f32x16 (&a)[D / 32], float mul, const float* __restrict__ cos_tab,
                                                 const float* __restrict__ sin_tab, int lane, bool valid) {
  if (!valid) return;
  constexpr int H = D / 64, D2 = D / 2;
#pragma unroll
  for (int t = 0; t < H; t++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const int f = t * 32 + (lane >> 5) * 4 + 8 * g;
      const float4 c = *reinterpret_cast<const float4*>(cos_tab + int64_t(pos) * D2 + f);
      const float4 sn = *reinterpret_cast<const float4*>(sin_tab + int64_t(pos) * D2 + f);
      const float cs[4] = {c.x, c.y, c.z, c.w}, ss[4] = {sn.x, sn.y, sn.z, sn.w};
      float o1[4], o2[4];
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const float g1 = a[t][g * 4 + r] * mul, g2 = a[t + H][g * 4 + r] * mul;
        o1[r] = g1 * cs[r] + g2 * ss[r];
        o2[r] = g2 * cs[r] - g1 * ss[r];
      }
      uint2 v1, v2;
      v1.x = pack_bf16x2(o1[0], o1[1]); v1.y = pack_bf16x2(o1[2], o1[3]);
      v2.x = pack_bf16x2(o2[0], o2[1]); v2.y = pack_bf16x2(o2[2], o2[3]);
      *reinterpret_cast<uint2*>(out + int64_t(token) * ld + col0 + f) = v1;
      *reinterpret_cast<uint2*>(out + int64_t(token) * ld + col0 + D2 + f) = v2;
    }
}

// ================================================================ forward
// grid (n_q, q blocks of 128, b) with the longest query blocks dispatched first over all heads; wave w owns
// query rows q0 + 32w .. +31; loops over KV blocks of 64.  Two workgroups fit a CU.
template <int D>
__global__ __launch_bounds__(AT_THREADS, 2) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, int64_t ld, bf16_t* __restrict__ o, int64_t ldo,
                                                                 float* __restrict__ lse, int S, int nq, int nkv) {
  using TL = Tile<D>;
  constexpr int KD = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(1024))) bf16_t lds[2][2][TR * D];  // [buffer][K|V]
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qb = gridDim.y - 1 - blockIdx.y;  // longest rows first
  const int hq = blockIdx.x, bi = blockIdx.z, hk = hq / (nq / nkv);
  const bf16_t* base = qkv + int64_t(bi) * S * ld;
  const int q0 = qb * 128, qw = q0 + wave * 32, qi = qw + (lane & 31);
  const float sc = rsqrtf((float)D) * LOG2E;
  const i32x4 rsrc = make_rsrc(base, uint32_t(int64_t(S) * ld * 2));
  const uint32_t lds0 = (uint32_t)(uintptr_t)(MLS_LDS bf16_t*)&lds[0][0][0];
  TL tl;
  tl.init(ld, wave, lane);
  auto issue = [&](int blk, bool live) {  // K and V rows [64 blk, 64 blk + 64) into buffer blk & 1
    const uint32_t t = lds0 + (blk & 1) * 2 * TL::BYTES;
    tl.dma(rsrc, ld, blk * TR, (nq + hk) * D, t, wave, live);
    tl.dma(rsrc, ld, blk * TR, (nq + nkv + hk) * D, t + TL::BYTES, wave, live);
  };

  bf16x8 qf[KD];
#pragma unroll
  for (int kk = 0; kk < KD; kk++) qf[kk] = gfrag(base, ld, qi, hq * D + kk * 16 + (lane >> 5) * 8, qi < S);

  f32x16 acc[DT];
#pragma unroll
  for (int t = 0; t < DT; t++) acc[t] = zero16();
  float m = -INFINITY, l = 0.f;

  const int kv_end = min(S, q0 + 128);
  const int nblk = (kv_end + TR - 1) / TR;
  issue(0, true);
  for (int blk = 0; blk < nblk; blk++) {
    const int cur = blk & 1, j0 = blk * TR;
    wait_dma();       // this wave's part of block blk has landed ...
    __syncthreads();  // ... and so has everyone's; all reads of the other buffer are retired
    issue(blk + 1, blk + 1 < nblk);
    if (j0 <= qw + 31) {  // wave-uniform: some (i, j) pair of this wave is unmasked
      const bf16_t* ks = lds[cur][0];
      const bf16_t* vs = lds[cur][1];
      f32x16 st[2];
#pragma unroll
      for (int jt = 0; jt < 2; jt++) {
        st[jt] = zero16();
#pragma unroll
        for (int kk = 0; kk < KD; kk++)
          st[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_rows(ks, jt, kk, lane), qf[kk], st[jt], 0, 0, 0);
      }
      // row maximum of the raw scores (the scale is positive: it commutes with the maximum and is folded into the
      // exponent below); the mask arithmetic is compiled only into the diagonal-block path
      float mx = -INFINITY;
      auto mask_max = [&](auto MASK) {
#pragma unroll
        for (int jt = 0; jt < 2; jt++)
#pragma unroll
          for (int e = 0; e < 16; e++) {
            const int j = j0 + jt * 32 + (lane >> 5) * 4 + 8 * (e >> 2) + (e & 3);
            if (decltype(MASK)::value && j > qi) st[jt][e] = -INFINITY;
            mx = fmaxf(mx, st[jt][e]);
          }
      };
      if (j0 + TR - 1 > qw) mask_max(std::true_type{}); else mask_max(std::false_type{});  // some pair masked?
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mn = fmaxf(m, mx * sc);  // finite: block 0 always holds j = 0 <= i
      float ps = 0.f;
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const float p = __builtin_amdgcn_exp2f(st[jt][e] * sc - mn);
          st[jt][e] = p;
          ps += p;
        }
      // the running maximum rarely moves after the first blocks: rescale only when some row's did
      if (__any(mn > m)) {
        const float corr = __builtin_amdgcn_exp2f(m - mn);
        l *= corr;
#pragma unroll
        for (int t = 0; t < DT; t++)
#pragma unroll
          for (int e = 0; e < 16; e++) acc[t][e] *= corr;
        m = mn;
      }
      l += ps;
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int s = 0; s < 2; s++) {
          const bf16x8 pf = acc_to_b(st[jt], s);
#pragma unroll
          for (int t = 0; t < DT; t++)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_cols(vs, t, jt * 2 + s, lane), pf, acc[t], 0, 0, 0);
        }
    }
  }
  wait_dma();
  l += __shfl_xor(l, 32, 64);
  const float inv = 1.f / l;
  bf16_t* ob = o + int64_t(bi) * S * ldo;
#pragma unroll
  for (int t = 0; t < DT; t++) store_t(ob, ldo, qi, hq * D + t * 32, acc[t], inv, lane, qi < S);
  if (lane < 32 && qi < S) lse[(int64_t(bi) * nq + hq) * S + qi] = (m + __builtin_amdgcn_logf(l)) * LN2;
}

// ================================================================ backward: dQ
// Same decomposition as the forward.  Per KV block: S^T = K Q^T, dP^T = V dO^T, dS^T = P^T (dP^T - delta),
// dQ^T += K^T dS^T.
template <int D>
__global__ __launch_bounds__(AT_THREADS, 2) void attn_dq_kernel(const bf16_t* __restrict__ qkv, int64_t ld,
                                                                const bf16_t* __restrict__ o, int64_t ld_o,
                                                                const bf16_t* __restrict__ d_o, int64_t ldo,
                                                                const float* __restrict__ lse,
                                                                float* __restrict__ delta,
                                                                bf16_t* __restrict__ dqkv, int64_t ldg, int S, int nq,
                                                                int nkv, const float* __restrict__ cos_tab,
                                                                const float* __restrict__ sin_tab) {
  using TL = Tile<D>;
  constexpr int KD = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(1024))) bf16_t lds[2][2][TR * D];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qb = gridDim.y - 1 - blockIdx.y;
  const int hq = blockIdx.x, bi = blockIdx.z, hk = hq / (nq / nkv);
  const bf16_t* base = qkv + int64_t(bi) * S * ld;
  const bf16_t* dob = d_o + int64_t(bi) * S * ldo;
  const int q0 = qb * 128, qw = q0 + wave * 32, qi = qw + (lane & 31);
  const float scale = rsqrtf((float)D), sc = scale * LOG2E;
  const i32x4 rsrc = make_rsrc(base, uint32_t(int64_t(S) * ld * 2));
  const uint32_t lds0 = (uint32_t)(uintptr_t)(MLS_LDS bf16_t*)&lds[0][0][0];
  TL tl;
  tl.init(ld, wave, lane);
  auto issue = [&](int blk, bool live) {
    const uint32_t t = lds0 + (blk & 1) * 2 * TL::BYTES;
    tl.dma(rsrc, ld, blk * TR, (nq + hk) * D, t, wave, live);
    tl.dma(rsrc, ld, blk * TR, (nq + nkv + hk) * D, t + TL::BYTES, wave, live);
  };

  bf16x8 qf[KD], dof[KD];
#pragma unroll
  for (int kk = 0; kk < KD; kk++) {
    qf[kk] = gfrag(base, ld, qi, hq * D + kk * 16 + (lane >> 5) * 8, qi < S);
    dof[kk] = gfrag(dob, ldo, qi, hq * D + kk * 16 + (lane >> 5) * 8, qi < S);
  }
  const int64_t si = (int64_t(bi) * nq + hq) * S + qi;
  const float L2 = qi < S ? lse[si] * LOG2E : 0.f;
  // delta = dO . O of this lane's query row (the two lane halves hold complementary features); it is also
  // written out for the dK kernel, which runs after this one
  float dl = 0.f;
  {
    const bf16_t* ob = o + int64_t(bi) * S * ld_o;
#pragma unroll
    for (int kk = 0; kk < KD; kk++) {
      const bf16x8 of = gfrag(ob, ld_o, qi, hq * D + kk * 16 + (lane >> 5) * 8, qi < S);
#pragma unroll
      for (int e = 0; e < 8; e++) dl += (float)of[e] * (float)dof[kk][e];
    }
    dl += __shfl_xor(dl, 32, 64);
    if (lane < 32 && qi < S) delta[si] = dl;
  }

  f32x16 acc[DT];
#pragma unroll
  for (int t = 0; t < DT; t++) acc[t] = zero16();

  const int kv_end = min(S, q0 + 128);
  const int nblk = (kv_end + TR - 1) / TR;
  issue(0, true);
  for (int blk = 0; blk < nblk; blk++) {
    const int cur = blk & 1, j0 = blk * TR;
    wait_dma();
    __syncthreads();
    issue(blk + 1, blk + 1 < nblk);
    if (j0 <= qw + 31) {
      const bf16_t* ks = lds[cur][0];
      const bf16_t* vs = lds[cur][1];
      const bool diag = j0 + TR - 1 > qw;  // some pair of this wave is masked
      // one 32-key sub-block at a time, so that only one S^T / dP^T pair is live
#pragma unroll
      for (int jt = 0; jt < 2; jt++) {
        f32x16 st = zero16(), dp = zero16();
        read_ahead<2 * KD, 3, 1>(
            [&](int i) { return TL::frag_rows((i & 1) ? vs : ks, jt, i >> 1, lane); },
            [&](int i, const bf16x8& f) {
              if (i & 1) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, dof[i >> 1], dp, 0, 0, 0);
              else st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, qf[i >> 1], st, 0, 0, 0);
            });
        // key j = j0 + 32 jt + 4 (lane / 32) + off(e) is masked when j > qi, i.e. off(e) > lim; the mask arithmetic
        // is compiled only into the diagonal-block path
        const int lim = qi - (j0 + jt * 32 + (lane >> 5) * 4);
        auto to_ds = [&](auto MASK) {
#pragma unroll
          for (int e = 0; e < 16; e++) {
            float p = __builtin_amdgcn_exp2f(st[e] * sc - L2);
            if (decltype(MASK)::value && 8 * (e >> 2) + (e & 3) > lim) p = 0.f;
            st[e] = p * (dp[e] - dl);
          }
        };
        if (diag) to_ds(std::true_type{}); else to_ds(std::false_type{});
        const bf16x8 df[2] = {acc_to_b(st, 0), acc_to_b(st, 1)};
        read_ahead<2 * DT, 2, 2>([&](int i) { return TL::frag_cols(ks, i % DT, jt * 2 + i / DT, lane); },
                                 [&](int i, const bf16x8& f) {
                                   acc[i % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, df[i / DT], acc[i % DT], 0, 0, 0);
                                 });
      }
    }
  }
  wait_dma();
  bf16_t* out = dqkv + int64_t(bi) * S * ldg;
  if (cos_tab) {  // the gradient w.r.t. the rotated q, turned back to the projection's output on the way out
    store_t_unrotate<D>(out, ldg, qi, qi, hq * D, acc, scale, cos_tab, sin_tab, lane, qi < S);
  } else {
#pragma unroll
    for (int t = 0; t < DT; t++) store_t(out, ldg, qi, hq * D + t * 32, acc[t], scale, lane, qi < S);
  }
}

// ================================================================ backward: dK and dV (one kernel each)
// grid (n_kv, kv blocks of 128, b), longest first; wave w owns key rows j0 + 32w .. +31 and keeps their K (and V)
// as B operands.  Loops over the query heads of the group and the query blocks of 64 rows at or below the
// diagonal: S = Q K^T (lane column = key row), then
//   WHAT = 0 (dK):  dP = dO V^T, dS = P (dP - delta), dK^T += Q^T dS
//   WHAT = 1 (dV):  dV^T += dO^T P
// Two kernels on purpose: with both accumulators in one kernel the register demand passes 256, the MFMAs fall
// back to the accumulation-register form with hundreds of register copies per iteration, and only one workgroup
// fits a CU.  Apart, S is recomputed once more but each kernel runs two workgroups per CU.
template <int D, int WHAT>
__global__ __launch_bounds__(AT_THREADS, 2) void attn_dkv_kernel(const bf16_t* __restrict__ qkv, int64_t ld,
                                                                 const bf16_t* __restrict__ d_o, int64_t ldo,
                                                                 const float* __restrict__ lse,
                                                                 const float* __restrict__ delta,
                                                                 bf16_t* __restrict__ dqkv, int64_t ldg, int S, int nq,
                                                                 int nkv, int nsplit, float* __restrict__ part,
                                                                 const float* __restrict__ cos_tab,
                                                                 const float* __restrict__ sin_tab) {
  using TL = Tile<D>;
  constexpr bool DKM = WHAT == 0;
  constexpr int KD = D / 16, DT = D / 32;
  __shared__ __attribute__((aligned(1024))) bf16_t lds[2][2][TR * D];  // [buffer][Q|dO]
  __shared__ float stat[2][2][TR];                                       // [buffer][lse*log2e | delta]
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // nsplit > 1: the query heads of a group are shared out over nsplit workgroups (few KV heads would otherwise
  // leave most CUs idle); each writes its fp32 partial sum to `part`, which gqa_reduce_kernel adds up in order
  const int kb = blockIdx.y, hk = blockIdx.x / nsplit, sp = blockIdx.x % nsplit, bi = blockIdx.z;
  const int grp = nq / nkv / nsplit, hq0 = hk * (nq / nkv) + sp * grp;
  const bf16_t* base = qkv + int64_t(bi) * S * ld;
  const bf16_t* dob = d_o + int64_t(bi) * S * ldo;
  const int j0 = kb * 128, jw = j0 + wave * 32, ji = jw + (lane & 31);
  const float scale = rsqrtf((float)D), sc = scale * LOG2E;

  bf16x8 kf[KD], vf[DKM ? KD : 1];
#pragma unroll
  for (int kk = 0; kk < KD; kk++) {
    kf[kk] = gfrag(base, ld, ji, (nq + hk) * D + kk * 16 + (lane >> 5) * 8, ji < S);
    if (DKM) vf[kk] = gfrag(base, ld, ji, (nq + nkv + hk) * D + kk * 16 + (lane >> 5) * 8, ji < S);
  }
  f32x16 acc[DT];
#pragma unroll
  for (int t = 0; t < DT; t++) acc[t] = zero16();

  const int qb0 = j0 / TR, nqb = (S + TR - 1) / TR - qb0;  // query blocks per head
  const int niter = nqb > 0 ? nqb * grp : 0;
  const i32x4 rq_src = make_rsrc(base, uint32_t(int64_t(S) * ld * 2)), rd_src = make_rsrc(dob, uint32_t(int64_t(S) * ldo * 2));
  const uint32_t lds0 = (uint32_t)(uintptr_t)(MLS_LDS bf16_t*)&lds[0][0][0];
  TL tq, td;
  tq.init(ld, wave, lane);
  td.init(ldo, wave, lane);
  // The query blocks of a head are walked from the last one down to the diagonal: the workgroups of all key blocks
  // of that head (same XCD, started together) then read the same Q / dO tile at about the same time and share it in L2.
  // iteration `it`: Q and dO rows of one 64-row query block of one head of the group -> buffer it & 1; the row
  // statistics go through registers (threads 0..63: lse*log2e of row tid; threads 64..127: delta of row tid-64)
  float rs = 0.f;
  auto issue = [&](int it, bool live) {
    const int hq = hq0 + (live ? it / nqb : 0), i0 = (qb0 + (live ? nqb - 1 - it % nqb : 0)) * TR;
    const uint32_t t = lds0 + (it & 1) * 2 * TL::BYTES;
    tq.dma(rq_src, ld, i0, hq * D, t, wave, live);
    td.dma(rd_src, ldo, i0, hq * D, t + TL::BYTES, wave, live);
    if (live && threadIdx.x < (DKM ? 2 : 1) * TR) {
      const int r = threadIdx.x & (TR - 1);
      const int64_t si = (int64_t(bi) * nq + hq) * S + i0 + r;
      rs = 0.f;
      if (i0 + r < S) rs = threadIdx.x < TR ? lse[si] * LOG2E : delta[si];
    }
  };
  // the statistics fetched by issue(it) are stored after the compute of iteration it-1 (or before the loop)
  auto put_stat = [&](int it) {
    if (threadIdx.x < (DKM ? 2 : 1) * TR) stat[it & 1][threadIdx.x >> 6][threadIdx.x & (TR - 1)] = rs;
  };
  issue(0, niter > 0);
  put_stat(0);
  for (int it = 0; it < niter; it++) {
    const int cur = it & 1, i0 = (qb0 + nqb - 1 - it % nqb) * TR;
    wait_dma();
    __syncthreads();
    issue(it + 1, it + 1 < niter);
    if (i0 + TR - 1 >= jw) {  // wave-uniform: some query row at or below this wave's first key row
      const bf16_t* qs = lds[cur][0];
      const bf16_t* ds_ = lds[cur][1];
      const bool diag = i0 < jw + 31 || i0 + TR > S;  // some pair is masked, or the block runs past the last row
      const bf16_t* tx = DKM ? qs : ds_;
      // one 32-query sub-block at a time, so that only one S / dP pair is live
#pragma unroll
      for (int itl = 0; itl < 2; itl++) {
        f32x16 st = zero16(), dp = zero16();
        if (DKM) {
          read_ahead<2 * KD, 3, 1>(
              [&](int i) { return TL::frag_rows((i & 1) ? ds_ : qs, itl, i >> 1, lane); },
              [&](int i, const bf16x8& f) {
                if (i & 1) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, vf[DKM ? i >> 1 : 0], dp, 0, 0, 0);
                else st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, kf[i >> 1], st, 0, 0, 0);
              });
          auto to_ds = [&](auto MASK) {  // the mask arithmetic is compiled only into the diagonal-block path
#pragma unroll
            for (int e = 0; e < 16; e++) {
              const int r = itl * 32 + (lane >> 5) * 4 + 8 * (e >> 2) + (e & 3);
              float p = __builtin_amdgcn_exp2f(st[e] * sc - stat[cur][0][r]);
              if (decltype(MASK)::value && (i0 + r < ji || i0 + r >= S)) p = 0.f;
              st[e] = p * (dp[e] - stat[cur][1][r]);  // dS
            }
          };
          if (diag) to_ds(std::true_type{}); else to_ds(std::false_type{});
        } else {
          read_ahead<KD, 3, 1>([&](int i) { return TL::frag_rows(qs, itl, i, lane); },
                               [&](int i, const bf16x8& f) {
                                 st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, kf[i], st, 0, 0, 0);
                               });
          auto softmax = [&](auto MASK) {  // the mask arithmetic is compiled only into the diagonal-block path
#pragma unroll
            for (int e = 0; e < 16; e++) {
              const int r = itl * 32 + (lane >> 5) * 4 + 8 * (e >> 2) + (e & 3);
              float p = __builtin_amdgcn_exp2f(st[e] * sc - stat[cur][0][r]);
              if (decltype(MASK)::value && (i0 + r < ji || i0 + r >= S)) p = 0.f;
              st[e] = p;
            }
          };
          if (diag) softmax(std::true_type{}); else softmax(std::false_type{});
        }
        const bf16x8 bf[2] = {acc_to_b(st, 0), acc_to_b(st, 1)};
        read_ahead<2 * DT, 2, 2>([&](int i) { return TL::frag_cols(tx, i % DT, itl * 2 + i / DT, lane); },
                                 [&](int i, const bf16x8& f) {
                                   acc[i % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, bf[i / DT], acc[i % DT], 0, 0, 0);
                                 });
      }
    }
    if (it + 1 < niter) put_stat(it + 1);
  }
  wait_dma();
  if (nsplit == 1) {
    bf16_t* out = dqkv + int64_t(bi) * S * ldg;
    if (DKM && cos_tab) {  // dK is a gradient w.r.t. the rotated k (partial sums are turned back by the reduction)
      store_t_unrotate<D>(out, ldg, ji, ji, (nq + hk) * D, acc, scale, cos_tab, sin_tab, lane, ji < S);
    } else {
#pragma unroll
      for (int t = 0; t < DT; t++)
        store_t(out, ldg, ji, (DKM ? nq + hk : nq + nkv + hk) * D + t * 32, acc[t], DKM ? scale : 1.f, lane, ji < S);
    }
  } else if (ji < S) {
    // part: [dK | dV][b][n_kv][nsplit][S][D] fp32
    float* out = part + ((((int64_t(WHAT) * gridDim.z + bi) * nkv + hk) * nsplit + sp) * S + ji) * D;
    const float mul = DKM ? scale : 1.f;
#pragma unroll
    for (int t = 0; t < DT; t++)
#pragma unroll
      for (int g = 0; g < 4; g++)
        *reinterpret_cast<float4*>(out + t * 32 + (lane >> 5) * 4 + 8 * g) =
            make_float4(acc[t][g * 4] * mul, acc[t][g * 4 + 1] * mul, acc[t][g * 4 + 2] * mul, acc[t][g * 4 + 3] * mul);
  }
}

// dK, dV <- the partial sums of the nsplit workgroups of each KV head, added in ascending order.  A thread owns 8
// features of the first half of a head vector and their 8 partners in the second half, so that dK (a gradient
// w.r.t. the rotated k) can be turned back by the rotary angle when the tables are given.
__global__ __launch_bounds__(256) void gqa_reduce_kernel(const float* __restrict__ part, int nsplit, int b, int S, int D,
                                                         int nq, int nkv, bf16_t* __restrict__ dqkv, int64_t ldg,
                                                         const float* __restrict__ cos_tab,
                                                         const float* __restrict__ sin_tab) {
  const int64_t id = int64_t(blockIdx.x) * 256 + threadIdx.x;
  const int d2 = D >> 1, cpr = d2 >> 3;
  const int64_t total = int64_t(2) * b * nkv * S * cpr;
  if (id >= total) return;
  const int c = int(id % cpr) * 8;
  const int64_t row = id / cpr;               // (what, bi, hk, token)
  const int token = int(row % S);
  const int hk = int((row / S) % nkv), bi = int((row / S / nkv) % b), what = int(row / S / nkv / b);
  const float* p = part + ((((int64_t(what) * b + bi) * nkv + hk) * nsplit) * S + token) * D + c;
  float a1[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, a2[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int sp = 0; sp < nsplit; sp++) {
    float v1[8], v2[8];
    load8(p + int64_t(sp) * S * D, v1);
    load8(p + int64_t(sp) * S * D + d2, v2);
#pragma unroll
    for (int e = 0; e < 8; e++) {
      a1[e] += v1[e];
      a2[e] += v2[e];
    }
  }
  if (what == 0 && cos_tab) {
    float cs[8], sn[8];
    load8(cos_tab + int64_t(token) * d2 + c, cs);
    load8(sin_tab + int64_t(token) * d2 + c, sn);
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const float g1 = a1[e], g2 = a2[e];
      a1[e] = g1 * cs[e] + g2 * sn[e];
      a2[e] = g2 * cs[e] - g1 * sn[e];
    }
  }
  bf16_t* out = dqkv + (int64_t(bi) * S + token) * ldg + (what ? nq + nkv + hk : nq + hk) * D + c;
  store8(out, a1);
  store8(out + d2, a2);
}

}  // namespace

namespace mls {

hipError_t attn_fwd_bf16(const void* qkv, int64_t ld_qkv, void* o, int64_t ld_o, float* lse, int b, int S, int nq, int nkv,
                         int d, hipStream_t st) {
  if (b == 0 || S == 0) return hipSuccess;
  dim3 grid(nq, (S + 127) / 128, b);
  if (d == 128)
    hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, dim3(AT_THREADS), 0, st, (const bf16_t*)qkv, ld_qkv, (bf16_t*)o, ld_o,
                       lse, S, nq, nkv);
  else if (d == 64)
    hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, dim3(AT_THREADS), 0, st, (const bf16_t*)qkv, ld_qkv, (bf16_t*)o, ld_o,
                       lse, S, nq, nkv);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

// how many workgroups share the query heads of one KV group in the dK / dV kernels: the smallest divisor of the
// group size that gives every CU two workgroups (1 when the plain grid already does)
int gqa_split(int b, int S, int nq, int nkv) {
  const int grp = nq / nkv, blocks = nkv * ((S + 127) / 128) * b;
  int n = 1;
  while (n < grp && blocks * n < 512) {
    n++;
    while (grp % n) n++;
  }
  return n;
}

size_t attn_bwd_scratch_floats(int dt, int b, int S, int nq, int nkv, int d) {
  if (dt != DT_BF16 || nkv <= 0 || nq % nkv) return 0;
  const int n = gqa_split(b, S, nq, nkv);
  return n > 1 ? size_t(2) * b * nkv * n * S * d : 0;
}

hipError_t attn_bwd_bf16(const void* qkv, int64_t ld_qkv, const void* o, int64_t ld_o, const float* lse, const void* d_o,
                         int64_t ld_do, void* dqkv, int64_t ld_dqkv, float* delta, int b, int S, int nq, int nkv, int d,
                         hipStream_t st, float* part, const float* cos_tab, const float* sin_tab) {
  if (b == 0 || S == 0) return hipSuccess;
  if (!cos_tab != !sin_tab) return hipErrorInvalidValue;
  const int ns = part ? gqa_split(b, S, nq, nkv) : 1;
  dim3 gq(nq, (S + 127) / 128, b), gk(nkv * ns, (S + 127) / 128, b);
  if (d == 128) {
    hipLaunchKernelGGL(attn_dq_kernel<128>, gq, dim3(AT_THREADS), 0, st, (const bf16_t*)qkv, ld_qkv, (const bf16_t*)o, ld_o,
                       (const bf16_t*)d_o, ld_do, lse, delta, (bf16_t*)dqkv, ld_dqkv, S, nq, nkv, cos_tab, sin_tab);
    hipLaunchKernelGGL((attn_dkv_kernel<128, 0>), gk, dim3(AT_THREADS), 0, st, (const bf16_t*)qkv, ld_qkv,
                       (const bf16_t*)d_o, ld_do, lse, delta, (bf16_t*)dqkv, ld_dqkv, S, nq, nkv, ns, part, cos_tab, sin_tab);
    hipLaunchKernelGGL((attn_dkv_kernel<128, 1>), gk, dim3(AT_THREADS), 0, st, (const bf16_t*)qkv, ld_qkv,
                       (const bf16_t*)d_o, ld_do, lse, delta, (bf16_t*)dqkv, ld_dqkv, S, nq, nkv, ns, part, cos_tab, sin_tab);
  } else if (d == 64) {
    hipLaunchKernelGGL(attn_dq_kernel<64>, gq, dim3(AT_THREADS), 0, st, (const bf16_t*)qkv, ld_qkv, (const bf16_t*)o, ld_o,
                       (const bf16_t*)d_o, ld_do, lse, delta, (bf16_t*)dqkv, ld_dqkv, S, nq, nkv, cos_tab, sin_tab);
    hipLaunchKernelGGL((attn_dkv_kernel<64, 0>), gk, dim3(AT_THREADS), 0, st, (const bf16_t*)qkv, ld_qkv,
                       (const bf16_t*)d_o, ld_do, lse, delta, (bf16_t*)dqkv, ld_dqkv, S, nq, nkv, ns, part, cos_tab, sin_tab);
    hipLaunchKernelGGL((attn_dkv_kernel<64, 1>), gk, dim3(AT_THREADS), 0, st, (const bf16_t*)qkv, ld_qkv,
                       (const bf16_t*)d_o, ld_do, lse, delta, (bf16_t*)dqkv, ld_dqkv, S, nq, nkv, ns, part, cos_tab, sin_tab);
  } else {
    return hipErrorInvalidValue;
  }
  if (ns > 1) {
    const int64_t total = int64_t(2) * b * nkv * S * (d >> 4);
    hipLaunchKernelGGL(gqa_reduce_kernel, dim3(unsigned((total + 255) / 256)), dim3(256), 0, st, part, ns, b, S, d, nq, nkv,
                       (bf16_t*)dqkv, ld_dqkv, cos_tab, sin_tab);
  }
  return hipGetLastError();
}

hipError_t attn_fwd(int dt, const void* qkv, int64_t ld_qkv, void* o, int64_t ld_o, float* lse, int b, int S, int nq,
                    int nkv, int d, hipStream_t st) {
  return dt == DT_BF16 ? attn_fwd_bf16(qkv, ld_qkv, o, ld_o, lse, b, S, nq, nkv, d, st)
                       : attn_fwd_f32(qkv, ld_qkv, o, ld_o, lse, b, S, nq, nkv, d, st);
}
hipError_t attn_bwd(int dt, const void* qkv, int64_t ld_qkv, const void* o, int64_t ld_o, const float* lse,
                    const void* d_o, int64_t ld_do, void* dqkv, int64_t ld_dqkv, float* delta, int b, int S, int nq,
                    int nkv, int d, hipStream_t st, float* part, const float* cos_tab, const float* sin_tab) {
  if (dt != DT_BF16 && cos_tab) return hipErrorInvalidValue;  // only the bf16 kernels turn the rotation back themselves
  return dt == DT_BF16
             ? attn_bwd_bf16(qkv, ld_qkv, o, ld_o, lse, d_o, ld_do, dqkv, ld_dqkv, delta, b, S, nq, nkv, d, st, part, cos_tab, sin_tab)
             : attn_bwd_f32(qkv, ld_qkv, o, ld_o, lse, d_o, ld_do, dqkv, ld_dqkv, delta, b, S, nq, nkv, d, st);
}

}  // namespace mls
