// dK, dV of the causal flash attention at head width 128 on 16-row wave tiles
// (v_mfma_f32_16x16x32_bf16).  See attn_mfma_common.h for the LDS tile layout and the loads.
//
// Why 16 rows and not the 32 of the other attention kernels: with 32 keys per wave the accumulators
// of dK and dV and the K and V operands take 192 registers, the kernel runs one wave per SIMD, and
// every wait of that lone wave is idle time of its matrix core (measured: matrix cores 39 % busy).
// With 16 keys per wave they take 96 (64 accumulator + 32 operand registers), a workgroup of four
// waves covers 64 keys and needs 66 KB of LDS, and two independent workgroups share a CU: while
// one waits or does its vector work, the other feeds the matrix core.  The price is LDS traffic:
// a wave reads the same 32 KB of Q / dO fragments per 32 queries as before, for half as many
// keys (116 B/clk/CU): the LDS is busy half of the time, which is why its reads have to be free of
// bank conflicts here (swz16 below).  Measured at 128 heads x 2048^2: 711 K -> 580 K clocks per CU,
// matrix cores 47 % busy, the backward pass (dQ + dK/dV) 620 -> 595 us.
//
// MFMA 16x16x32 lane layout (lane l, i = l & 15, g = l >> 4): first operand element e of row i is
// k = 8 g + e; second operand likewise for column i; accumulator r = 0..3 holds row 4 g + r,
// column i.  Per 32-query half and wave:
//   P1  S = Q K^T and dP = dO V^T: first operand = 16 query rows x 32 dh from LDS (128-bit reads),
//       second = this wave's 16 keys from registers; two query groups x four k-steps each
//   V   P = 2^(c S - lse log2 e), dS = P (dP - delta), packed to bf16.  A lane then holds, for its
//       key, queries 4 g + r of both query groups: taken as the second operand of the next
//       products this assigns k-slot (g, e) to query 4 g + e (e < 4) or 16 + 4 g + e - 4
//   P3  dV^T += dO^T P and dK^T += Q^T dS, eight 16-wide d tiles each, one MFMA per tile (the
//       contraction is the 32 queries); first operand through the LDS transpose read, whose two
//       reads deliver exactly those two runs of four query rows.
// One writer per key row, no atomics.
#include "attn_mfma_common.h"

namespace fax {

typedef __attribute__((ext_vector_type(4))) float f32x4;

// LDS tiles here are [64 rows][DH] bf16 like everywhere else, but with a swizzle of their own: the
// 16-byte chunk index is XOR-ed with s(row) = (pair(row) << 1) | bit 3 of row, where
// pair(row) = (row & 3) | ((bit 2 ^ bit 3 of row) << 2).
//   * 128-bit row-fragment reads: 16 lanes take 16 consecutive rows at one chunk position; s is a
//     bijection on 16 rows, so they land in 16 distinct chunks = all 64 banks.
//   * transpose reads: a 16-lane block takes 4 rows x 32 bytes, so 32 lanes take 8 rows and need 8
//     distinct 32-byte pairs of the 256-byte row.  Which two blocks the LDS serves together is not
//     documented; pair() is distinct over rows 0-7 and 8-15 (blocks 0+1, 2+3) and also over rows
//     {0-3, 8-11} and {4-7, 12-15} (blocks 0+2, 1+3).  Measured: a swizzle that only covers the first
//     grouping left 31 % of the LDS cycles in bank conflicts (the other kernels' swizzle, made
//     for 32-row tiles, 47 %); this one leaves none, and the kernel went from 648 K to 580 K clocks.
__device__ __forceinline__ int swz16(int row) {
  const int pair = (row & 3) | ((((row >> 2) ^ (row >> 3)) & 1) << 2);
  return (pair << 1) | ((row >> 3) & 1);
}

// Segment i of this wave's share of a 64 x DH tile, as tile_dma_seg() but with the swizzle above.
template <int DH>
__device__ __forceinline__ void tile_dma_seg16(unsigned lds, const bf16_t* __restrict__ src, size_t ld, int wave, int i) {
  constexpr int NCH = DH / 8, RPI = 64 / NCH;
  static_assert(NCH == 16, "the swizzle is written for 16 chunks per row");
  const int lane = threadIdx.x & 63;
  const int seg = wave * (DH / 32) + i;
  const int row = seg * RPI + lane / NCH;
  const int chunk = (lane % NCH) ^ swz16(row);
  lds_dma16(src, (unsigned)(((size_t)row * ld + chunk * 8) * sizeof(bf16_t)), lds + seg * 1024u);
}

// First operand, 16 rows rb..rb+15 of the tile (rb a multiple of 16), k-step ks (32 columns).
template <int DH>
__device__ __forceinline__ bf16x8 frag_rows16(const char* lds, int rb, int ks, int lane) {
  const int i = lane & 15, gq = lane >> 4;
  const unsigned lane_part = i * (DH * 2) + ((gq ^ swz16(i)) << 4);                     // row i, chunk gq
  const unsigned off = (lane_part ^ (unsigned)(ks << 6)) + (unsigned)(rb * (DH * 2));  // row rb + i, chunk 4 ks + gq
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(lds + off));
}

// First operand = transpose of the tile: output rows are tile columns cb..cb+15 (cb a multiple of
// 16), contraction over tile rows r0 + 4 g + {0..3} and r0 + 16 + 4 g + {0..3} (r0 a multiple of 32).
// A 16-lane block reads four rows x 16 columns; lane i of it addresses row (i >> 2), columns
// 4 (i & 3) .. + 3, and receives column i of all four rows.
template <int DH>
__device__ __forceinline__ bf16x8 frag_cols16(const char* lds, int cb, int r0, int lane) {
  const int blk = lane >> 4, i = lane & 15;
  const int rl = blk * 4 + (i >> 2);    // row within the group of 16
  const int cl = (i & 3) * 4;           // column within the block of 16
  const unsigned lane_part = rl * (DH * 2) + (((cl >> 3) ^ swz16(rl)) << 4) + ((cl >> 2) & 1) * 8;
  const unsigned x = lane_part ^ (unsigned)((cb >> 3) << 4);
  typedef __attribute__((address_space(3))) short4v lds_s4;
  const char* p0 = lds + x + (unsigned)(r0 * (DH * 2));
  const char* p1 = lds + x + (unsigned)((r0 + 16) * (DH * 2));  // 16 rows further down: the swizzle's row bits are the same
  const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)p0);
  const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)p1);
  const short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

template <int DH>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv16_mfma_kernel(int S, int H, int BH, const bf16_t* __restrict__ qkv,
                                                                     const float* __restrict__ lse,
                                                                     const float* __restrict__ delta,
                                                                     const bf16_t* __restrict__ dctx,
                                                                     bf16_t* __restrict__ dqkv) {
  constexpr int KS = DH / 32;   // k-steps of the score products
  constexpr int DT = DH / 16;   // 16-wide d tiles of dK^T, dV^T
  constexpr int TB = TR * DH * 2;
  constexpr int LD_OFF = 2 * TB, STAGE = 2 * TB + 4 * 256;  // Q tile | dO tile | lse and delta (see tile_load)
  constexpr int N = 4 * KS;     // MFMAs per phase and half: {S, dP} x two query groups x KS, or {dV, dK} x DT
  constexpr int LEAD = 8;       // fragments in flight
  constexpr int NSEG = DH / 32;
  static_assert(N == 2 * DT && N % LEAD == 0 && 2 * NSEG + 1 <= N, "slot plan");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int n_kt = S / TR;      // 64-key tiles
  int pair, bh;
  pair_of_tiles(n_kt, BH, pair, bh);
  const int b = bh / H, h = bh % H;
  const int Hd = H * DH;
  const size_t ld = 3 * (size_t)Hd;
  const bf16_t* base = qkv + (size_t)b * S * ld + h * DH;
  const bf16_t* dob = dctx + (size_t)b * S * Hd + h * DH;
  const float* lrow = lse + ((size_t)b * H + h) * S;
  const float* drow = delta + ((size_t)b * H + h) * S;
  const int lane = threadIdx.x & 63, gq = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const float c = rsqrtf((float)DH) * LOG2E;
  const unsigned sm = lds_addr(smem);

  for (int pass = 0; pass < 2; pass++) {
    const int kt = pass == 0 ? pair : n_kt - 1 - pair;
    if (pass == 1 && kt == pair) break;  // odd number of key tiles: the middle one stands alone
    const int jk = kt * TR + wave * 16 + (lane & 15);  // this lane's key
    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      kf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)jk * ld + Hd + ks * 32 + gq * 8));
      vf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)jk * ld + 2 * Hd + ks * 32 + gq * 8));
    }
#pragma unroll
    for (int ks = 0; ks < KS; ks++) { settle(kf[ks]); settle(vf[ks]); }
    f32x4 dk[DT], dv[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int r = 0; r < 4; r++) dk[dt][r] = dv[dt][r] = 0.f;

    const int i_first = kt * TR;           // first query that meets these keys: the tile on the diagonal
    const int n_q = (S - i_first) / TR;
    // Tile of queries i0.. into buffer `buf`, one load instruction per call: this wave's NSEG
    // segments of Q (i < NSEG), of dO (i < 2 NSEG), and its 16 lse and 16 delta values (lanes 0-15
    // lse, 16-31 delta, 32-63 the same again: one 4-byte load instruction moves 64 lanes).
    auto tile_load = [&](int i0, int buf, int i) {
      const unsigned st = sm + buf * STAGE;
      if (i < NSEG) tile_dma_seg16<DH>(st, base + (size_t)i0 * ld, ld, wave, i);
      else if (i < 2 * NSEG) tile_dma_seg16<DH>(st + TB, dob + (size_t)i0 * Hd, (size_t)Hd, wave, i - NSEG);
      else lds_dma4(((lane & 16) ? drow : lrow) + i0 + wave * 16 + (lane & 15), st + LD_OFF + wave * 256);
    };
    bf16x8 f[LEAD];  // one ring for both kinds of fragment: slot i reloads the register it has just used
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    // One 64-query tile, a 32-query half at a time.  MASK: the tile on the diagonal.
    auto tile = [&](auto mask_c, int t) {
      constexpr bool MASK = decltype(mask_c)::value;
      const char* st = smem + (t & 1) * STAGE;
      const int i0n = i_first + min(t + 1, n_q - 1) * TR;  // past the end: the last tile again, into the buffer nobody reads
      // P1 slot i of half it: S (Q rows) or dP (dO rows) by bit 0; query group (i / 2) / KS, k-step (i / 2) % KS
      auto row_frag = [&](int it, int i) {
        return frag_rows16<DH>(i % 2 ? st + TB : st, it * 32 + ((i / 2) / KS) * 16, (i / 2) % KS, lane);
      };
      // P3 slot i of half it: dV (dO^T) or dK (Q^T) by bit 0, d tile i / 2
      auto col_frag = [&](int it, int i) { return frag_cols16<DH>(i % 2 ? st : st + TB, (i / 2) * 16, it * 32, lane); };
      // lse / delta of the queries 32 it + 16 qg + 4 g + 0..3 that this lane meets in the accumulators of query group qg
      auto stat4 = [&](int it, int qg, int which) {
        const int row = it * 32 + qg * 16 + gq * 4;
        return *reinterpret_cast<const float4*>(st + LD_OFF + (row >> 4) * 256 + which * 64 + (row & 15) * 4);
      };
#pragma unroll
      for (int i = 0; i < LEAD; i++) f[i] = row_frag(0, i);  // cold start: exposed once per tile
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int it = 0; it < 2; it++) {
        const int i0h = i_first + t * TR + it * 32;  // first query of the half
        f32x4 sc[2], dp[2];
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int i = 0; i < N; i++) {
          const int qg = (i / 2) / KS, ks = (i / 2) % KS;
          if (i % 2 == 0) sc[qg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[i % LEAD], kf[ks], ks == 0 ? zero : sc[qg], 0, 0, 0);
          else dp[qg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[i % LEAD], vf[ks], ks == 0 ? zero : dp[qg], 0, 0, 0);
          if (i + LEAD < N) f[i % LEAD] = row_frag(it, i + LEAD);
          else f[i % LEAD] = col_frag(it, i + LEAD - N);
          if (it == 0 && i <= 2 * NSEG) tile_load(i0n, (t + 1) & 1, i);
          __builtin_amdgcn_sched_barrier(0);
        }
        bf16x8 pb, db;
        __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int qg = 0; qg < 2; qg++) {
          const float4 l4 = stat4(it, qg, 0), d4 = stat4(it, qg, 1);
#pragma unroll
          for (int r = 0; r < 4; r++) {
            float p = __builtin_amdgcn_exp2f(fmaf(sc[qg][r], c, -LOG2E * f4_get(l4, r)));
            if (MASK && jk > i0h + qg * 16 + gq * 4 + r) p = 0.f;
            const float d = p * (dp[qg][r] - f4_get(d4, r));
            pb[qg * 4 + r] = (__bf16)p;
            db[qg * 4 + r] = (__bf16)d;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int i = 0; i < N; i++) {
          const int dt = i / 2;
          if (i % 2 == 0) dv[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[i % LEAD], pb, dv[dt], 0, 0, 0);
          else dk[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[i % LEAD], db, dk[dt], 0, 0, 0);
          if (i + LEAD < N) f[i % LEAD] = col_frag(it, i + LEAD);
          else if (it == 0) f[i % LEAD] = row_frag(1, i + LEAD - N);  // the second half's first rows
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      __builtin_amdgcn_s_setprio(0);
      lds_dma_wait();
      __syncthreads();
    };

#pragma unroll
    for (int i = 0; i <= 2 * NSEG; i++) tile_load(i_first, 0, i);
    lds_dma_wait();
    __syncthreads();
    tile(T_{}, 0);  // the tile on the diagonal; every later query comes after all of this workgroup's keys
    for (int t = 1; t < n_q; t++) tile(F_{}, t);

    // a lane owns one key row and, per d tile, the four consecutive d's 16 dt + 4 g + 0..3
    const float scale = rsqrtf((float)DH);
    bf16_t* out = dqkv + ((size_t)b * S + jk) * ld + h * DH;
#pragma unroll
    for (int dt = 0; dt < DT; dt++) {
      bf16x4 ok, ov;
#pragma unroll
      for (int r = 0; r < 4; r++) {
        ok[r] = (__bf16)(dk[dt][r] * scale);
        ov[r] = (__bf16)dv[dt][r];
      }
      *reinterpret_cast<bf16x4*>(out + Hd + dt * 16 + gq * 4) = ok;
      *reinterpret_cast<bf16x4*>(out + 2 * Hd + dt * 16 + gq * 4) = ov;
    }
  }  // pass
}

int attn_bwd_dkv16_mfma(int B, int S, int H, const bf16_t* qkv, const float* lse, const float* delta, const bf16_t* dctx,
                        bf16_t* dqkv, hipStream_t s) {
  constexpr int DH = 128;
  constexpr size_t lds_kv = 2 * (2 * (size_t)TR * DH * 2 + 4 * 256);  // two stages of Q tile | dO tile | lse, delta
  FAX_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_dkv16_mfma_kernel<DH>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_kv));
  const int n_kt = S / TR;
  const dim3 grid(((n_kt + 1) / 2) * B * H);
  hipLaunchKernelGGL((attn_bwd_dkv16_mfma_kernel<DH>), grid, dim3(256), lds_kv, s, S, H, B * H, qkv, lse, delta, dctx, dqkv);
  return FAX_OK;
}

}  // namespace fax
