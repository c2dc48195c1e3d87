// dK, dV of the causal flash attention at head width 128 (see attn_mfma_common.h for the layouts and
// kernels_attn_mfma.hip for the other kernels).  A file of its own because of how it is compiled:
// this kernel runs one wave per SIMD with all 512 registers, its 128 accumulator registers in
// AGPRs, where the matrix core reads and writes them in place; the other attention kernels share a
// SIMD between two or three waves and are built with MFMA results forced into ordinary registers,
// an option that here makes the compiler shuffle values between the two register files (+27 %
// vector instructions).
#include "attn_mfma_common.h"

namespace fax {

// ---------------------------------------------------------------------------------------------
// dK, dV (used for DH = 128).  Wave w owns keys 128 kt + 32 w .. + 31, held in registers as the B operands; 64-query
// tiles of Q and dO (plus their lse and delta) stream through three LDS buffers, starting at the
// diagonal.  Per 32-query half u:
//   S(u) = Q K^T and dP(u) = dO V^T, alternating (row fragments of Q and dO)
//   V(u): P = 2^(c S - lse log2 e), dS = P (dP - delta), both packed to bf16
//   P3(u): dV^T += dO^T P and dK^T += Q^T dS, alternating (transpose-read fragments)
// The vector work is about as long as one of the MFMA phases, so it is hidden behind the score
// MFMAs of the *next* half: the loop body is
//   C(u)  = slot by slot: one MFMA of S/dP(u+1), one fragment read, one element of V(u)
//   P3(u) = slot by slot: one MFMA of dV/dK(u), one fragment read (the tile loads ride here too)
// with two sets of score accumulators taking turns.  Past the last half the "next" scores are
// computed from the last half again and dropped, which keeps the loop body free of special cases.
// One barrier per tile, before P3 of the tile's first half: it publishes the next tile (first
// needed by the row prefetch at the end of that P3) and frees the buffer of the previous one,
// into which the tile after next is then requested.
// ---------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma_kernel(int S, int H, int BH, const bf16_t* __restrict__ qkv,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ delta,
                                                                const bf16_t* __restrict__ dctx,
                                                                bf16_t* __restrict__ dqkv) {
  constexpr int KS = DH / 16, DT = DH / 32, TB = TR * DH * 2;
  // Q tile | dO tile | per wave w: lse[16 w .. +15], delta[16 w .. +15], and a copy of both (the
  // 64 lanes of one 4-byte load instruction: 32 useful values, fetched twice)
  constexpr int LD_OFF = 2 * TB, STAGE = 2 * TB + 4 * 256, NBUF = 3;
  constexpr int N = 2 * KS;                   // MFMAs per phase
  constexpr int LEAD = N < 8 ? N : 8;         // fragments in flight
  constexpr int NSEG = DH / 32;               // 1 KB load instructions per wave per tile and operand
  constexpr int EPS = 16 / N;                 // score elements per slot of C
  static_assert(16 % N == 0 && 2 * NSEG + 1 <= N && 8 <= N, "slot plan");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int n_kt = S / 128;
  int pair, bh;
  pair_of_tiles(n_kt, BH, pair, bh);
  const int b = bh / H, h = bh % H;
  const int Hd = H * DH;
  const size_t ld = 3 * (size_t)Hd;
  const bf16_t* base = qkv + (size_t)b * S * ld + h * DH;
  const bf16_t* dob = dctx + (size_t)b * S * Hd + h * DH;
  const float* lrow = lse + ((size_t)b * H + h) * S;
  const float* drow = delta + ((size_t)b * H + h) * S;
  const int lane = threadIdx.x & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const float c = rsqrtf((float)DH) * LOG2E;
  const unsigned sm = lds_addr(smem);

  for (int pass = 0; pass < 2; pass++) {
    const int kt = pass == 0 ? pair : n_kt - 1 - pair;
    if (pass == 1 && kt == pair) break;  // odd number of key tiles: the middle one stands alone
    const int j0w = kt * 128 + wave * 32, jk = j0w + (lane & 31);
    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      kf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)jk * ld + Hd + ks * 16 + g * 8));
      vf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)jk * ld + 2 * Hd + ks * 16 + g * 8));
    }
#pragma unroll
    for (int ks = 0; ks < KS; ks++) { settle(kf[ks]); settle(vf[ks]); }
    f32x16 dk[DT], dv[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int v = 0; v < 16; v++) dk[dt][v] = dv[dt][v] = 0.f;

    const int i_first = kt * 128;
    const int n_q = (S - i_first) / TR, n_half = 2 * n_q;
    // Tile of queries i0.. into buffer `buf`, one load instruction per call: this wave's NSEG
    // segments of Q (i < NSEG), of dO (i < 2 NSEG), and its 16 lse and 16 delta values.
    auto tile_load = [&](int i0, int buf, int i) {
      const unsigned st = sm + buf * STAGE;
      if (i < NSEG) tile_dma_seg<DH>(st, base + (size_t)i0 * ld, ld, wave, i);
      else if (i < 2 * NSEG) tile_dma_seg<DH>(st + TB, dob + (size_t)i0 * Hd, (size_t)Hd, wave, i - NSEG);
      else lds_dma4(((lane & 16) ? drow : lrow) + i0 + wave * 16 + (lane & 15), st + LD_OFF + wave * 256);
    };
    auto stage = [&](int t) { return smem + (min(t, n_q - 1) % NBUF) * STAGE; };  // past the end: the last tile again
    auto row_frag = [&](const char* st, int it, int i) { return frag_rows<DH>(i % 2 ? st + TB : st, it * 32, i / 2, lane); };
    auto col_frag = [&](const char* st, int it, int i) {
      return frag_cols<DH>(i % 2 ? st : st + TB, ((i / 2) % DT) * 32, it * 32 + (i / (2 * DT)) * 16, lane);
    };
    // lse / delta of the rows 32 it + 8 q + 4 g + 0..3 that this lane meets in accumulator group q
    auto stat4 = [&](const char* st, int it, int q, int which) {
      const int row = it * 32 + q * 8 + g * 4;
      return *reinterpret_cast<const float4*>(st + LD_OFF + (row >> 4) * 256 + which * 64 + (row & 15) * 4);
    };

    bf16x8 fr[LEAD], fc[LEAD];
    f32x16 sc[2], dp[2];  // [u & 1]: scores of half u
    float4 l4[4], d4[4];
    bf16x8 pb[2], db[2];
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    // MFMA i of S/dP for the half whose row fragments are in flight, into score set `par`
    auto score_mfma = [&](int par, int i) {
      if (i % 2 == 0) sc[par] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % LEAD], kf[i / 2], i < 2 ? zero : sc[par], 0, 0, 0);
      else dp[par] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % LEAD], vf[i / 2], i < 2 ? zero : dp[par], 0, 0, 0);
    };
    // Half u (it = u & 1 fixed at compile time): C(u), [barrier], P3(u).
    auto step = [&](auto mask_c, auto it_c, int u) {
      constexpr bool MASK = decltype(mask_c)::value;
      constexpr int IT = decltype(it_c)::value;
      const int t = u >> 1;
      const char* st = stage(t);                    // tile of half u
      const char* st1 = stage((u + 1) >> 1);        // ... of half u + 1
      const char* st2 = stage(t + 1);               // ... of half u + 2
      const int i0h = i_first + t * TR + IT * 32;   // first query of half u
#pragma unroll
      for (int i = 0; i < N; i++) {
        score_mfma(IT ^ 1, i);
        if (i + LEAD < N) fr[i % LEAD] = row_frag(st1, IT ^ 1, i + LEAD);
        else fc[i + LEAD - N] = col_frag(st, IT, i + LEAD - N);
#pragma unroll
        for (int e = 0; e < EPS; e++) {
          const int v = i * EPS + e, q = v >> 2, r = v & 3;
          float p = __builtin_amdgcn_exp2f(fmaf(sc[IT][v], c, -LOG2E * f4_get(l4[q], r)));
          if (MASK && jk > i0h + q * 8 + g * 4 + r) p = 0.f;
          const float d = p * (dp[IT][v] - f4_get(d4[q], r));
          pb[v >> 3][v & 7] = (__bf16)p;
          db[v >> 3][v & 7] = (__bf16)d;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (IT == 0) {
        // every load issued so far (the newest: tile t + 1) has landed; all waves are past P3 of
        // half u - 1, the last reader of tile t - 1
        lds_dma_wait();
        __syncthreads();
      }
      const int i0n = i_first + min(t + 2, n_q - 1) * TR;
#pragma unroll
      for (int i = 0; i < N; i++) {
        const int hh = i / (2 * DT), dt = (i / 2) % DT;
        if (i % 2 == 0) dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fc[i % LEAD], pb[hh], dv[dt], 0, 0, 0);
        else dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fc[i % LEAD], db[hh], dk[dt], 0, 0, 0);
        if (i + LEAD < N) fc[i % LEAD] = col_frag(st, IT, i + LEAD);
        else fr[i + LEAD - N] = row_frag(st2, IT, i + LEAD - N);
        if (i < 8) {  // statistics of half u + 1, for the next C
          if (i < 4) l4[i] = stat4(st1, IT ^ 1, i, 0);
          else d4[i - 4] = stat4(st1, IT ^ 1, i - 4, 1);
        }
        if (IT == 0 && i <= 2 * NSEG) tile_load(i0n, (t + 2) % NBUF, i);
        __builtin_amdgcn_sched_barrier(0);
      }
    };

#pragma unroll
    for (int i = 0; i <= 2 * NSEG; i++) tile_load(i_first, 0, i);
#pragma unroll
    for (int i = 0; i <= 2 * NSEG; i++) tile_load(i_first + TR, 1, i);
    lds_dma_wait();
    __syncthreads();
    // scores of half 0, cold: fragment reads exposed once per pass
    {
      const char* st = stage(0);
#pragma unroll
      for (int i = 0; i < LEAD; i++) fr[i] = row_frag(st, 0, i);
#pragma unroll
      for (int q = 0; q < 4; q++) { l4[q] = stat4(st, 0, q, 0); d4[q] = stat4(st, 0, q, 1); }
#pragma unroll
      for (int i = 0; i < N; i++) {
        score_mfma(0, i);
        if (i + LEAD < N) fr[i % LEAD] = row_frag(st, 0, i + LEAD);
        else fr[i + LEAD - N] = row_frag(st, 1, i + LEAD - N);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // the first two tiles (four halves) straddle the diagonal of this workgroup's 128 keys
    step(T_{}, I<0>{}, 0);
    step(T_{}, I<1>{}, 1);
    step(T_{}, I<0>{}, 2);
    step(T_{}, I<1>{}, 3);
    for (int u = 4; u < n_half; u += 2) {
      step(F_{}, I<0>{}, u);
      step(F_{}, I<1>{}, u + 1);
    }
    lds_dma_wait();   // the re-requested last tile
    __syncthreads();  // LDS is reused by the next pass

    const float scale = rsqrtf((float)DH);
    bf16_t* out = dqkv + ((size_t)b * S + jk) * ld + h * DH;
    store_rows<DH>(out + Hd, dk, scale, g);
    store_rows<DH>(out + 2 * Hd, dv, 1.f, g);
  }  // pass
}

int attn_bwd_dkv128_mfma(int B, int S, int H, const bf16_t* qkv, const float* lse, const float* delta, const bf16_t* dctx,
                         bf16_t* dqkv, hipStream_t s) {
  constexpr int DH = 128;
  constexpr size_t lds_kv = 3 * (2 * (size_t)TR * DH * 2 + 4 * 256);  // three stages of Q tile | dO tile | lse, delta
  FAX_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_dkv_mfma_kernel<DH>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_kv));
  const dim3 grid(((S / 128 + 1) / 2) * B * H);
  hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<DH>), grid, dim3(256), lds_kv, s, S, H, B * H, qkv, lse, delta, dctx, dqkv);
  return FAX_OK;
}

}  // namespace fax
