// Causal flash attention on the CDNA4 matrix cores: bf16 operands, fp32 scores and statistics.
//
// All three kernels work on "transposed" MFMA products so that the softmax row of one query
// (forward, dQ) or the column of one key (dK/dV) sits inside one lane plus its partner lane
// (lane ^ 32), and the probabilities come out of the score accumulators already in the
// register layout the next MFMA wants as its B operand: no cross-lane shuffles of P.
//
//   forward   S^T = K Q^T (A = K tile from LDS, B = Q rows held in registers)
//             O^T += V^T P^T (A = V tile through the LDS transpose read, B = P registers)
//   dQ        S^T, dP^T = V dO^T as above, dS^T = P^T (dP^T - delta);  dQ^T += K^T dS^T
//   dK, dV    S = Q K^T, dP = dO V^T (A = Q / dO tile from LDS, B = K / V rows in registers),
//             dV^T += dO^T P,  dK^T += Q^T dS   (A through the transpose read)
//
// 32x32x16 MFMA lane layout (lane l, g = l >> 5): operand element e of row/col (l & 31) is
// k = 8 g + e; accumulator v holds row 8 (v >> 2) + 4 g + (v & 3), column (l & 31).  Taking
// accumulator elements 8 h .. 8 h + 7 as the B operand of step h therefore assigns k-slot
// (g, e) to row 16 h + 8 (e >> 2) + 4 g + (e & 3): two runs of four consecutive rows, which is
// exactly what two ds_read_b64_tr_b16 deliver for the matching A operand.
//
// LDS tiles are [64 rows][DH] bf16 with the 16-byte chunk index XOR-ed by
// f(row) = ((row & 3) << 1) | ((row >> 2) & 1), plus (row & 8) when a row has 16 chunks:
// consecutive rows land in distinct chunks (128-bit row-fragment reads) and 4 consecutive rows in
// 4 distinct 32-byte pairs (transpose reads), so one copy of a tile serves both access patterns.
// Measured on gfx950 with 256-byte rows: row-fragment reads 122 B/clk/CU with the (row & 8) term,
// 102 without; transpose reads 77 B/clk/CU either way (55 unswizzled) -- ds_read_b64_tr_b16 tops
// out at about 60 % of the plain read rate.
//
// No atomics: dQ has one writer per query row, dK/dV one writer per key row; S and dP are
// recomputed in both backward kernels (7 tile products instead of 5).
#include "attn_mfma_common.h"

namespace fax {

// dK, dV at DH = 128: kernels_attn_dkv16.hip (16 keys per wave, its own LDS swizzle)
int attn_bwd_dkv16_mfma(int B, int S, int H, const bf16_t* qkv, const float* lse, const float* delta, const bf16_t* dctx,
                        bf16_t* dqkv, hipStream_t s);

// ---------------------------------------------------------------------------------------------
// Forward.  Wave w owns queries 128 qt + 32 w .. + 31 (B operand, in registers); 64-key tiles of
// K and V stream through two LDS buffers.  Per tile: P1 = S^T for both 32-key halves, V = online
// softmax over the 64 keys, P3 = O^T += V^T P^T.
// ---------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, DH == 64 ? 3 : 2) void attn_fwd_mfma_kernel(int S, int H, int BH, const bf16_t* __restrict__ qkv,
                                                            bf16_t* __restrict__ ctx, float* __restrict__ lse) {
  constexpr int KS = DH / 16, DT = DH / 32, TB = TR * DH * 2;
  constexpr int N = 2 * KS;            // MFMAs per phase (P3: 2 halves x 2 k-steps x DT = 2 KS as well)
  constexpr int LEAD = N < 8 ? N : 8;  // fragments in flight
  constexpr int NSEG = DH / 32;        // 1 KB load instructions per wave per tile
  extern __shared__ __attribute__((aligned(16))) char smem[];  // 2 x [K tile | V tile]
  const int n_qt = S / 128;
  int pair, bh;
  pair_of_tiles(n_qt, BH, pair, bh);
  const int b = bh / H, h = bh % H;
  const int Hd = H * DH;
  const size_t ld = 3 * (size_t)Hd;
  const bf16_t* base = qkv + (size_t)b * S * ld + h * DH;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), g = lane >> 5;
  const float scale = rsqrtf((float)DH);
  const float c = scale * LOG2E;
  const unsigned sm = lds_addr(smem);

  for (int pass = 0; pass < 2; pass++) {
    const int qt = pass == 0 ? n_qt - 1 - pair : pair;  // the long one first
    if (pass == 1 && qt == n_qt - 1 - pair) break;      // odd number of tiles: the middle one stands alone
    const int q0w = qt * 128 + wave * 32, iq = q0w + (lane & 31);
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
      qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)iq * ld + ks * 16 + g * 8));
#pragma unroll
    for (int ks = 0; ks < KS; ks++) settle(qf[ks]);
    float m = -INFINITY, l = 0.f;
    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int v = 0; v < 16; v++) oacc[dt][v] = 0.f;

    const int n_kv = 2 * (qt + 1);
    auto tile_load = [&](int j0, int buf, int i) {
      const unsigned st = sm + buf * 2 * TB;
      if (i < NSEG) tile_dma_seg<DH>(st, base + (size_t)j0 * ld + Hd, ld, wave, i);
      else tile_dma_seg<DH>(st + TB, base + (size_t)j0 * ld + 2 * Hd, ld, wave, i - NSEG);
    };
    bf16x8 fr[LEAD], fc[LEAD];
    // One 64-key tile.  MASK: the tile may reach past the wave's first query.
    auto tile = [&](auto mask_c, int t) {
      constexpr bool MASK = decltype(mask_c)::value;
      const char* kt_ = smem + (t & 1) * 2 * TB;
      const char* vt_ = kt_ + TB;
      const int j0 = t * TR;
      const int j0n = min(t + 1, n_kv - 1) * TR;  // past the end: the last tile again, into the buffer nobody reads
      auto row_frag = [&](int i) { return frag_rows<DH>(kt_, (i % 2) * 32, i / 2, lane); };
      // P3 slot i: d-tile dt = i % DT (so that MFMAs on the same accumulator are DT slots apart),
      // then key half jt and k-step hh from i / DT
      auto col_frag = [&](int i) {
        return frag_cols<DH>(vt_, (i % DT) * 32, ((i / DT) % 2) * 32 + ((i / DT) / 2) * 16, lane);
      };
#pragma unroll
      for (int i = 0; i < LEAD; i++) fr[i] = row_frag(i);  // cold start: exposed once per tile
      f32x16 s[2];
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int v = 0; v < 16; v++) s[jt][v] = 0.f;
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(1);
#pragma unroll
      for (int i = 0; i < N; i++) {
        s[i % 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % LEAD], qf[i / 2], s[i % 2], 0, 0, 0);
        if (i + LEAD < N) fr[i % LEAD] = row_frag(i + LEAD);
        else fc[i + LEAD - N] = col_frag(i + LEAD - N);
        if (i < 2 * NSEG) tile_load(j0n, (t + 1) & 1, i);
        __builtin_amdgcn_sched_barrier(0);
      }
      __builtin_amdgcn_s_setprio(0);
      // Scores stay unscaled; the softmax scale rides in the exponent: p = 2^(c s - c m), c = scale log2 e.
      if (MASK) {
#pragma unroll
        for (int jt = 0; jt < 2; jt++)
#pragma unroll
          for (int v = 0; v < 16; v++) {
            const int key = j0 + jt * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
            if (key > iq) s[jt][v] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int v = 0; v < 16; v++) mx = fmaxf(mx, s[jt][v]);
      mx = max32(mx);
      // The reference point of the exponentials, m, follows the running maximum lazily: it moves
      // (and the accumulators are rescaled) only when some query's maximum has risen more than
      // MAX_LAG octaves above it, which after the first few tiles is rare.  Probabilities are then
      // at most 2^MAX_LAG instead of 1; numerator, denominator and lse all use the same m, so
      // the result is the same softmax.
      const float mn = fmaxf(m, mx);  // finite: key 0 is visible to every query and comes in the first tile
      if (__builtin_amdgcn_ballot_w64((mn - m) * c > MAX_LAG) != 0) {
        const float corr = __builtin_amdgcn_exp2f((m - mn) * c);
        l *= corr;
#pragma unroll
        for (int dt = 0; dt < DT; dt++)
#pragma unroll
          for (int v = 0; v < 16; v++) oacc[dt][v] *= corr;
        m = mn;
      }
      const float mc = m * c;
      float rs = 0.f;
      bf16x8 pb[2][2];
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[jt][v], c, -mc));
          rs += p;
          pb[jt][v >> 3][v & 7] = (__bf16)p;
        }
      rs = sum32(rs);
      l += rs;
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(1);
#pragma unroll
      for (int i = 0; i < N; i++) {
        const int dt = i % DT;
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fc[i % LEAD], pb[(i / DT) % 2][(i / DT) / 2], oacc[dt], 0, 0, 0);
        if (i + LEAD < N) fc[i % LEAD] = col_frag(i + LEAD);
        __builtin_amdgcn_sched_barrier(0);
      }
      __builtin_amdgcn_s_setprio(0);
      lds_dma_wait();
      __syncthreads();
    };

#pragma unroll
    for (int i = 0; i < 2 * NSEG; i++) tile_load(0, 0, i);
    lds_dma_wait();
    __syncthreads();
    for (int t = 0; t < n_kv - 2; t++) tile(F_{}, t);
    tile(T_{}, n_kv - 2);  // the last two tiles (128 keys) straddle the diagonal of this workgroup's 128 queries
    tile(T_{}, n_kv - 1);

    store_rows<DH>(ctx + ((size_t)b * S + iq) * Hd + h * DH, oacc, 1.f / l, g);
    if (g == 0) lse[((size_t)b * H + h) * S + iq] = m * scale + logf(l);
  }  // pass
}

// ---------------------------------------------------------------------------------------------
// dQ (and delta).  Wave w owns queries 128 qt + 32 w .. + 31 (Q and dO rows in registers as B
// operands); 64-key tiles of K and V stream through two LDS buffers.  One 32-key half after the
// other:
//   P1: S^T = K Q^T and dP^T = V dO^T, alternating (row fragments of K and V, 2 KS MFMAs)
//   V:  dS^T = P^T (dP^T - delta), P^T = 2^(c S^T - lse log2 e), packed to bf16
//   P3: dQ^T += K^T dS^T (transpose-read fragments of K)
// One barrier per 64-key tile.  Registers budgeted for two waves per SIMD, LDS for two workgroups
// per CU (see above).
// ---------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_mfma_kernel(int S, int H, int BH, const bf16_t* __restrict__ qkv,
                                                                         const float* __restrict__ lse,
                                                                         const bf16_t* __restrict__ ctx,
                                                                         const bf16_t* __restrict__ dctx,
                                                                         float* __restrict__ delta,
                                                                         bf16_t* __restrict__ dqkv) {
  constexpr int KS = DH / 16, DT = DH / 32, TB = TR * DH * 2;
  constexpr int N1 = 2 * KS;   // score MFMAs per 32-key half: S and dP, KS each
  constexpr int N3 = 2 * DT;   // dQ MFMAs per half: two k-steps x DT
  constexpr int LEAD = N3;     // fragments in flight
  constexpr int NSEG = DH / 32;
  static_assert(2 * NSEG <= N1 && N1 % LEAD == 0, "slot plan");
  extern __shared__ __attribute__((aligned(16))) char smem[];  // 2 x [K tile | V tile]
  const int n_qt = S / 128;
  int pair, bh;
  pair_of_tiles(n_qt, BH, pair, bh);
  const int b = bh / H, h = bh % H;
  const int Hd = H * DH;
  const size_t ld = 3 * (size_t)Hd;
  const bf16_t* base = qkv + (size_t)b * S * ld + h * DH;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), g = lane >> 5;
  const float scale = rsqrtf((float)DH);
  const float c = scale * LOG2E;
  const unsigned sm = lds_addr(smem);

  for (int pass = 0; pass < 2; pass++) {
    const int qt = pass == 0 ? n_qt - 1 - pair : pair;
    if (pass == 1 && qt == n_qt - 1 - pair) break;
    const int q0w = qt * 128 + wave * 32, iq = q0w + (lane & 31);
    bf16x8 qf[KS], dof[KS];
    const bf16_t* dorow = dctx + ((size_t)b * S + iq) * Hd + h * DH;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)iq * ld + ks * 16 + g * 8));
      dof[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(dorow + ks * 16 + g * 8));
    }
    float li = lse[((size_t)b * H + h) * S + iq] * LOG2E;
    float di = 0.f;  // delta_i = sum_d dO[i, d] O[i, d], half of the row per lane
    const bf16_t* orow = ctx + ((size_t)b * S + iq) * Hd + h * DH;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      const bf16x8 o = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(orow + ks * 16 + g * 8));
#pragma unroll
      for (int e = 0; e < 8; e++) di = fmaf((float)o[e], (float)dof[ks][e], di);
    }
    di = sum32(di);
    if (g == 0) delta[((size_t)b * H + h) * S + iq] = di;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) { settle(qf[ks]); settle(dof[ks]); }
    settle(li); settle(di);
    f32x16 dq[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int v = 0; v < 16; v++) dq[dt][v] = 0.f;

    const int n_kv = 2 * (qt + 1);
    auto tile_load = [&](int j0, int buf, int i) {
      const unsigned st = sm + buf * 2 * TB;
      if (i < NSEG) tile_dma_seg<DH>(st, base + (size_t)j0 * ld + Hd, ld, wave, i);
      else tile_dma_seg<DH>(st + TB, base + (size_t)j0 * ld + 2 * Hd, ld, wave, i - NSEG);
    };
    bf16x8 f[LEAD];  // one ring for both kinds of fragment: slot i reloads the register it has just used
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // One 64-key tile, a 32-key half at a time.  MASK: the tile may reach past the wave's first query.
    auto tile = [&](auto mask_c, int t) {
      constexpr bool MASK = decltype(mask_c)::value;
      const char* kt_ = smem + (t & 1) * 2 * TB;
      const char* vt_ = kt_ + TB;
      const int j0n = min(t + 1, n_kv - 1) * TR;  // past the end: the last tile again, into the buffer nobody reads
      // P1 slot i of half jt: S (K rows x Q) or dP (V rows x dO) by bit 0, k-step i / 2
      auto row_frag = [&](int jt, int i) { return frag_rows<DH>((i & 1) ? vt_ : kt_, jt * 32, i / 2, lane); };
      // P3 slot i of half jt: d-tile i % DT, k-step i / DT
      auto col_frag = [&](int jt, int i) { return frag_cols<DH>(kt_, (i % DT) * 32, jt * 32 + (i / DT) * 16, lane); };
#pragma unroll
      for (int i = 0; i < LEAD; i++) f[i] = row_frag(0, i);  // cold start: exposed once per tile
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int jt = 0; jt < 2; jt++) {
        f32x16 sc, dp;
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int i = 0; i < N1; i++) {
          const int ks = i / 2;
          if (i & 1) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % LEAD], dof[ks], i < 2 ? zero : dp, 0, 0, 0);
          else sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % LEAD], qf[ks], i < 2 ? zero : sc, 0, 0, 0);
          if (i + LEAD < N1) f[i % LEAD] = row_frag(jt, i + LEAD);
          else f[i % LEAD] = col_frag(jt, i + LEAD - N1);  // (N1 is a multiple of LEAD)
          if (jt == 0 && i < 2 * NSEG) tile_load(j0n, (t + 1) & 1, i);
          __builtin_amdgcn_sched_barrier(0);
        }
        bf16x8 db[2];
        __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int v = 0; v < 16; v++) {
          float p = __builtin_amdgcn_exp2f(fmaf(sc[v], c, -li));
          if (MASK && t * TR + jt * 32 + (v >> 2) * 8 + g * 4 + (v & 3) > iq) p = 0.f;
          db[v >> 3][v & 7] = (__bf16)(p * (dp[v] - di));
        }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int i = 0; i < N3; i++) {
          dq[i % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % LEAD], db[i / DT], dq[i % DT], 0, 0, 0);
          if (jt == 0) f[i % LEAD] = row_frag(1, i);  // the second half's first rows (N3 = LEAD)
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      __builtin_amdgcn_s_setprio(0);
      lds_dma_wait();
      __syncthreads();
    };

#pragma unroll
    for (int i = 0; i < 2 * NSEG; i++) tile_load(0, 0, i);
    lds_dma_wait();
    __syncthreads();
    for (int t = 0; t < n_kv - 2; t++) tile(F_{}, t);
    tile(T_{}, n_kv - 2);  // the last two tiles (128 keys) straddle the diagonal of this workgroup's 128 queries
    tile(T_{}, n_kv - 1);

    store_rows<DH>(dqkv + ((size_t)b * S + iq) * ld + h * DH, dq, scale, g);
  }  // pass
}

// ---------------------------------------------------------------------------------------------
// dK, dV without the skew (used for DH = 64, where the kernel then fits the register budget of
// two waves per SIMD and several workgroups share a CU).  The same arithmetic as the kernel above,
// a 32-query half at a time: P1 = S and dP (2 KS MFMAs), V = P and dS packed to bf16, P3 = dV^T and
// dK^T (2 KS MFMAs); two LDS buffers, one barrier per 64-query tile.
// ---------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_phased_mfma_kernel(int S, int H, int BH, const bf16_t* __restrict__ qkv,
                                                                          const float* __restrict__ lse,
                                                                          const float* __restrict__ delta,
                                                                          const bf16_t* __restrict__ dctx,
                                                                          bf16_t* __restrict__ dqkv) {
  constexpr int KS = DH / 16, DT = DH / 32, TB = TR * DH * 2;
  constexpr int LD_OFF = 2 * TB, STAGE = 2 * TB + 4 * 256;  // Q tile | dO tile | lse and delta as above
  constexpr int N = 2 * KS;                   // MFMAs per phase and half
  constexpr int LEAD = N < 8 ? N : 8;         // fragments in flight
  constexpr int NSEG = DH / 32;
  static_assert(N % LEAD == 0 && 2 * NSEG + 1 <= N, "slot plan");
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
    const int n_q = (S - i_first) / TR;
    auto tile_load = [&](int i0, int buf, int i) {
      const unsigned st = sm + buf * STAGE;
      if (i < NSEG) tile_dma_seg<DH>(st, base + (size_t)i0 * ld, ld, wave, i);
      else if (i < 2 * NSEG) tile_dma_seg<DH>(st + TB, dob + (size_t)i0 * Hd, (size_t)Hd, wave, i - NSEG);
      else lds_dma4(((lane & 16) ? drow : lrow) + i0 + wave * 16 + (lane & 15), st + LD_OFF + wave * 256);
    };
    bf16x8 f[LEAD];  // one ring for both kinds of fragment: slot i reloads the register it has just used
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // One 64-query tile, a 32-query half at a time.  MASK: the tile may reach back before the wave's last key.
    auto tile = [&](auto mask_c, int t) {
      constexpr bool MASK = decltype(mask_c)::value;
      const char* st = smem + (t & 1) * STAGE;
      const int i0n = i_first + min(t + 1, n_q - 1) * TR;  // past the end: the last tile again, into the buffer nobody reads
      // P1 slot i of half it: S (Q rows x K) or dP (dO rows x V) by bit 0, k-step i / 2
      auto row_frag = [&](int it, int i) { return frag_rows<DH>(i % 2 ? st + TB : st, it * 32, i / 2, lane); };
      // P3 slot i: dV (dO^T) or dK (Q^T) by bit 0, d-tile (i / 2) % DT, k-step i / (2 DT)
      auto col_frag = [&](int it, int i) {
        return frag_cols<DH>(i % 2 ? st : st + TB, ((i / 2) % DT) * 32, it * 32 + (i / (2 * DT)) * 16, lane);
      };
      // lse / delta of the rows 32 it + 8 q + 4 g + 0..3 that this lane meets in accumulator group q
      auto stat4 = [&](int it, int q, int which) {
        const int row = it * 32 + q * 8 + g * 4;
        return *reinterpret_cast<const float4*>(st + LD_OFF + (row >> 4) * 256 + which * 64 + (row & 15) * 4);
      };
#pragma unroll
      for (int i = 0; i < LEAD; i++) f[i] = row_frag(0, i);  // cold start: exposed once per tile
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int it = 0; it < 2; it++) {
        const int i0h = i_first + t * TR + it * 32;  // first query of the half
        f32x16 sc, dp;
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int i = 0; i < N; i++) {
          if (i % 2 == 0) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % LEAD], kf[i / 2], i < 2 ? zero : sc, 0, 0, 0);
          else dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % LEAD], vf[i / 2], i < 2 ? zero : dp, 0, 0, 0);
          if (i + LEAD < N) f[i % LEAD] = row_frag(it, i + LEAD);
          else f[i % LEAD] = col_frag(it, i + LEAD - N);
          if (it == 0 && i <= 2 * NSEG) tile_load(i0n, (t + 1) & 1, i);
          __builtin_amdgcn_sched_barrier(0);
        }
        bf16x8 pb[2], db[2];
        __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const float4 l4 = stat4(it, q, 0), d4 = stat4(it, q, 1);
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const int v = q * 4 + r;
            float p = __builtin_amdgcn_exp2f(fmaf(sc[v], c, -LOG2E * f4_get(l4, r)));
            if (MASK && jk > i0h + q * 8 + g * 4 + r) p = 0.f;
            const float d = p * (dp[v] - f4_get(d4, r));
            pb[v >> 3][v & 7] = (__bf16)p;
            db[v >> 3][v & 7] = (__bf16)d;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int i = 0; i < N; i++) {
          const int hh = i / (2 * DT), dt = (i / 2) % DT;
          if (i % 2 == 0) dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % LEAD], pb[hh], dv[dt], 0, 0, 0);
          else dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i % LEAD], db[hh], dk[dt], 0, 0, 0);
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
    tile(T_{}, 0);  // the first two tiles (128 queries) straddle the diagonal of this workgroup's 128 keys
    tile(T_{}, 1);
    for (int t = 2; t < n_q; t++) tile(F_{}, t);

    const float scale = rsqrtf((float)DH);
    bf16_t* out = dqkv + ((size_t)b * S + jk) * ld + h * DH;
    store_rows<DH>(out + Hd, dk, scale, g);
    store_rows<DH>(out + 2 * Hd, dv, 1.f, g);
  }  // pass
}

bool attn_mfma_supported(int dtype, int B, int S, int H, int dh) {
  (void)B; (void)H;
  return dtype == FAX_BF16 && (dh == 64 || dh == 128) && S > 0 && S % 128 == 0;
}

template <typename K>
static int set_lds(K kern, size_t bytes) {
  FAX_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return FAX_OK;
}

template <int DH>
static int fwd_t(int B, int S, int H, const bf16_t* qkv, bf16_t* ctx, float* lse, hipStream_t s) {
  constexpr size_t lds = 2 * (2 * (size_t)TR * DH * 2);  // two stages of K tile | V tile
  FAX_TRY(set_lds(attn_fwd_mfma_kernel<DH>, lds));
  hipLaunchKernelGGL((attn_fwd_mfma_kernel<DH>), dim3(((S / 128 + 1) / 2) * B * H), dim3(256), lds, s, S, H, B * H, qkv, ctx,
                     lse);
  FAX_LAUNCH_CHECK("attn_fwd_mfma");
  return FAX_OK;
}

int attn_fwd_mfma(int B, int S, int H, int dh, const void* qkv, void* ctx, float* lse, hipStream_t s) {
  if (dh == 64) return fwd_t<64>(B, S, H, (const bf16_t*)qkv, (bf16_t*)ctx, lse, s);
  return fwd_t<128>(B, S, H, (const bf16_t*)qkv, (bf16_t*)ctx, lse, s);
}

template <int DH>
static int bwd_t(int B, int S, int H, const bf16_t* qkv, const bf16_t* ctx, const float* lse, const bf16_t* dctx,
                 bf16_t* dqkv, float* delta, hipStream_t s, const AttnBwdSplit* split) {
  constexpr size_t lds_q = 2 * (2 * (size_t)TR * DH * 2);  // two stages of K tile | V tile
  const dim3 grid(((S / 128 + 1) / 2) * B * H);
  FAX_TRY(set_lds(attn_bwd_dq_mfma_kernel<DH>, lds_q));
  auto dkv = [&](hipStream_t st) -> int {
    if constexpr (DH == 64) {
      constexpr size_t lds_kv = 2 * (2 * (size_t)TR * DH * 2 + 4 * 256);  // two stages of Q tile | dO tile | lse, delta
      FAX_TRY(set_lds(attn_bwd_dkv_phased_mfma_kernel<DH>, lds_kv));
      hipLaunchKernelGGL((attn_bwd_dkv_phased_mfma_kernel<DH>), grid, dim3(256), lds_kv, st, S, H, B * H, qkv, lse, delta, dctx,
                         dqkv);
    } else {
      FAX_TRY(attn_bwd_dkv16_mfma(B, S, H, qkv, lse, delta, dctx, dqkv, st));
    }
    return FAX_OK;
  };
  // Few workgroups (a tensor-parallel share at batch 1: 40 to 128 of them on 256 CUs): the dQ and the
  // dK/dV kernel fit on the chip side by side.  What ties them together is delta, which the dQ
  // kernel produces as it goes; a small kernel of its own computes it first, the dQ kernel writes
  // its copy to scratch, and with a second stream the two kernels run at the same time.  Whether
  // this form is used depends on the shape only, so that one or two streams give the same bits.
  if (split && split->delta_scratch && attn_bwd_side_by_side(B, S, H)) {
    FAX_TRY(attn_delta(FAX_BF16, B, S, H, DH, ctx, dctx, delta, s));
    const bool two = split->side && split->fork && split->join;
    if (two) {
      FAX_HIP(hipEventRecord(split->fork, s));
      FAX_HIP(hipStreamWaitEvent(split->side, split->fork, 0));
      FAX_TRY(dkv(split->side));
      FAX_HIP(hipEventRecord(split->join, split->side));
    }
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<DH>), grid, dim3(256), lds_q, s, S, H, B * H, qkv, lse, ctx, dctx,
                       split->delta_scratch, dqkv);
    if (two) FAX_HIP(hipStreamWaitEvent(s, split->join, 0));
    else FAX_TRY(dkv(s));
    FAX_LAUNCH_CHECK("attn_bwd_mfma");
    return FAX_OK;
  }
  // dQ first: it also produces delta, which the dK/dV kernel reads
  hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<DH>), grid, dim3(256), lds_q, s, S, H, B * H, qkv, lse, ctx, dctx, delta, dqkv);
  FAX_TRY(dkv(s));
  FAX_LAUNCH_CHECK("attn_bwd_mfma");
  return FAX_OK;
}

// dK/dV runs one workgroup per CU, dQ two: side by side they need 1.5 CUs per pair of row tiles.
bool attn_bwd_side_by_side(int B, int S, int H) {
  const long long n = (long long)((S / 128 + 1) / 2) * B * H;
  return 3 * n <= 2 * 256;
}

int attn_bwd_mfma(int B, int S, int H, int dh, const void* qkv, const void* ctx, const float* lse, const void* dctx,
                  void* dqkv, float* delta, hipStream_t s, const AttnBwdSplit* split) {
  if (dh == 64)
    return bwd_t<64>(B, S, H, (const bf16_t*)qkv, (const bf16_t*)ctx, lse, (const bf16_t*)dctx, (bf16_t*)dqkv, delta, s, split);
  return bwd_t<128>(B, S, H, (const bf16_t*)qkv, (const bf16_t*)ctx, lse, (const bf16_t*)dctx, (bf16_t*)dqkv, delta, s, split);
}

}  // namespace fax
