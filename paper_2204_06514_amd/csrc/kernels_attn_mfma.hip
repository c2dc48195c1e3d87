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
// f(row) = ((row & 3) << 1) | ((row >> 2) & 1): 8 consecutive rows land in 8 distinct chunks
// (128-bit row-fragment reads) and 4 consecutive rows in 4 distinct 32-byte pairs (transpose
// reads), so one copy of a tile serves both access patterns.
//
// No atomics: dQ has one writer per query row, dK/dV one writer per key row; S and dP are
// recomputed in both backward kernels (7 tile products instead of 5).
#include "fax_internal.h"

namespace fax {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static constexpr float LOG2E = 1.4426950408889634f;
static constexpr int TR = 64;  // rows per LDS tile

__device__ __forceinline__ int swz(int row) { return ((row & 3) << 1) | ((row >> 2) & 1); }

template <int DH>
__device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * (DH * 2) + ((chunk ^ swz(row)) << 4);
}

// A 64 x DH tile moved global -> LDS directly (global_load_lds_dwordx4: no staging registers, no
// LDS store instructions).  One wave instruction fills 1024 consecutive LDS bytes, lane i at
// +16 i, so the swizzle is applied on the global side: the lane that owns physical chunk p of
// row r fetches logical chunk p ^ f(r).  lds_dma_wait() must precede the barrier that publishes
// the tile.
template <int DH>
__device__ __forceinline__ void tile_dma(unsigned lds, const bf16_t* __restrict__ src, size_t ld) {
  constexpr int NCH = DH / 8;         // 16-byte chunks per row
  constexpr int RPI = 64 / NCH;       // rows per wave instruction
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < DH / 32; i++) {
    const int seg = wave * (DH / 32) + i;  // which 1 KB segment of the tile
    const int row = seg * RPI + lane / NCH;
    const int chunk = (lane % NCH) ^ swz(row);
    lds_dma16(src + (size_t)row * ld + chunk * 8, lds + seg * 1024u);
  }
}

// A operand, rows rb..rb+31 of the tile, contraction over the tile's columns (k-step ks).
template <int DH>
__device__ __forceinline__ bf16x8 frag_rows(const char* lds, int rb, int ks, int lane) {
  const int row = rb + (lane & 31);
  const uint4 v = *reinterpret_cast<const uint4*>(lds + tile_off<DH>(row, ks * 2 + (lane >> 5)));
  return __builtin_bit_cast(bf16x8, v);
}

// A operand = transpose of the tile: output rows are tile columns cb..cb+31, contraction over
// tile rows r0 + {0..3, 8..11} + 4 g (the k-slot order described in the header).
template <int DH>
__device__ __forceinline__ bf16x8 frag_cols(const char* lds, int cb, int r0, int lane) {
  const int blk = lane >> 4, i = lane & 15;
  const int row = r0 + (blk >> 1) * 4 + (i >> 2);
  const int col = cb + (blk & 1) * 16 + (i & 3) * 4;
  typedef __attribute__((address_space(3))) short4v lds_s4;
  const char* p0 = lds + tile_off<DH>(row, col >> 3) + ((col >> 2) & 1) * 8;
  const char* p1 = lds + tile_off<DH>(row + 8, col >> 3) + ((col >> 2) & 1) * 8;
  const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)p0);
  const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)p1);
  const short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int h) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; e++) r[e] = (__bf16)a[h * 8 + e];
  return r;
}

__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32, 64); }

// Store a transposed 32(d) x 32(row) accumulator set: lane owns one row, DH/32 tiles of 16 d's.
template <int DH>
__device__ __forceinline__ void store_rows(bf16_t* __restrict__ dst, const f32x16 (&acc)[DH / 32], float mul, int g) {
#pragma unroll
  for (int dt = 0; dt < DH / 32; dt++)
#pragma unroll
    for (int q = 0; q < 4; q++) {
      bf16x4 o;
#pragma unroll
      for (int r = 0; r < 4; r++) o[r] = (__bf16)(acc[dt][q * 4 + r] * mul);
      *reinterpret_cast<bf16x4*>(dst + dt * 32 + q * 8 + g * 4) = o;
    }
}

// ---------------------------------------------------------------------------------------------
// Forward.  grid (S/128, B*H); wave w owns queries 128 qt + 32 w .. + 31; 64-key tiles.
// ---------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(int S, int H, const bf16_t* __restrict__ qkv,
                                                            bf16_t* __restrict__ ctx, float* __restrict__ lse) {
  constexpr int KS = DH / 16, DT = DH / 32, TB = TR * DH * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];  // 2 x [K tile | V tile]
  const int qt = gridDim.x - 1 - blockIdx.x;                   // longest rows first
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int Hd = H * DH;
  const size_t ld = 3 * (size_t)Hd;
  const bf16_t* base = qkv + (size_t)b * S * ld + h * DH;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const int q0w = qt * 128 + wave * 32, iq = q0w + (lane & 31);
  const float scale = rsqrtf((float)DH);

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++)
    qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)iq * ld + ks * 16 + g * 8));

  float m = -INFINITY, l = 0.f;
  f32x16 oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int v = 0; v < 16; v++) oacc[dt][v] = 0.f;

  auto step = [&](const char* kt, const char* vt, int j0) {
    if (j0 > q0w + 31) return;  // every key of this tile is in the future of this wave's queries
    f32x16 s[2];
#pragma unroll
    for (int jt = 0; jt < 2; jt++) {
#pragma unroll
      for (int v = 0; v < 16; v++) s[jt][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ks++)
        s[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DH>(kt, jt * 32, ks, lane), qf[ks], s[jt], 0, 0, 0);
    }
    // Scores stay unscaled; the softmax scale rides in the exponent: p = 2^(c s - c m), c = scale log2 e.
    const bool diag = j0 + 63 > q0w;
    const float c = scale * LOG2E;
    float mx = -INFINITY;
    if (diag) {
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int key = j0 + jt * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
          if (key > iq) s[jt][v] = -INFINITY;
          mx = fmaxf(mx, s[jt][v]);
        }
    } else {
#pragma unroll
      for (int jt = 0; jt < 2; jt++)
#pragma unroll
        for (int v = 0; v < 16; v++) mx = fmaxf(mx, s[jt][v]);
    }
    mx = fmaxf(mx, xor32(mx));
    const float mn = fmaxf(m, mx);  // finite: key j0 <= q0w is visible to every query of the wave
    const float corr = __builtin_amdgcn_exp2f((m - mn) * c);
    const float mc = mn * c;
    float rs = 0.f;
#pragma unroll
    for (int jt = 0; jt < 2; jt++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[jt][v], c, -mc));
        s[jt][v] = p;
        rs += p;
      }
    rs += xor32(rs);
    l = l * corr + rs;
    m = mn;
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
      for (int v = 0; v < 16; v++) oacc[dt][v] *= corr;
#pragma unroll
    for (int jt = 0; jt < 2; jt++)
#pragma unroll
      for (int hh = 0; hh < 2; hh++) {
        const bf16x8 pb = pack8(s[jt], hh);
#pragma unroll
        for (int dt = 0; dt < DT; dt++)
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<DH>(vt, dt * 32, jt * 32 + hh * 16, lane), pb,
                                                             oacc[dt], 0, 0, 0);
      }
  };

  const int n_kv = 2 * (qt + 1);
  const unsigned sm = lds_addr(smem);
  tile_dma<DH>(sm, base + Hd, ld);
  tile_dma<DH>(sm + TB, base + 2 * Hd, ld);
  lds_dma_wait();
  __syncthreads();
  for (int t = 0; t < n_kv - 1; t++) {
    const char* cur = smem + (t & 1) * 2 * TB;
    const unsigned nxt = sm + ((t + 1) & 1) * 2 * TB;
    tile_dma<DH>(nxt, base + (size_t)(t + 1) * TR * ld + Hd, ld);  // lands while this tile is computed
    tile_dma<DH>(nxt + TB, base + (size_t)(t + 1) * TR * ld + 2 * Hd, ld);
    step(cur, cur + TB, t * TR);
    lds_dma_wait();
  __syncthreads();
  }
  {
    const char* cur = smem + ((n_kv - 1) & 1) * 2 * TB;
    step(cur, cur + TB, (n_kv - 1) * TR);
  }

  store_rows<DH>(ctx + ((size_t)b * S + iq) * Hd + h * DH, oacc, 1.f / l, g);
  if (g == 0) lse[((size_t)b * H + h) * S + iq] = m * scale + logf(l);
}

// ---------------------------------------------------------------------------------------------
// dQ.  Same decomposition as the forward pass; K and V tiles in LDS.
// ---------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_mfma_kernel(int S, int H, const bf16_t* __restrict__ qkv,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ delta,
                                                               const bf16_t* __restrict__ dctx,
                                                               bf16_t* __restrict__ dqkv) {
  constexpr int KS = DH / 16, DT = DH / 32, TB = TR * DH * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int qt = gridDim.x - 1 - blockIdx.x;
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int Hd = H * DH;
  const size_t ld = 3 * (size_t)Hd;
  const bf16_t* base = qkv + (size_t)b * S * ld + h * DH;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const int q0w = qt * 128 + wave * 32, iq = q0w + (lane & 31);
  const float scale = rsqrtf((float)DH);

  bf16x8 qf[KS], dof[KS];
  const bf16_t* dorow = dctx + ((size_t)b * S + iq) * Hd + h * DH;
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)iq * ld + ks * 16 + g * 8));
    dof[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(dorow + ks * 16 + g * 8));
  }
  const float li = lse[((size_t)b * H + h) * S + iq] * LOG2E;
  const float di = delta[((size_t)b * H + h) * S + iq];

  f32x16 dq[DT];
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int v = 0; v < 16; v++) dq[dt][v] = 0.f;

  auto step = [&](const char* kt, const char* vt, int j0) {
    if (j0 > q0w + 31) return;
    f32x16 s[2], dp[2];
#pragma unroll
    for (int jt = 0; jt < 2; jt++) {
#pragma unroll
      for (int v = 0; v < 16; v++) s[jt][v] = dp[jt][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        s[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DH>(kt, jt * 32, ks, lane), qf[ks], s[jt], 0, 0, 0);
        dp[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DH>(vt, jt * 32, ks, lane), dof[ks], dp[jt], 0, 0, 0);
      }
    }
    const bool diag = j0 + 63 > q0w;
#pragma unroll
    for (int jt = 0; jt < 2; jt++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int key = j0 + jt * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
        float p = __builtin_amdgcn_exp2f(s[jt][v] * (scale * LOG2E) - li);
        if (diag && key > iq) p = 0.f;
        s[jt][v] = p * (dp[jt][v] - di);
      }
#pragma unroll
    for (int jt = 0; jt < 2; jt++)
#pragma unroll
      for (int hh = 0; hh < 2; hh++) {
        const bf16x8 db = pack8(s[jt], hh);
#pragma unroll
        for (int dt = 0; dt < DT; dt++)
          dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<DH>(kt, dt * 32, jt * 32 + hh * 16, lane), db, dq[dt],
                                                           0, 0, 0);
      }
  };

  const int n_kv = 2 * (qt + 1);
  const unsigned sm = lds_addr(smem);
  tile_dma<DH>(sm, base + Hd, ld);
  tile_dma<DH>(sm + TB, base + 2 * Hd, ld);
  lds_dma_wait();
  __syncthreads();
  for (int t = 0; t < n_kv - 1; t++) {
    const char* cur = smem + (t & 1) * 2 * TB;
    const unsigned nxt = sm + ((t + 1) & 1) * 2 * TB;
    tile_dma<DH>(nxt, base + (size_t)(t + 1) * TR * ld + Hd, ld);  // lands while this tile is computed
    tile_dma<DH>(nxt + TB, base + (size_t)(t + 1) * TR * ld + 2 * Hd, ld);
    step(cur, cur + TB, t * TR);
    lds_dma_wait();
  __syncthreads();
  }
  {
    const char* cur = smem + ((n_kv - 1) & 1) * 2 * TB;
    step(cur, cur + TB, (n_kv - 1) * TR);
  }
  store_rows<DH>(dqkv + ((size_t)b * S + iq) * ld + h * DH, dq, scale, g);
}

// ---------------------------------------------------------------------------------------------
// dK, dV.  grid (S/128, B*H); wave w owns keys 128 kt + 32 w .. + 31; 64-query tiles of Q and
// dO (plus their lse and delta) stream through LDS, starting at the diagonal.
// ---------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma_kernel(int S, int H, const bf16_t* __restrict__ qkv,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ delta,
                                                                const bf16_t* __restrict__ dctx,
                                                                bf16_t* __restrict__ dqkv) {
  constexpr int KS = DH / 16, DT = DH / 32, TB = TR * DH * 2;
  constexpr int STAGE = 2 * TB + 2 * TR * 4;  // Q tile | dO tile | lse[64] | delta[64]
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int kt = blockIdx.x;  // key tile 0 sees every query: longest first
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int Hd = H * DH;
  const size_t ld = 3 * (size_t)Hd;
  const bf16_t* base = qkv + (size_t)b * S * ld + h * DH;
  const bf16_t* dob = dctx + (size_t)b * S * Hd + h * DH;
  const float* lrow = lse + ((size_t)b * H + h) * S;
  const float* drow = delta + ((size_t)b * H + h) * S;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5;
  const int j0w = kt * 128 + wave * 32, jk = j0w + (lane & 31);
  const float scale = rsqrtf((float)DH);

  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    kf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)jk * ld + Hd + ks * 16 + g * 8));
    vf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(base + (size_t)jk * ld + 2 * Hd + ks * 16 + g * 8));
  }
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int v = 0; v < 16; v++) dk[dt][v] = dv[dt][v] = 0.f;

  // One 64-query tile, as two halves of 32 so that only one half's scores are live at a time.
  auto step = [&](const char* qt_, const char* dot_, const float* ls, const float* ds_, int i0) {
    if (i0 + 63 < j0w) return;  // every query of this tile precedes this wave's keys
    const bool diag = i0 < j0w + 31;
#pragma unroll
    for (int it = 0; it < 2; it++) {
      f32x16 s, dp;
#pragma unroll
      for (int v = 0; v < 16; v++) s[v] = dp[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DH>(qt_, it * 32, ks, lane), kf[ks], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DH>(dot_, it * 32, ks, lane), vf[ks], dp, 0, 0, 0);
      }
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int r0 = it * 32 + q * 8 + g * 4;
        const float4 l4 = *reinterpret_cast<const float4*>(ls + r0);   // lse * log2(e), pre-scaled on the way in
        const float4 d4 = *reinterpret_cast<const float4*>(ds_ + r0);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dvv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int v = q * 4 + r;
          float p = __builtin_amdgcn_exp2f(fmaf(s[v], scale * LOG2E, -lv[r]));
          if (diag && jk > i0 + r0 + r) p = 0.f;
          s[v] = p;
          dp[v] = p * (dp[v] - dvv[r]);
        }
      }
#pragma unroll
      for (int hh = 0; hh < 2; hh++) {
        const bf16x8 pb = pack8(s, hh), db = pack8(dp, hh);
#pragma unroll
        for (int dt = 0; dt < DT; dt++) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<DH>(dot_, dt * 32, it * 32 + hh * 16, lane), pb,
                                                           dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<DH>(qt_, dt * 32, it * 32 + hh * 16, lane), db,
                                                           dk[dt], 0, 0, 0);
        }
      }
    }
  };

  const int i_first = kt * 128;
  const int n_q = (S - i_first) / TR;
  float rl = 0.f, rdl = 0.f;
  const unsigned sm = lds_addr(smem);
  auto load = [&](int i0, int buf) {
    tile_dma<DH>(sm + buf * STAGE, base + (size_t)i0 * ld, ld);
    tile_dma<DH>(sm + buf * STAGE + TB, dob + (size_t)i0 * Hd, (size_t)Hd);
    if (threadIdx.x < TR) {
      rl = lrow[i0 + threadIdx.x] * LOG2E;
      rdl = drow[i0 + threadIdx.x];
    }
  };
  auto store = [&](char* st) {
    if (threadIdx.x < TR) {
      reinterpret_cast<float*>(st + 2 * TB)[threadIdx.x] = rl;
      reinterpret_cast<float*>(st + 2 * TB + TR * 4)[threadIdx.x] = rdl;
    }
  };
  load(i_first, 0);
  store(smem);
  lds_dma_wait();
  __syncthreads();
  for (int t = 0; t < n_q - 1; t++) {
    const char* cur = smem + (t & 1) * STAGE;
    char* nxt = smem + ((t + 1) & 1) * STAGE;
    load(i_first + (t + 1) * TR, (t + 1) & 1);
    step(cur, cur + TB, reinterpret_cast<const float*>(cur + 2 * TB), reinterpret_cast<const float*>(cur + 2 * TB + TR * 4),
         i_first + t * TR);
    store(nxt);
    lds_dma_wait();
  __syncthreads();
  }
  {
    const char* cur = smem + ((n_q - 1) & 1) * STAGE;
    step(cur, cur + TB, reinterpret_cast<const float*>(cur + 2 * TB), reinterpret_cast<const float*>(cur + 2 * TB + TR * 4),
         i_first + (n_q - 1) * TR);
  }
  bf16_t* out = dqkv + ((size_t)b * S + jk) * ld + h * DH;
  store_rows<DH>(out + Hd, dk, scale, g);
  store_rows<DH>(out + 2 * Hd, dv, 1.f, g);
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
  constexpr size_t lds = 4 * (size_t)TR * DH * 2;
  FAX_TRY(set_lds(attn_fwd_mfma_kernel<DH>, lds));
  hipLaunchKernelGGL((attn_fwd_mfma_kernel<DH>), dim3(S / 128, B * H), dim3(256), lds, s, S, H, qkv, ctx, lse);
  FAX_LAUNCH_CHECK("attn_fwd_mfma");
  return FAX_OK;
}

int attn_fwd_mfma(int B, int S, int H, int dh, const void* qkv, void* ctx, float* lse, hipStream_t s) {
  if (dh == 64) return fwd_t<64>(B, S, H, (const bf16_t*)qkv, (bf16_t*)ctx, lse, s);
  return fwd_t<128>(B, S, H, (const bf16_t*)qkv, (bf16_t*)ctx, lse, s);
}

template <int DH>
static int bwd_t(int B, int S, int H, const bf16_t* qkv, const float* lse, const float* delta, const bf16_t* dctx,
                 bf16_t* dqkv, hipStream_t s) {
  constexpr size_t lds_q = 4 * (size_t)TR * DH * 2;
  constexpr size_t lds_kv = 2 * (2 * (size_t)TR * DH * 2 + 2 * TR * 4);
  FAX_TRY(set_lds(attn_bwd_dq_mfma_kernel<DH>, lds_q));
  FAX_TRY(set_lds(attn_bwd_dkv_mfma_kernel<DH>, lds_kv));
  hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<DH>), dim3(S / 128, B * H), dim3(256), lds_kv, s, S, H, qkv, lse, delta,
                     dctx, dqkv);
  hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<DH>), dim3(S / 128, B * H), dim3(256), lds_q, s, S, H, qkv, lse, delta, dctx,
                     dqkv);
  FAX_LAUNCH_CHECK("attn_bwd_mfma");
  return FAX_OK;
}

int attn_bwd_mfma(int B, int S, int H, int dh, const void* qkv, const void* ctx, const float* lse, const void* dctx,
                  void* dqkv, float* delta, hipStream_t s) {
  FAX_TRY(attn_delta(FAX_BF16, B, S, H, dh, ctx, dctx, delta, s));
  if (dh == 64)
    return bwd_t<64>(B, S, H, (const bf16_t*)qkv, lse, delta, (const bf16_t*)dctx, (bf16_t*)dqkv, s);
  return bwd_t<128>(B, S, H, (const bf16_t*)qkv, lse, delta, (const bf16_t*)dctx, (bf16_t*)dqkv, s);
}

}  // namespace fax
