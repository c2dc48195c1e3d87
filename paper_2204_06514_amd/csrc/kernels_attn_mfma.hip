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
#include <type_traits>

#include "fax_internal.h"

namespace fax {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
template <int V> using I = std::integral_constant<int, V>;
using T_ = std::true_type;
using F_ = std::false_type;

static constexpr float LOG2E = 1.4426950408889634f;
static constexpr int TR = 64;  // rows per LDS tile
static constexpr float MAX_LAG = 8.f;  // forward: octaves the running maximum may rise above the exponent's reference point

template <int DH>
__device__ __forceinline__ int swz(int row) {
  const int f = ((row & 3) << 1) | ((row >> 2) & 1);
  return DH >= 128 ? f | (row & 8) : f;  // 16 chunks per row: 16 consecutive rows in 16 distinct chunks
}

template <int DH>
__device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * (DH * 2) + ((chunk ^ swz<DH>(row)) << 4);
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
    const int chunk = (lane % NCH) ^ swz<DH>(row);
    lds_dma16(src + (size_t)row * ld + chunk * 8, lds + seg * 1024u);
  }
}

// The two fragment readers below are called with compile-time tile coordinates.  Their addresses
// are written as (one per-lane value, the same for every call) XOR (a constant) + (a constant):
// the swizzle only involves row bits 0..3 and chunk bits, which the tile coordinates (multiples of
// 16 rows, whole k-steps, 32-column blocks) enter without carries.  Spelled as tile_off(row, chunk)
// per call, each coordinate pair is a separate loop-invariant vector value to the compiler: some
// fifty registers per kernel, more than the register budget of two waves per SIMD leaves.

// A operand, rows rb..rb+31 of the tile (rb a multiple of 16), contraction over the tile's columns
// (k-step ks).
template <int DH>
__device__ __forceinline__ bf16x8 frag_rows(const char* lds, int rb, int ks, int lane) {
  const int l31 = lane & 31;
  const unsigned lane_part = l31 * (DH * 2) + (((lane >> 5) ^ swz<DH>(l31)) << 4);  // tile_off(l31, lane >> 5)
  const unsigned off = (lane_part ^ (unsigned)(ks << 5)) + (unsigned)(rb * (DH * 2));  // tile_off(rb + l31, 2 ks + (lane >> 5))
  const uint4 v = *reinterpret_cast<const uint4*>(lds + off);
  return __builtin_bit_cast(bf16x8, v);
}

// A operand = transpose of the tile: output rows are tile columns cb..cb+31 (cb a multiple of 32),
// contraction over tile rows r0 + {0..3, 8..11} + 4 g (r0 a multiple of 16; the k-slot order
// described in the header).
template <int DH>
__device__ __forceinline__ bf16x8 frag_cols(const char* lds, int cb, int r0, int lane) {
  const int blk = lane >> 4, i = lane & 15;
  const int rl = (blk >> 1) * 4 + (i >> 2);        // row within the group of 16
  const int cl = (blk & 1) * 16 + (i & 3) * 4;     // column within the block of 32
  const unsigned lane_part = rl * (DH * 2) + (((cl >> 3) ^ swz<DH>(rl)) << 4) + ((cl >> 2) & 1) * 8;
  const unsigned x = lane_part ^ (unsigned)((cb >> 3) << 4);
  typedef __attribute__((address_space(3))) short4v lds_s4;
  const char* p0 = lds + x + (unsigned)(r0 * (DH * 2));
  // eight rows further down: row bit 3 flips, and with it (at 16 chunks per row) chunk bit 3
  const char* p1 = lds + (x ^ (DH >= 128 ? 0x80u : 0u)) + (unsigned)((r0 + 8) * (DH * 2));
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

// Combine a value across lanes l and l ^ 32 (the two lanes that share a row of a 32x32 MFMA tile).
// v_permlane32_swap hands every lane both values through the vector ALU; a shuffle would go
// through LDS and, being returned in order with the fragment reads in flight, wait for all of them.
__device__ __forceinline__ float max32(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum32(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// The tiles arrive through inline-assembly loads that the compiler does not count.  A value it
// loads itself before the main loop and first uses inside it makes the compiler put its own
// "at most N loads outstanding" wait inside the loop, which then also waits for the tile loads
// issued a moment earlier, every iteration.  Passing such values through here forces that wait to
// happen once, before the loop.
template <typename T>
__device__ __forceinline__ void settle(T& v) { asm volatile("" : "+v"(v)); }

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

// Segment i of this wave's share of a 64 x DH tile (see tile_dma above), as one load instruction:
// wave-uniform tile address in scalar registers plus a per-lane byte offset that depends only on
// the lane, the segment and the row stride, so the compiler computes it once per kernel and a load
// costs no vector arithmetic.  `wave` must be wave-uniform (readfirstlane).
template <int DH>
__device__ __forceinline__ void tile_dma_seg(unsigned lds, const bf16_t* __restrict__ src, size_t ld, int wave, int i) {
  constexpr int NCH = DH / 8, RPI = 64 / NCH;
  const int lane = threadIdx.x & 63;
  const int seg = wave * (DH / 32) + i;
  const int row = seg * RPI + lane / NCH;
  const int chunk = (lane % NCH) ^ swz<DH>(row);
  lds_dma16(src, (unsigned)(((size_t)row * ld + chunk * 8) * sizeof(bf16_t)), lds + seg * 1024u);
}

// Workgroup -> (pair of 128-row tiles, batch-head) for the three kernels.  Under the causal mask
// row tile r of the forward / dQ kernels meets r + 1 key blocks and key tile r of the dK/dV
// kernel meets n - r query blocks, so tiles p and n - 1 - p are done by one workgroup, one after
// the other: every workgroup then has the same amount of work and the grid drains without a
// ragged tail.  Consecutive workgroup ids go to different XCDs; all workgroups of one
// (batch, head) are dealt to the same XCD so that its K/V (Q/dO) stay in that XCD's L2.
__device__ __forceinline__ void pair_of_tiles(int n_tiles, int BH, int& pair, int& bh) {
  const int n_pair = (n_tiles + 1) / 2;
  if (BH % 8 == 0) {
    const int slot = blockIdx.x / 8;
    bh = (slot / n_pair) * 8 + blockIdx.x % 8;
    pair = slot % n_pair;
  } else {
    bh = blockIdx.x / n_pair;
    pair = blockIdx.x % n_pair;
  }
}

// The work on one block of keys (queries) is laid out by hand as three phases,
//   P1  MFMAs that produce scores (row fragments of the streamed tiles from LDS)
//   V   the vector work on the scores
//   P3  MFMAs that consume the packed probabilities (transpose-read fragments)
// and inside P1 and P3 every MFMA is followed by the LDS read of a fragment needed LEAD MFMAs
// later (sched_barrier pins that order), so the matrix core does not wait for an LDS round trip.
// P1's last reads fetch P3's first fragments; P3's last reads fetch the next P1's first rows.
// MFMAs that accumulate into the same registers are kept at least two slots apart.
//
// Within one wave the three phases use different units (matrix core and LDS, vector unit, matrix
// core and LDS) one after the other.  Two ways of filling the idle ones were built and measured:
//   * skew: the vector work of half u rides slot by slot on the MFMAs of its neighbours within
//     the same wave (three LDS buffers, two sets of score registers);
//   * occupancy: keep the kernel within the register budget of two waves per SIMD and the LDS
//     budget of two workgroups per CU and let the hardware interleave two workgroups' phases
//     (a wave raises its priority for its MFMA phases, so the matrix core is fed first: -4 %).
// Occupancy won wherever the kernel fits (forward 208 -> 167 us and dQ 261 -> 217 us at dh = 128,
// dK/dV 13.2 -> 11.2 ms over the 124M model's twelve layers at dh = 64; the skewed forward and dQ
// kernels were 4-20 % slower than these and are gone).  dK/dV at dh = 128 holds 192 registers of
// accumulators and B operands alone and stays a one-wave-per-SIMD kernel with the skew.

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
__device__ __forceinline__ float f4_get(const float4& v, int r) { return r == 0 ? v.x : r == 1 ? v.y : r == 2 ? v.z : v.w; }

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
                 bf16_t* dqkv, float* delta, hipStream_t s) {
  constexpr size_t lds_q = 2 * (2 * (size_t)TR * DH * 2);  // two stages of K tile | V tile
  const dim3 grid(((S / 128 + 1) / 2) * B * H);
  // dQ first: it also produces delta, which the dK/dV kernel reads
  FAX_TRY(set_lds(attn_bwd_dq_mfma_kernel<DH>, lds_q));
  hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<DH>), grid, dim3(256), lds_q, s, S, H, B * H, qkv, lse, ctx, dctx, delta, dqkv);
  if constexpr (DH == 64) {
    constexpr size_t lds_kv = 2 * (2 * (size_t)TR * DH * 2 + 4 * 256);  // two stages of Q tile | dO tile | lse, delta
    FAX_TRY(set_lds(attn_bwd_dkv_phased_mfma_kernel<DH>, lds_kv));
    hipLaunchKernelGGL((attn_bwd_dkv_phased_mfma_kernel<DH>), grid, dim3(256), lds_kv, s, S, H, B * H, qkv, lse, delta, dctx,
                       dqkv);
  } else {
    constexpr size_t lds_kv = 3 * (2 * (size_t)TR * DH * 2 + 4 * 256);  // three stages
    FAX_TRY(set_lds(attn_bwd_dkv_mfma_kernel<DH>, lds_kv));
    hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<DH>), grid, dim3(256), lds_kv, s, S, H, B * H, qkv, lse, delta, dctx, dqkv);
  }
  FAX_LAUNCH_CHECK("attn_bwd_mfma");
  return FAX_OK;
}

int attn_bwd_mfma(int B, int S, int H, int dh, const void* qkv, const void* ctx, const float* lse, const void* dctx,
                  void* dqkv, float* delta, hipStream_t s) {
  if (dh == 64)
    return bwd_t<64>(B, S, H, (const bf16_t*)qkv, (const bf16_t*)ctx, lse, (const bf16_t*)dctx, (bf16_t*)dqkv, delta, s);
  return bwd_t<128>(B, S, H, (const bf16_t*)qkv, (const bf16_t*)ctx, lse, (const bf16_t*)dctx, (bf16_t*)dqkv, delta, s);
}

}  // namespace fax
