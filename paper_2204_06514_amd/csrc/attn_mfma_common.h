// Shared pieces of the attention kernels on the CDNA4 matrix cores: LDS tile layout, direct
// global -> LDS tile loads, fragment readers, lane-pair reductions, workgroup -> tile mapping.
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
#pragma once
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

__device__ __forceinline__ float f4_get(const float4& v, int r) { return r == 0 ? v.x : r == 1 ? v.y : r == 2 ? v.z : v.w; }

}  // namespace fax
