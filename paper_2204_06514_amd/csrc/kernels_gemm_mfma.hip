// bf16 GEMM on the CDNA4 matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulate.
//
// One 256-thread workgroup (4 wavefronts, 2x2) computes a BM x BN tile of C, stepping over K in
// slabs of 64.  Slabs of A and B go from global memory straight into LDS
// (global_load_lds_dwordx4: no staging registers, no LDS store instructions), three buffers for
// A and two for B, each slab requested about a slab of MFMAs before it is needed and its load
// instructions spread over that time.
//
// An operand whose contraction index is contiguous in memory ("KC": A stored [M,K], B stored
// [N,K]) is kept in LDS as [row][64] with the 16-byte chunk index XOR-ed with ((row >> 1) & 7):
// measured on gfx950, the 128-bit fragment reads of 32 consecutive rows then run at the full LDS
// rate (XOR with row & 7 is 15 % slower, no swizzle 4x slower).
// An operand whose M/N index is contiguous ("MC": A stored [K,M], B stored [K,N]) is kept as
// [k][rows] and fetched with ds_read_b64_tr_b16, the LDS transpose read: 16 lanes pick up four
// k-rows x 16 columns and each lane receives 4 consecutive k for its own column; two such reads
// make one MFMA operand.  There the 32-byte column-group index is XOR-ed with mc_swizzle(k), which
// spreads the eight k-rows that two 16-lane blocks read in one pass over all banks (see there;
// SQ_LDS_BANK_CONFLICT reads 0 for every flavour of the kernel, where XOR with (k & 3) left 31 %
// of the LDS cycles in conflicts with one such operand and 49 % with two -- at the same kernel
// time: these kernels do not wait for the LDS).  A direct-to-LDS load writes 1024
// consecutive LDS bytes per wave instruction (lane i at +16 i), so both swizzles are applied on
// the global side: each lane fetches the chunk that belongs at its LDS position.
//
// MFMA 32x32x16 lane layout (lane l): first/second operand = row/column (l & 31) of the product,
// k = 8 (l >> 5) + 0..7; accumulator v = 0..15 holds element [8 (v >> 2) + 4 (l >> 5) + (v & 3)][l & 31].
// The kernel feeds the B fragment as first operand and the A fragment as second, i.e. it
// accumulates C^T tiles: a lane then owns row m = l & 31 of C and, in v = 4 g .. 4 g + 3, the four
// consecutive columns n = 8 g + 4 (l >> 5) + 0..3 -- a 16-byte unit for the epilogue.
#include <type_traits>

#include <algorithm>

#include "fax_internal.h"

namespace fax {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
template <int V> using I = std::integral_constant<int, V>;
using T_ = std::true_type;
using F_ = std::false_type;

static constexpr int GK = 64;  // K slab

template <int ROWS, bool KC>
struct TileLds {
  static constexpr int BYTES = ROWS * GK * 2;
  static constexpr int NSEG = BYTES / 1024 / 4;  // 1 KB segments (= load instructions) per wave per slab
};

// Byte offset, from the slab's first element, of the 16 bytes that belong at LDS byte offset `b`
// of the slab.  Inverse of the layouts that frag_load() reads.  Does not depend on the slab's
// position: each lane computes its offsets once and only the (wave-uniform) slab base moves.
// XOR applied to the 32-byte column-group index of k-row kr of an M/N-contiguous operand.  A
// transpose read has each 16-lane block fetch four k-rows x 32 bytes; blocks 0 and 1 take the same
// k-rows at neighbouring groups, blocks 2 and 3 the k-rows eight further down.  Whichever two
// blocks the LDS serves in one pass, (0, 1) or (0, 2), their eight 32-byte pieces must fall into
// eight different groups of the 256-byte bank window: bits 0-1 of kr go to bits 1-2 of the XOR
// (four rows, two apart), bit 3 of kr to bit 0.
__device__ __forceinline__ int mc_swizzle(int kr) { return ((kr & 3) << 1) | ((kr >> 3) & 1); }

template <int ROWS, bool KC>
__device__ __forceinline__ unsigned slab_lane_offset(int ld, int b) {
  if (KC) {
    const int row = b >> 7, pc = (b >> 4) & 7;
    return (unsigned)(row * ld + ((pc ^ ((row >> 1) & 7)) << 3)) * 2u;
  }
  constexpr int RB = ROWS * 2;  // bytes per k-row
  const int kr = b / RB, pc = (b % RB) >> 4;
  const int lc = (((pc >> 1) ^ mc_swizzle(kr)) << 1) | (pc & 1);
  return (unsigned)(kr * ld + (lc << 3)) * 2u;
}

// One MFMA operand (8 bf16 per lane) for the 32 rows starting at rb, k-step ks (16 wide).
template <int ROWS, bool KC>
__device__ __forceinline__ bf16x8 frag_load(const char* lds, int rb, int ks, int lane) {
  if (KC) {
    const int row = rb + (lane & 31);
    const int chunk = ks * 2 + (lane >> 5);
    const uint4 v = *reinterpret_cast<const uint4*>(lds + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
    return __builtin_bit_cast(bf16x8, v);
  } else {
    const int blk = lane >> 4, i = lane & 15;
    const int kr = ks * 16 + (blk >> 1) * 8 + (i >> 2);  // kr + 4 has the same swizzle
    const int col = rb + (blk & 1) * 16 + (i & 3) * 4;
    const char* p = lds + kr * (ROWS * 2) + (((col >> 4) ^ mc_swizzle(kr)) << 5) + (col & 15) * 2;
    typedef __attribute__((address_space(3))) short4v lds_s4;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(p));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(p + 4 * ROWS * 2));
    const short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

// Epilogue flavours, fixed at compile time: a kind, plus flags for the optional operands.  Nothing
// in the store loop may hang on a run-time condition: stores count towards the same counter as
// loads on this target, so the conservative wait the compiler places where branches that contain
// loads rejoin would also wait for every earlier store to be acknowledged, once per row.
enum { EK_STORE = 0, EK_GELU_TANH = 1, EK_GELU_ERF = 2, EK_DGELU = 3, EK_F32 = 5 };
enum {
  EM_RES = 8,  // bf16 kinds: add the residual R;  EK_F32: add to what C already holds
  EM_C2 = 16,  // EK_STORE: also write the plain product (before bias and residual) to C2
  EM_COLSUM = 32  // EK_F32, B stored [K, N]: also colsum[n] (+)= sum_k B[k, n]
};
constexpr int em_kind(int em) { return em & 7; }
constexpr bool em_dgelu(int em) { return em_kind(em) == EK_DGELU; }
constexpr bool em_gelu(int em) { return em_kind(em) == EK_GELU_TANH || em_kind(em) == EK_GELU_ERF; }

// tanh-form GELU through the logistic function: (1 + tanh z) / 2 = 1 / (1 + exp(-2 z)), one
// v_exp_f32 and one v_rcp_f32 per element, a few ulp in fp32 (the outputs are rounded to bf16).
// This runs in the GEMM's epilogue with the matrix cores idle, so the operation count matters:
// 18 issue slots per element (the two quarter-rate instructions count four each), with u^2
// shared between the argument and the derivative and every constant folded:
//   -2 z log2(e) = u (A + B u^2),  A = -2 sqrt(2/pi) log2(e),  B = 0.044715 A
//   gelu = u s,  gelu' = s + (gelu - gelu s) (C + D u^2),  C = 2 sqrt(2/pi),  D = 3 * 0.044715 C
__device__ __forceinline__ void gelu_tanh_both(float u, float& g, float& dg) {
  const float u2 = u * u;
  const float e = __builtin_amdgcn_exp2f(u * fmaf(-0.10294324f, u2, -2.3022082f));
  const float sg = __builtin_amdgcn_rcpf(1.f + e);
  g = u * sg;
  dg = fmaf(fmaf(-g, sg, g), fmaf(0.21406445f, u2, 1.5957691216057308f), sg);
}

// Four consecutive columns n..n+3 of row m at once: 8-byte bf16 loads and stores.
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
__device__ __forceinline__ float4 ld_bf16x4(const void* base, size_t idx) {
  const bf16x4 v = *reinterpret_cast<const bf16x4*>((const bf16_t*)base + idx);
  return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
}
__device__ __forceinline__ void st_bf16x4(void* base, size_t idx, float4 a) {
  bf16x4 v;
  v[0] = (__bf16)a.x; v[1] = (__bf16)a.y; v[2] = (__bf16)a.z; v[3] = (__bf16)a.w;
  // Streaming store: the tile is not read again by this kernel, and a round of tiles is as large as the
  // L2s (32 x 128 KB per XCD against 4 MB), where it would push out the operand panels that the
  // XCD's workgroups share.  Measured against plain stores, A-B-A-B on one box: the 768-wide model
  // 64.8-66.2 -> 63.9-64.0 ms (forward 21.4-22.1 -> 20.55 ms), the 1024-wide one -0.6 %, d_model 4096
  // unchanged.
  __builtin_nontemporal_store(v, reinterpret_cast<bf16x4*>((bf16_t*)base + idx));
}
// `side` is the row's residual (R) or, for the GELU' flavour, the stored derivative (U), fetched by
// the caller ahead of time so that its latency overlaps the LDS turn-around.
// For the fp32 flavour (plain product, optionally added to what C holds) `side` is the old C.
template <int EM>
__device__ __forceinline__ void mfma_epilogue4(const EpiArgs& e, int m, int n, float4 a, float4 bias, float4 side) {
  constexpr int KIND = em_kind(EM);
  if (KIND == EK_F32) {
    if (EM & EM_RES) { a.x += side.x; a.y += side.y; a.z += side.z; a.w += side.w; }
    typedef __attribute__((ext_vector_type(4))) float f32x4s;
    const f32x4s av = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(av, reinterpret_cast<f32x4s*>((float*)e.C + (size_t)m * e.ldc + n));  // as st_bf16x4
    return;
  }
  if (EM & EM_C2) st_bf16x4(e.C2, (size_t)m * e.ldc2 + n, a);
  a.x += bias.x; a.y += bias.y; a.z += bias.z; a.w += bias.w;
  if (!em_dgelu(EM) && (EM & EM_RES)) {
    a.x += side.x; a.y += side.y; a.z += side.z; a.w += side.w;
  }
  if (em_gelu(EM)) {  // C = gelu'(acc), C2 = gelu(acc)
    float4 g, dg;
    if (KIND == EK_GELU_TANH) {
      gelu_tanh_both(a.x, g.x, dg.x); gelu_tanh_both(a.y, g.y, dg.y);
      gelu_tanh_both(a.z, g.z, dg.z); gelu_tanh_both(a.w, g.w, dg.w);
    } else {
      g = make_float4(gelu_f(a.x, FAX_GELU_ERF), gelu_f(a.y, FAX_GELU_ERF), gelu_f(a.z, FAX_GELU_ERF),
                      gelu_f(a.w, FAX_GELU_ERF));
      dg = make_float4(gelu_grad_f(a.x, FAX_GELU_ERF), gelu_grad_f(a.y, FAX_GELU_ERF), gelu_grad_f(a.z, FAX_GELU_ERF),
                       gelu_grad_f(a.w, FAX_GELU_ERF));
    }
    st_bf16x4(e.C, (size_t)m * e.ldc + n, dg);
    st_bf16x4(e.C2, (size_t)m * e.ldc2 + n, g);
    return;
  }
  if (em_dgelu(EM)) { a.x *= side.x; a.y *= side.y; a.z *= side.z; a.w *= side.w; }
  st_bf16x4(e.C, (size_t)m * e.ldc + n, a);
}

// Tile number -> tile of the persistent kernel (comment at its use below).  Host and device: the
// host copy lets the tests check that every walk visits every tile exactly once.
__host__ __device__ inline void tile_walk(int id, int tiles_m, int tiles_n, int group, int& tm_i, int& tn_i) {
  if (group == 0) {
    // 256 workgroups, tile counts that are multiples of 16 both ways: round number id >> 8 is a
    // 16 x 16 block of tiles (walked down the tile rows first), XCD x takes the 4 x 8 block at
    // (x & 3, x >> 2) of it, its workgroup j the tile (j & 3, j >> 2) of that.  The eight XCDs then
    // work on 16 + 16 operand panels at any time instead of 32 + 8.
    const int x = id & 7, j = (id >> 3) & 31, sb = id >> 8;
    const int sbm = tiles_m >> 4;
    tm_i = ((sb % sbm) << 4) + ((x & 3) << 2) + (j & 3);
    tn_i = ((sb / sbm) << 4) + ((x >> 2) << 3) + (j >> 2);
    return;
  }
  const int nt = tiles_m * tiles_n;
  if (nt % 8 == 0) id = (id % 8) * (nt / 8) + id / 8;
  const int per_group = group * tiles_n;
  const int g = id / per_group;
  const int gm0 = g * group;
  const int gsz = group < tiles_m - gm0 ? group : tiles_m - gm0;
  tm_i = gm0 + (id % per_group) % gsz;
  tn_i = (id % per_group) / gsz;
}

template <int BM, int BN, bool A_KC, bool B_KC, int EM>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(int M, int N, int K, const bf16_t* __restrict__ A, int lda,
                                                        const bf16_t* __restrict__ B, int ldb, EpiArgs e, int tiles_m,
                                                        int tiles_n) {
  using LA = TileLds<BM, A_KC>;
  using LB = TileLds<BN, B_KC>;
  constexpr int TM = BM / 64, TN = BN / 64;  // 32x32 MFMA tiles per wave in each direction
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // LDS: three buffers for A slabs, then two for B slabs (see the pipeline below).
  constexpr int A_BUFS = 3;  // and two for B
  constexpr int B_BASE = A_BUFS * LA::BYTES;

  // Persistent workgroups: workgroup b works through tiles b, b + gridDim.x, ...  (the host
  // launches one workgroup per CU, or fewer when there are fewer tiles).  The point is the seam
  // between two tiles: the first slabs of the next tile are requested before the epilogue of the
  // finished one, so their latency (about 3 us from a cold start) runs behind the epilogue.
  //
  // Tile number -> tile.  Consecutive workgroup ids land on different XCDs (8 of them, each with
  // its own L2) and gridDim.x is a multiple of 8 whenever that matters, so a workgroup's tile
  // numbers all have its own residue mod 8; the number is first re-dealt so that each XCD owns a
  // contiguous run of tiles, then tiles are walked in column-major groups of e.group (4 or 8, chosen
  // on the host) tile-rows to keep the working set of A and B panels small.  e.group = 0 selects the
  // walk in which the XCDs' blocks of a round lie side by side (below).
  const int nt = tiles_m * tiles_n;
  auto tile_of = [&](int id, int& tm_i, int& tn_i) { tile_walk(id, tiles_m, tiles_n, e.group, tm_i, tn_i); };

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // in a scalar register: LDS segment addresses stay scalar
  const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);

  // This wave's share of a slab: segments wave*NSEG .. +NSEG-1 of A and likewise of B.  Segment
  // q of a slab is bytes [1024 q, 1024 q + 1024) of its buffer; this lane's 16 bytes sit at
  // +16 lane.  The global address of a segment is (uniform slab base) + (this lane's offset,
  // fixed for the whole kernel), so stepping along K is scalar arithmetic only.
  constexpr int NSA = LA::NSEG, NSB = LB::NSEG;
  unsigned a_lane_off[NSA], b_lane_off[NSB];
#pragma unroll
  for (int q = 0; q < NSA; q++) a_lane_off[q] = slab_lane_offset<BM, A_KC>(lda, (wave * NSA + q) * 1024 + lane * 16);
#pragma unroll
  for (int q = 0; q < NSB; q++) b_lane_off[q] = slab_lane_offset<BN, B_KC>(ldb, (wave * NSB + q) * 1024 + lane * 16);
  const size_t a_kstride = A_KC ? 1 : (size_t)lda, b_kstride = B_KC ? 1 : (size_t)ldb;
  const unsigned smem_addr = lds_addr(smem);
  auto a_tile_of = [&](int tm_i) { return A + (A_KC ? (size_t)tm_i * BM * lda : (size_t)tm_i * BM); };
  auto b_tile_of = [&](int tn_i) { return B + (B_KC ? (size_t)tn_i * BN * ldb : (size_t)tn_i * BN); };
  // segment q of the A (B) slab at k0 of the tile at `tile_base` -> A (B) buffer number `buf`
  auto dma_a_from = [&](const bf16_t* tile_base, int q, int k0, int buf) {
    lds_dma16(tile_base + k0 * a_kstride, a_lane_off[q], smem_addr + buf * LA::BYTES + (wave * NSA + q) * 1024);
  };
  auto dma_b_from = [&](const bf16_t* tile_base, int q, int k0, int buf) {
    lds_dma16(tile_base + k0 * b_kstride, b_lane_off[q], smem_addr + B_BASE + buf * LB::BYTES + (wave * NSB + q) * 1024);
  };
  // With the contraction split (fp32-output form) the work items are (K range, tile) pairs: item
  // v is tile v % nt over slabs [r nkt / splits, (r + 1) nkt / splits), r = v / nt, nkt = K / GK,
  // and writes the partial product r (and the partial column sums r).
  const int splits = e.splits > 1 ? e.splits : 1;
  const int nk_total = K / GK;
  auto k_range = [&](int item, int& first, int& count) {
    const int r = item / nt;
    first = (int)((unsigned)r * (unsigned)nk_total / (unsigned)splits);  // r < 32, nk_total < 2^25
    count = (int)((unsigned)(r + 1) * (unsigned)nk_total / (unsigned)splits) - first;
  };
  // A tile starts with slab 0 in A[0], B[0] and slab 1 in A[1], B[1].  Everything but B of slab 1
  // can be requested while the previous tile's epilogue still uses A[2] and B[1].
  auto request_first_slabs = [&](const bf16_t* a_base, const bf16_t* b_base, int nk) {
#pragma unroll
    for (int q = 0; q < NSA; q++) dma_a_from(a_base, q, 0, 0);
#pragma unroll
    for (int q = 0; q < NSB; q++) dma_b_from(b_base, q, 0, 0);
    if (nk > 1) {
#pragma unroll
      for (int q = 0; q < NSA; q++) dma_a_from(a_base, q, GK, 1);
    }
  };

  int tm_i, tn_i;
  int k_first, nk_item;
  tile_of(blockIdx.x % nt, tm_i, tn_i);
  k_range(blockIdx.x, k_first, nk_item);
  size_t k_begin = (size_t)k_first * GK;
  request_first_slabs(a_tile_of(tm_i) + k_begin * a_kstride, b_tile_of(tn_i) + k_begin * b_kstride, nk_item);
  for (int tile = blockIdx.x; tile < nt * splits; tile += gridDim.x) {
  const int nk = nk_item;
  const int m0 = tm_i * BM, n0 = tn_i * BN;
  const bf16_t* const a_tile = a_tile_of(tm_i) + k_begin * a_kstride;
  const bf16_t* const b_tile = b_tile_of(tn_i) + k_begin * b_kstride;
  EpiArgs et = e;  // this item's view of the epilogue operands
  if (em_kind(EM) == EK_F32) {
    et.C = (float*)e.C + (size_t)(tile / nt) * e.split_stride;
    if (EM & EM_COLSUM) et.colsum = e.colsum + (size_t)(tile / nt) * e.colsum_stride;
  }
  auto dma_a = [&](int q, int k0, int buf) { dma_a_from(a_tile, q, k0, buf); };
  auto dma_b = [&](int q, int k0, int buf) { dma_b_from(b_tile, q, k0, buf); };
  lds_dma_wait();   // slab 0 and A of slab 1 (requested a whole epilogue ago, except for the first tile)
  __syncthreads();  // ... are visible; every wave is done with the previous tile's epilogue staging
  if (nk > 1) {
#pragma unroll
    for (int q = 0; q < NSB; q++) dma_b(q, GK, 1);  // B of slab 1: needed at the first in-loop barrier, waited for there
  }
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  // Software pipeline.  A slab is four k-steps ("phases") of TM x TN MFMAs each.  Operand
  // fragments are double buffered in registers: phase s issues the LDS reads for phase s+1.
  //
  // With one wave per SIMD nothing else can fill the matrix core while this wave issues other
  // instructions, so they are slotted between MFMAs: slot t of a phase follows MFMA t and holds
  // at most one fragment read and one slab load.  sched_barrier after each slot keeps the
  // compiler from regrouping them.
  //
  // The slab loads set the pace of the schedule.  The CU's address unit takes 16 cycles per
  // 1 KB load instruction and is shared by the four waves, so a slab (64 instructions at 256^2)
  // keeps it busy for half of the slab's MFMA time: requested in one burst, the loads block the
  // issuing waves and with them the matrix cores.  They are therefore spread over the whole slab,
  // which needs somewhere to put them while both resident slabs are still being read: A gets a
  // third buffer.  While slab kt is multiplied,
  //   phases 0-1:          request A(kt+2) into the spare A buffer, a load every few slots;
  //   phase 2, slot PB:    all fragment reads of slab kt are done; wait until everything older
  //                        than the A loads just issued has landed (that is slab kt+1), barrier:
  //                        slab kt+1 is published and the B buffer of slab kt is free;
  //   rest of phase 2, 3:  request B(kt+2) into that buffer; phase 3 also reads the first
  //                        fragments of slab kt+1.
  // One barrier per slab.  PB leaves four MFMAs between the last fragment read and the wait.
  static_assert(GK / 16 == 4, "pipeline below is written for four k-steps per slab");
  constexpr int NSLOT = TM * TN;
  static_assert(TM + TN <= NSLOT, "slots per phase");
  constexpr int PB = (TM + TN + 4 < NSLOT) ? TM + TN + 4 : NSLOT;  // barrier position within phase 2
  constexpr int SLOTS_A = 2 * NSLOT;             // slots open to the A loads
  constexpr int SLOTS_B = NSLOT - PB + NSLOT;    // ... and to the B loads
  static_assert(NSA <= SLOTS_A && NSB <= SLOTS_B && NSA < 64, "load schedule");
  // Optional by-product (EM_COLSUM, B stored [K, N]): colsum[n] (+)= sum over k of B[k, n], which for
  // a weight-gradient product is the bias gradient.  Every workgroup sweeps all of K, so the
  // workgroups of tile row 0 between them see every column of B in full; their waves add up the
  // B fragments they feed to the matrix core anyway (lane = column, 8 k's per fragment).  The
  // two waves that share a column range (wm = 0 and wm != 0) take alternate elements, one
  // element per wave and slot at 256^2, and combine through LDS after the loop.  The main loop
  // exists in three copies (no sums, even elements, odd elements) so that the other workgroups
  // pay nothing and the element indices stay compile-time constants.
  constexpr bool CS = (EM & EM_COLSUM) != 0;
  static_assert(!CS || !B_KC, "column sums are taken from [K, N] fragments");
  const bool cs_on = CS && tm_i == 0;
  const int cs_half = wm != 0;
  float cs[TN];
#pragma unroll
  for (int j = 0; j < TN; j++) cs[j] = 0.f;
  auto main_loop = [&](auto cs_c, auto half_c) {
  constexpr bool CSON = decltype(cs_c)::value;
  constexpr int CS_HALF = decltype(half_c)::value;  // which element of each pair this wave sums
  constexpr int EPSL = 8 * TN / NSLOT;  // fragment elements summed per slot
  static_assert(EPSL % 2 == 0, "two waves share the elements of a slot");
  bf16x8 fa[2][TM], fb[2][TN];
  // Slots [T0, T1) of one phase: MFMA t on fragment buffer USE, then fragment read t of k-step ks
  // from (srcA, srcB) into buffer USE ^ 1 (when LOADF), then the slab loads that the schedule
  // puts at this slot: LOADS 1 = A loads, slot number t + OFS of SLOTS_A; LOADS 2 = B loads,
  // slot number t + OFS of SLOTS_B; segment q goes to slot floor(q * SLOTS / NSEG).
  auto phase = [&](auto use_c, auto loadf_c, auto loads_c, auto ofs_c, auto t0_c, auto t1_c, const char* srcA,
                   const char* srcB, int ks, int k_next, int buf) {
    constexpr int USE = decltype(use_c)::value, LOADS = decltype(loads_c)::value, OFS = decltype(ofs_c)::value;
    constexpr int T0 = decltype(t0_c)::value, T1 = decltype(t1_c)::value;
    constexpr bool LOADF = decltype(loadf_c)::value;
#pragma unroll
    for (int t = T0; t < T1; t++) {
      const int i = t / TN, j = t % TN;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[USE][j], fa[USE][i], acc[i][j], 0, 0, 0);  // C^T tile
      if (CSON) {  // this wave's half of the slot's elements: the wave with the other wm takes the rest
#pragma unroll
        for (int k = 0; k < EPSL / 2; k++) {
          const int el = t * EPSL + 2 * k + CS_HALF;
          cs[el / 8] += (float)fb[USE][el / 8][el % 8];
        }
      }
      if (LOADF) {
        if (t < TM) fa[USE ^ 1][t] = frag_load<BM, A_KC>(srcA, wm + t * 32, ks, lane);
        else if (t < TM + TN) fb[USE ^ 1][t - TM] = frag_load<BN, B_KC>(srcB, wn + (t - TM) * 32, ks, lane);
      }
      if (LOADS == 1) {
#pragma unroll
        for (int q = 0; q < NSA; q++)
          if (q * SLOTS_A / NSA == t + OFS) dma_a(q, k_next, buf);
      }
      if (LOADS == 2) {
#pragma unroll
        for (int q = 0; q < NSB; q++)
          if (q * SLOTS_B / NSB == t + OFS) dma_b(q, k_next, buf);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto a_buf = [&](int i) { return smem + i * LA::BYTES; };
  auto b_buf = [&](int i) { return smem + B_BASE + i * LB::BYTES; };

#pragma unroll
  for (int i = 0; i < TM; i++) fa[0][i] = frag_load<BM, A_KC>(a_buf(0), wm + i * 32, 0, lane);
#pragma unroll
  for (int j = 0; j < TN; j++) fb[0][j] = frag_load<BN, B_KC>(b_buf(0), wn + j * 32, 0, lane);
  int ia = 0;  // A buffer of the current slab: kt mod 3
  for (int kt = 0; kt < nk - 1; kt++) {
    const int ia1 = ia == 2 ? 0 : ia + 1, ia2 = ia1 == 2 ? 0 : ia1 + 1;
    const int ib = kt & 1;
    const char* curA = a_buf(ia);
    const char* curB = b_buf(ib);
    const int k_next = min(kt + 2, nk - 1) * GK;  // past the end: the last slab again, into buffers nobody reads
    phase(I<0>{}, T_{}, I<1>{}, I<0>{}, I<0>{}, I<NSLOT>{}, curA, curB, 1, k_next, ia2);
    phase(I<1>{}, T_{}, I<1>{}, I<NSLOT>{}, I<0>{}, I<NSLOT>{}, curA, curB, 2, k_next, ia2);
    phase(I<0>{}, T_{}, I<0>{}, I<0>{}, I<0>{}, I<PB>{}, curA, curB, 3, 0, 0);
    // Every fragment read of slab kt has returned (lgkmcnt) and, of this wave's loads, only the
    // NSA newest (A of slab kt+2) may still be in flight: slab kt+1 has landed.
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(NSA) : "memory");
    phase(I<0>{}, F_{}, I<2>{}, I<-PB>{}, I<PB>{}, I<NSLOT>{}, curA, curB, 3, k_next, ib);
    phase(I<1>{}, T_{}, I<2>{}, I<NSLOT - PB>{}, I<0>{}, I<NSLOT>{}, a_buf(ia1), b_buf(ib ^ 1), 0, k_next, ib);
    ia = ia1;
  }
  {
    const char* curA = a_buf(ia);
    const char* curB = b_buf((nk - 1) & 1);
    phase(I<0>{}, T_{}, I<0>{}, I<0>{}, I<0>{}, I<NSLOT>{}, curA, curB, 1, 0, 0);
    phase(I<1>{}, T_{}, I<0>{}, I<0>{}, I<0>{}, I<NSLOT>{}, curA, curB, 2, 0, 0);
    phase(I<0>{}, T_{}, I<0>{}, I<0>{}, I<0>{}, I<NSLOT>{}, curA, curB, 3, 0, 0);
    phase(I<1>{}, F_{}, I<0>{}, I<0>{}, I<0>{}, I<NSLOT>{}, curA, curB, 0, 0, 0);
  }
  };  // main_loop
  if constexpr (CS) {
    if (!cs_on) main_loop(F_{}, I<0>{});
    else if (cs_half) main_loop(T_{}, I<1>{});
    else main_loop(T_{}, I<0>{});
  } else {
    main_loop(F_{}, I<0>{});
  }
  lds_dma_wait();  // the re-requested last slab: nothing may be in flight when LDS is reused or the wave ends

  // Epilogue.  Each wave turns 32 rows of its tile at a time through LDS (fp32) and reads them
  // back row-wise, four consecutive columns per lane, so that a row of the wave tile leaves as
  // one contiguous run and bias, residual and the GELU side inputs move as 8-byte vectors.  On
  // the way in a lane writes the 16-byte units it owns (row l & 31); the 16-byte chunk index is
  // XOR-ed with (row & 7) so that neither those writes (8 lanes = 8 rows, same chunk) nor the
  // row-wise reads (8 lanes = 8 consecutive chunks) collide on LDS banks.  Reads are issued eight
  // rows ahead of the arithmetic and stores that consume them.  The staging areas are A[2] (waves
  // 0, 1) and B[1] (waves 2, 3): A[0], A[1] and B[0] are already receiving the next tile.
  constexpr int WC = TN * 32;     // columns of the wave tile
  constexpr int LPR = WC / 4;     // lanes per row on the way out
  constexpr int RPI = 64 / LPR;   // rows per store instruction
  constexpr int NIT = 32 / RPI;   // store instructions per 32 rows
  constexpr int BATCH = NIT < 8 ? NIT : 8;
  static_assert(NIT % BATCH == 0, "batching of the read-back");
  static_assert(2 * 32 * WC * 4 <= LA::BYTES && 2 * 32 * WC * 4 <= LB::BYTES, "two waves stage in one slab buffer");
  __syncthreads();                // every wave is done with the operand slabs
  float* wbuf = reinterpret_cast<float*>(smem + (wave < 2 ? 2 * LA::BYTES : B_BASE + LB::BYTES)) + (wave & 1) * 32 * WC;
  if constexpr (CS) {
    if (cs_on) {  // uniform over the workgroup
      // lanes l and l ^ 32 hold different k's of the same column; waves wm = 0 and wm != 0 different
      // elements.  Exchange through the start of the receiving wave's own staging area.
      float* xch = reinterpret_cast<float*>(smem + 2 * LA::BYTES) + (wave & 1) * 32 * WC;
#pragma unroll
      for (int j = 0; j < TN; j++) cs[j] += __shfl_xor(cs[j], 32, 64);
      if (cs_half && lane < 32) {
#pragma unroll
        for (int j = 0; j < TN; j++) xch[j * 32 + lane] = cs[j];
      }
      __syncthreads();
      if (!cs_half && lane < 32) {
#pragma unroll
        for (int j = 0; j < TN; j++) {
          const float v = cs[j] + xch[j * 32 + lane];
          float* o = et.colsum + n0 + wn + j * 32 + lane;
          *o = e.accumulate ? *o + v : v;
        }
      }
    }
  }
  // the next tile's first slabs, before anything else of the epilogue
  if (tile + (int)gridDim.x < nt * splits) {
    const int next = tile + gridDim.x;
    tile_of(next % nt, tm_i, tn_i);
    k_range(next, k_first, nk_item);
    k_begin = (size_t)k_first * GK;
    request_first_slabs(a_tile_of(tm_i) + k_begin * a_kstride, b_tile_of(tn_i) + k_begin * b_kstride, nk_item);
  }
  // (lane index through an opaque copy: otherwise everything derived from it below is hoisted out of
  // the tile loop and kept in registers across the main loop, which has none to spare)
  int lane_e = lane;
  asm volatile("" : "+v"(lane_e));
  const int c4 = (lane_e % LPR) * 4;
  const int rsub = lane_e / LPR;
  const int ncol = n0 + wn + c4;
  constexpr bool F32 = em_kind(EM) == EK_F32, DG = em_dgelu(EM);
  constexpr bool SIDE = !F32 && (DG || (EM & EM_RES));  // a bf16 side input: pre-activation U or residual R
  float4 bias = make_float4(0.f, 0.f, 0.f, 0.f);
  if (!F32 && e.bias) bias = ld_bf16x4(e.bias, ncol);
  const bf16_t* sp = (const bf16_t*)(DG ? e.U : e.R);
  const int lds_ = DG ? e.ldu : e.ldr;
  // the side input of 32 rows is requested one round ahead: the loads fly while the previous
  // rows turn through LDS
  bf16x4 side[2][SIDE ? NIT : 1];
  auto side_request = [&](int i, bf16x4 (&dst)[SIDE ? NIT : 1]) {
    if (SIDE) {
#pragma unroll
      for (int k = 0; k < NIT; k++)
        dst[k] = *reinterpret_cast<const bf16x4*>(sp + (size_t)(m0 + wm + i * 32 + rsub + k * RPI) * lds_ + ncol);
    }
  };
  side_request(0, side[0]);
#pragma unroll
  for (int i = 0; i < TM; i++) {
    const int mrow = m0 + wm + i * 32 + rsub;
    if (i + 1 < TM) side_request(i + 1, side[(i + 1) & 1]);
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const int row = lane_e & 31;
        const int chunk = j * 8 + g * 2 + (lane_e >> 5);
        const f32x16& t = acc[i][j];
        *reinterpret_cast<float4*>(wbuf + row * WC + ((chunk ^ (row & 7)) << 2)) =
            make_float4(t[g * 4], t[g * 4 + 1], t[g * 4 + 2], t[g * 4 + 3]);
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int k0 = 0; k0 < NIT; k0 += BATCH) {
      constexpr bool ADD_C = F32 && (EM & EM_RES);
      float4 a[BATCH], old_c[ADD_C ? BATCH : 1];
#pragma unroll
      for (int u = 0; u < BATCH; u++) {
        const int row = (k0 + u) * RPI + rsub;
        a[u] = *reinterpret_cast<const float4*>(wbuf + row * WC + (((c4 >> 2) ^ (row & 7)) << 2));
        if (ADD_C) old_c[u] = *reinterpret_cast<const float4*>((const float*)et.C + (size_t)(mrow + (k0 + u) * RPI) * e.ldc + ncol);
      }
#pragma unroll
      for (int u = 0; u < BATCH; u++) {
        float4 sd = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ADD_C) {
          sd = old_c[u];
        } else if (SIDE) {
          const bf16x4 v = side[i & 1][k0 + u];
          sd = make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
        }
        mfma_epilogue4<EM>(et, mrow + (k0 + u) * RPI, ncol, a[u], bias, sd);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  }  // tile loop
  lds_dma_wait();  // nothing is in flight here; stated for whoever reads the assembly in a straight line
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Tile rows per group of the tile walk (see tile_of in the kernel): the 32 tiles an XCD works on
// at a time form a block of `group` tile rows x 32 / group tile columns.  8 x 4 and 4 x 8 fetch the
// same twelve operand panels; measured inside the benchmark steps, 4 x 8 is the faster one wherever
// the output is wide enough to hold whole blocks of eight columns and the contraction is long
// (d_model 4096 block -0.8 %, the 12288-wide share -2 %, the 2048-wide model -1.2 %, the 1024-wide
// one -1.6 %), and the slower one (+0.3 to 0.5 %) for the 768-wide model with its 3 to 12 tile
// columns and K = 768, which therefore keeps 8 x 4.
// Where both tile counts are multiples of 16 (and the product is not split) the blocks of the eight
// XCDs are laid side by side as well, 4 x 2 of them to a 16 x 16 block of tiles per round (group 0;
// the launch falls back to 4 when it does not run 256 workgroups): the d_model 4096 block another
// -0.4 % (8.065 -> 8.03 ms, A-B on one box), the others unchanged.
static int walk_group(int tiles_m, int tiles_n, int K, int splits) {
  if (K < 1024 || !(tiles_n >= 16 || tiles_n % 8 == 0)) return 8;
  return (splits == 1 && tiles_m % 16 == 0 && tiles_n % 16 == 0) ? 0 : 4;
}

// Both heuristics are written for the 256 CUs of the MI355X.  No device query here on purpose:
// plans decide workspace sizes, and those are computed on hosts without a GPU too (the launch
// itself sizes its grid from the device's own CU count, see launch_mfma).
static constexpr int kCUs = 256;

// Tile classes of the kernel, largest first, and what a workgroup pays per 64-wide K slab and per
// tile (microseconds, fitted to timings of this kernel).  The slab time is given for a full chip
// (`full_us`) and falls with the share of busy CUs towards `floor_us`: with fewer CUs busy the
// clock is higher (256^2: 1.55 us with all CUs busy, 1.15 with half of them) and each gets more of
// the L2s' bandwidth, which is what bounds the 256 x 128 class on a full chip (13.7 TB/s into LDS
// over all CUs: 0.89 us a slab on 256 CUs, 0.64 on 160).  The smaller the tile, the more LDS
// fragment traffic per flop (4 + 4 fragments per 16 MFMAs at 256^2, 4 + 2 per 8 at 256 x 128,
// 2 + 2 per 4 at 128^2).
struct TileClass {
  int m, n;
  double full_us, idle_share, floor_us;  // slab time = max(floor, full * (idle_share + (1 - idle_share) * busy share))
  double epi_bf16_us, epi_f32_us;
};
static constexpr TileClass kTiles[] = {{256, 256, 1.55, 0.48, 1.10, 7.0, 8.0},
                                       {256, 128, 0.89, 0.25, 0.64, 4.0, 4.5},
                                       {128, 128, 0.66, 1.00, 0.66, 3.0, 3.0}};

// Predicted duration of one launch: workgroups run in rounds of one per CU, the last one possibly
// partly filled (a 128^2 launch of at most two per CU runs them side by side, at shared LDS
// bandwidth); folding s partial products costs a launch plus their bytes, written once and read once.
static double tile_time_us(const TileClass& tc, int M, int N, int K, bool f32_out, int s) {
  const int slabs = (K / GK + s - 1) / s;
  const long long items = (long long)(M / tc.m) * (N / tc.n) * s;
  const double epi = f32_out ? tc.epi_f32_us : tc.epi_bf16_us;
  auto round_us = [&](double busy_share) {
    return slabs * std::max(tc.floor_us, tc.full_us * (tc.idle_share + (1.0 - tc.idle_share) * busy_share)) + epi;
  };
  double t;
  if (tc.m == 128 && items > kCUs && items <= 2 * kCUs && !f32_out) {
    t = 1.6 * round_us(1.0);
  } else {
    // (weight-gradient products, both operands through the LDS transpose read, gain nothing from a
    // partly filled round: every round at the full-chip price reproduces their measured plans)
    const long long full = items / kCUs, rest = items % kCUs;
    t = full * round_us(1.0) + (rest ? round_us(f32_out ? 1.0 : (double)rest / kCUs) : 0.0);
  }
  if (s > 1) t += 10.0 + (2.0 * s + 1.0) * M * N * 4.0 / 3.0e6;
  return t;
}

// Tile class (and, when `may_split`, number of K ranges) with the smallest predicted time; a
// smaller tile or a split has to be 3 % better than what is already chosen.  tile_m = 0: no class
// divides the shape.  The 256 x 128 class is used for bf16 outputs only: on weight-gradient
// products (both operands through the LDS transpose read, with or without K ranges) it measured
// 10-50 % above this model.
static GemmSplitPlan plan_tiles(int M, int N, int K, bool f32_out, bool may_split) {
  GemmSplitPlan best{0, 0, 1};
  if (M <= 0 || N <= 0 || K <= 0 || K % GK) return best;
  const int nkt = K / GK;
  double best_t = 1e30;
  for (const TileClass& tc : kTiles) {
    if (M % tc.m || N % tc.n) continue;
    if (f32_out && tc.m != tc.n) continue;
    for (int s = 1; s <= (may_split ? 32 : 1) && (s == 1 || nkt / s >= 8); s++) {
      const double t = tile_time_us(tc, M, N, K, f32_out, s);
      if (t < best_t * 0.97) {
        best_t = t;
        best = GemmSplitPlan{tc.m, tc.n, s};
      }
    }
  }
  return best;
}

GemmSplitPlan gemm_split_plan(int M, int N, int K) { return plan_tiles(M, N, K, true, true); }

// One dimension an odd multiple of 128 and the rest big enough to fill the chip with 256^2 tiles:
// the product is computed as two, the bulk on 256^2 tiles and the last 128 rows (1) or columns (2)
// on smaller ones.
static int tail_dim(int M, int N) {
  auto fills = [](int m, int n) { return m > 0 && n > 0 && m % 256 == 0 && n % 256 == 0 && (long long)(m / 256) * (n / 256) >= 2 * kCUs; };
  if (M % 256 == 128 && fills(M - 128, N)) return 1;
  if (N % 256 == 128 && fills(M, N - 128)) return 2;
  return 0;
}

// What gemm_mfma() does with a densely stored product, for inspection from the host: the strip
// decomposition (0, or 1 / 2 = last 128 rows / columns apart) and the plan of the bulk.
GemmSplitPlan gemm_plan_query(int M, int N, int K, bool f32_out, int* tail) {
  const int td = tail_dim(M, N);
  *tail = td;
  if (td == 1) return plan_tiles(M - 128, N, K, f32_out, f32_out);
  if (td == 2) return plan_tiles(M, N - 128, K, f32_out, false);  // the strip keeps C's leading dimension: no split
  return plan_tiles(M, N, K, f32_out, f32_out);
}

// The tile walk of the main launch of a product (not of the 128-wide strip an odd multiple of 128
// leaves over), as a table: tile number -> (tile row, tile column).  For the tests.
int gemm_tile_walk_query(int M, int N, int K, bool f32_out, int* tm, int* tn, int capacity, int* count, int* group) {
  int tail = 0;
  const GemmSplitPlan plan = gemm_plan_query(M, N, K, f32_out, &tail);
  if (plan.tile_m == 0) { *count = 0; *group = -1; return 0; }
  const int tiles_m = (tail == 1 ? M - 128 : M) / plan.tile_m, tiles_n = (tail == 2 ? N - 128 : N) / plan.tile_n;
  int grp = walk_group(tiles_m, tiles_n, K, plan.splits);
  const int nt = tiles_m * tiles_n;
  const int slots = (plan.tile_m == 128 && nt * plan.splits <= 2 * kCUs) ? 2 * kCUs : kCUs;
  if (grp == 0 && (nt < slots ? nt : slots) != 256) grp = 4;  // as launch_mfma decides
  *group = grp; *count = nt;
  for (int id = 0; id < nt && id < capacity; id++) tile_walk(id, tiles_m, tiles_n, grp, tm[id], tn[id]);
  return 0;
}

// partial products, then partial column sums
static size_t split_ws_bytes_1(int M, int N, int K) {
  const int s = gemm_split_plan(M, N, K).splits;
  return s > 1 ? (size_t)s * ((size_t)M * N + N) * sizeof(float) : 0;
}

size_t gemm_split_ws_bytes(int M, int N, int K) {
  if (tail_dim(M, N) == 1) return std::max(split_ws_bytes_1(M - 128, N, K), split_ws_bytes_1(128, N, K));
  return split_ws_bytes_1(M, N, K);  // a column strip keeps the leading dimension of C: no split there
}

static double time_estimate_1(int M, int N, int K, bool f32_out) {
  const GemmSplitPlan plan = plan_tiles(M, N, K, f32_out, f32_out);
  if (plan.tile_m == 0) return 2.0 * M * N * K / 15.0e6;  // the scalar kernel: about 15 TFLOP/s
  for (const TileClass& tc : kTiles)
    if (tc.m == plan.tile_m && tc.n == plan.tile_n) return 3.0 + tile_time_us(tc, M, N, K, f32_out, plan.splits);
  return 0.0;
}

double gemm_time_estimate_us(int M, int N, int K, bool f32_out) {
  switch (tail_dim(M, N)) {
    case 1: return time_estimate_1(M - 128, N, K, f32_out) + time_estimate_1(128, N, K, f32_out);
    case 2: return time_estimate_1(M, N - 128, K, f32_out) + time_estimate_1(M, 128, K, f32_out);
  }
  return time_estimate_1(M, N, K, f32_out);
}


bool gemm_mfma_supported(const GemmArgs& g) {
  if (g.dtype != FAX_BF16) return false;
  if (g.c_f32 && (g.bias || g.R || g.C2 || g.epi != EPI_NONE)) return false;  // fp32 C is the plain weight-gradient form
  if (g.colsum && !(g.c_f32 && g.ta && !g.tb)) return false;  // the column sums of B ride only on that form, A [K, M], B [K, N]
  // the GELU epilogues exist for the orientations the block uses them in: forward (A [M,K], B [K,N])
  // and input-gradient (A [M,K], B [N,K])
  if (g.epi == EPI_GELU && (g.ta || g.tb || g.R)) return false;
  if (g.epi == EPI_DGELU && (g.ta || !g.tb || g.R)) return false;
  // the second output likewise: forward orientation only
  if (g.epi == EPI_NONE && g.C2 && (g.ta || g.tb)) return false;
  if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.K % GK != 0) return false;
  if (g.lda % 8 || g.ldb % 8 || !aligned16(g.A) || !aligned16(g.B)) return false;
  if (g.c_f32) {  // the epilogue moves four columns at a time: 16-byte fp32 units ...
    if (g.ldc % 4 || !aligned16(g.C)) return false;
  } else {        // ... or 8-byte bf16 units
    auto vec_ok = [](const void* p, int ld) { return !p || (ld % 4 == 0 && (reinterpret_cast<uintptr_t>(p) & 7) == 0); };
    if (!vec_ok(g.C, g.ldc) || !vec_ok(g.C2, g.ldc2) || !vec_ok(g.R, g.ldr) || !vec_ok(g.U, g.ldu) || !vec_ok(g.bias, 4))
      return false;
  }
  return g.M % 128 == 0 && g.N % 128 == 0;  // the smallest tile class
}

template <int BM, int BN, bool A_KC, bool B_KC, int EM>
static int launch_mfma(const GemmArgs& g, const EpiArgs& e, hipStream_t s) {
  constexpr size_t lds = 3 * (size_t)TileLds<BM, A_KC>::BYTES + 2 * (size_t)TileLds<BN, B_KC>::BYTES;  // 160 KB at 256^2; also covers the epilogue's staging
  auto kern = gemm_mfma_kernel<BM, BN, A_KC, B_KC, EM>;
  static bool configured = false;  // benign race: the attribute is idempotent
  if (!configured) {
    FAX_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    configured = true;
  }
  const int tiles_m = g.M / BM, tiles_n = g.N / BN;
  static int n_cu = 0;  // benign race: same value from every thread
  if (n_cu == 0) {
    int dev = 0, v = 0;
    FAX_HIP(hipGetDevice(&dev));
    FAX_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
    n_cu = v > 0 ? v : 256;
  }
  const int items = tiles_m * tiles_n * (e.splits > 1 ? e.splits : 1);
  // Persistent: one workgroup per CU.  A 128^2 workgroup needs 80 KB of LDS and under 256 registers,
  // so two fit on a CU; they share its LDS bandwidth, which bounds that kernel, and gain little
  // (measured: +-0.4 % with many tiles) except when that saves a second round for a few left-over
  // tiles (320 tiles: -4 % on the whole step).
  const int slots = (BM == 128 && items <= 2 * n_cu) ? 2 * n_cu : n_cu;
  const int grid = items < slots ? items : slots;
  EpiArgs ek = e;
  if (ek.group == 0 && grid != 256) ek.group = 4;  // the side-by-side walk is written for 8 XCDs x 32 workgroups
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, g.M, g.N, g.K, (const bf16_t*)g.A, g.lda,
                     (const bf16_t*)g.B, g.ldb, ek, tiles_m, tiles_n);
  FAX_LAUNCH_CHECK("gemm_mfma");
  return FAX_OK;
}

template <int BM, int BN>
static int dispatch(const GemmArgs& g, const EpiArgs& e, hipStream_t s) {
  const bool a_kc = !g.ta, b_kc = g.tb;
  const bool erf = g.gelu_form == FAX_GELU_ERF;
  if (g.epi == EPI_GELU)
    return erf ? launch_mfma<BM, BN, true, false, EK_GELU_ERF>(g, e, s) : launch_mfma<BM, BN, true, false, EK_GELU_TANH>(g, e, s);
  if (g.epi == EPI_DGELU)
    return launch_mfma<BM, BN, true, true, EK_DGELU>(g, e, s);
  if (g.c_f32 && g.colsum)
    return g.accumulate ? launch_mfma<BM, BN, false, false, EK_F32 | EM_RES | EM_COLSUM>(g, e, s)
                        : launch_mfma<BM, BN, false, false, EK_F32 | EM_COLSUM>(g, e, s);
  if (g.c_f32) {
    if (g.accumulate) {
      if (a_kc && b_kc) return launch_mfma<BM, BN, true, true, EK_F32 | EM_RES>(g, e, s);
      if (a_kc && !b_kc) return launch_mfma<BM, BN, true, false, EK_F32 | EM_RES>(g, e, s);
      if (!a_kc && b_kc) return launch_mfma<BM, BN, false, true, EK_F32 | EM_RES>(g, e, s);
      return launch_mfma<BM, BN, false, false, EK_F32 | EM_RES>(g, e, s);
    }
    if (a_kc && b_kc) return launch_mfma<BM, BN, true, true, EK_F32>(g, e, s);
    if (a_kc && !b_kc) return launch_mfma<BM, BN, true, false, EK_F32>(g, e, s);
    if (!a_kc && b_kc) return launch_mfma<BM, BN, false, true, EK_F32>(g, e, s);
    return launch_mfma<BM, BN, false, false, EK_F32>(g, e, s);
  }
  if (g.C2)  // forward orientation (checked by gemm_mfma_supported)
    return g.R ? launch_mfma<BM, BN, true, false, EK_STORE | EM_RES | EM_C2>(g, e, s)
               : launch_mfma<BM, BN, true, false, EK_STORE | EM_C2>(g, e, s);
  if (g.R) {
    if (a_kc && b_kc) return launch_mfma<BM, BN, true, true, EK_STORE | EM_RES>(g, e, s);
    if (a_kc && !b_kc) return launch_mfma<BM, BN, true, false, EK_STORE | EM_RES>(g, e, s);
    if (!a_kc && b_kc) return launch_mfma<BM, BN, false, true, EK_STORE | EM_RES>(g, e, s);
    return launch_mfma<BM, BN, false, false, EK_STORE | EM_RES>(g, e, s);
  }
  if (a_kc && b_kc) return launch_mfma<BM, BN, true, true, EK_STORE>(g, e, s);
  if (a_kc && !b_kc) return launch_mfma<BM, BN, true, false, EK_STORE>(g, e, s);
  if (!a_kc && b_kc) return launch_mfma<BM, BN, false, true, EK_STORE>(g, e, s);
  return launch_mfma<BM, BN, false, false, EK_STORE>(g, e, s);
}

static const void* offset(const void* p, size_t elements, size_t elem_bytes) {
  return p ? (const char*)p + elements * elem_bytes : nullptr;
}
static void* offset(void* p, size_t elements, size_t elem_bytes) { return p ? (char*)p + elements * elem_bytes : nullptr; }

int gemm_mfma(const GemmArgs& g0, hipStream_t s) {
  if (const int td = tail_dim(g0.M, g0.N)) {
    const size_t cb = g0.c_f32 ? 4 : 2;
    for (int part = 0; part < 2; part++) {
      GemmArgs h = g0;
      if (td == 1) {  // rows [m0, m0 + M')
        const size_t m0 = part ? g0.M - 128 : 0;
        h.M = part ? 128 : g0.M - 128;
        h.A = offset(g0.A, g0.ta ? m0 : m0 * g0.lda, 2);
        h.C = offset(g0.C, m0 * g0.ldc, cb);
        h.R = offset(g0.R, m0 * g0.ldr, 2);
        h.C2 = offset(g0.C2, m0 * g0.ldc2, 2);
        h.U = offset(g0.U, m0 * g0.ldu, 2);
        if (part) h.colsum = nullptr;  // the column sums of B are complete after the first product
      } else {        // columns [n0, n0 + N')
        const size_t n0 = part ? g0.N - 128 : 0;
        h.N = part ? 128 : g0.N - 128;
        h.B = offset(g0.B, g0.tb ? n0 * g0.ldb : n0, 2);
        h.C = offset(g0.C, n0, cb);
        h.bias = offset(g0.bias, n0, 2);
        h.R = offset(g0.R, n0, 2);
        h.C2 = offset(g0.C2, n0, 2);
        h.U = offset(g0.U, n0, 2);
        if (g0.colsum) h.colsum = g0.colsum + n0;
      }
      FAX_TRY(gemm_mfma(h, s));  // (neither part has a tail of its own)
    }
    return FAX_OK;
  }
  GemmArgs g = g0;
  // Split the contraction?  Only the fp32-output form, with scratch from the caller and C stored
  // densely; the partial products (and partial column sums) are then folded in a fixed order.
  const GemmSplitPlan plan = plan_tiles(g.M, g.N, g.K, g.c_f32, g.c_f32 && g.split_ws && g.ldc == g.N);
  if (plan.tile_m == 0) {
    set_error("gemm_mfma: %d x %d x %d fits no tile class", g.M, g.N, g.K);
    return FAX_ERR_UNSUPPORTED;
  }
  const int splits = plan.splits;
  const size_t mn = (size_t)g.M * g.N;
  float* const part_c = (float*)g.split_ws;
  float* const part_cs = part_c + (size_t)splits * mn;
  if (splits > 1) {
    g.C = part_c;
    if (g.colsum) g.colsum = part_cs;
    g.accumulate = false;
  }
  EpiArgs e{g.bias, g.R, g.ldr, g.C, g.ldc, g.C2, g.ldc2, g.U, g.ldu, g.epi, g.gelu_form, g.c_f32 ? 1 : 0,
            g.accumulate ? 1 : 0, g.colsum, splits, mn, (size_t)g.N,
            walk_group(g.M / plan.tile_m, g.N / plan.tile_n, g.K, splits)};
  if (plan.tile_n == 256) FAX_TRY((dispatch<256, 256>(g, e, s)));
  else if (plan.tile_m == 256) FAX_TRY((dispatch<256, 128>(g, e, s)));
  else FAX_TRY((dispatch<128, 128>(g, e, s)));
  if (splits > 1) {
    FAX_TRY(fold_partials(splits, mn, part_c, (float*)g0.C, g0.accumulate, s, g0.colsum ? g.N : 0, part_cs, g0.colsum));
  }
  return FAX_OK;
}

}  // namespace fax
