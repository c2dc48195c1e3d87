// bf16 GEMM on the CDNA4 matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulate.
//
// One 256-thread workgroup (4 wavefronts, 2x2) computes a BM x BN tile of C, stepping over K in
// slabs of 64.  Each slab of A and of B is staged through LDS, double buffered: global loads of
// slab k+1 are issued before the MFMAs of slab k and parked in registers meanwhile.
//
// An operand whose contraction index is contiguous in memory ("KC": A stored [M,K], B stored
// [N,K]) is kept in LDS as [row][64] with the 16-byte chunk index XOR-ed with (row & 7), so
// that the 128-bit fragment reads of 8 consecutive rows fall in 8 different bank groups.
// An operand whose M/N index is contiguous ("MC": A stored [K,M], B stored [K,N]) is kept as
// [k][rows + 16] and fetched with ds_read_b64_tr_b16, the LDS transpose read: 16 lanes pick up
// four k-rows x 16 columns and each lane receives 4 consecutive k for its own column; two such
// reads make one MFMA operand.  The 32-byte row padding spreads the four k-rows over all banks.
//
// MFMA 32x32x16 lane layout (lane l): A/B operand = row/column (l & 31), k = 8 (l >> 5) + 0..7;
// accumulator v = 0..15 holds C[8 (v >> 2) + 4 (l >> 5) + (v & 3)][l & 31].
#include "fax_internal.h"

namespace fax {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static constexpr int GK = 64;  // K slab

template <int ROWS, bool KC>
struct TileLds {
  static constexpr int STRIDE_MC = (ROWS + 16) * 2;  // bytes per k-row, MC layout
  static constexpr int BYTES = KC ? ROWS * 128 : GK * STRIDE_MC;
  static constexpr int NCHUNK = ROWS * GK / 8 / 256;  // 16-byte chunks per thread per slab
};

// Global -> registers for one slab of one operand.
template <int ROWS, bool KC>
__device__ __forceinline__ void slab_load(uint4 (&r)[ROWS * GK / 8 / 256], const bf16_t* __restrict__ P, int ld,
                                          int row0, int k0) {
#pragma unroll
  for (int i = 0; i < TileLds<ROWS, KC>::NCHUNK; i++) {
    const int id = threadIdx.x + i * 256;
    if (KC) {
      const int row = id >> 3, c = id & 7;
      r[i] = *reinterpret_cast<const uint4*>(P + (size_t)(row0 + row) * ld + k0 + c * 8);
    } else {
      constexpr int CPR = ROWS / 8;
      const int kr = id / CPR, c = id % CPR;
      r[i] = *reinterpret_cast<const uint4*>(P + (size_t)(k0 + kr) * ld + row0 + c * 8);
    }
  }
}

// Registers -> LDS.
template <int ROWS, bool KC>
__device__ __forceinline__ void slab_store(const uint4 (&r)[ROWS * GK / 8 / 256], char* lds) {
#pragma unroll
  for (int i = 0; i < TileLds<ROWS, KC>::NCHUNK; i++) {
    const int id = threadIdx.x + i * 256;
    if (KC) {
      const int row = id >> 3, c = id & 7;
      *reinterpret_cast<uint4*>(lds + row * 128 + ((c ^ (row & 7)) << 4)) = r[i];
    } else {
      constexpr int CPR = ROWS / 8;
      const int kr = id / CPR, c = id % CPR;
      *reinterpret_cast<uint4*>(lds + kr * TileLds<ROWS, KC>::STRIDE_MC + c * 16) = r[i];
    }
  }
}

// One MFMA operand (8 bf16 per lane) for the 32 rows starting at rb, k-step ks (16 wide).
template <int ROWS, bool KC>
__device__ __forceinline__ bf16x8 frag_load(const char* lds, int rb, int ks, int lane) {
  if (KC) {
    const int row = rb + (lane & 31);
    const int chunk = ks * 2 + (lane >> 5);
    const uint4 v = *reinterpret_cast<const uint4*>(lds + row * 128 + ((chunk ^ (row & 7)) << 4));
    return __builtin_bit_cast(bf16x8, v);
  } else {
    const int blk = lane >> 4, i = lane & 15;
    const int kr = ks * 16 + (blk >> 1) * 8 + (i >> 2);
    const int col = rb + (blk & 1) * 16 + (i & 3) * 4;
    const char* p = lds + kr * TileLds<ROWS, KC>::STRIDE_MC + col * 2;
    typedef __attribute__((address_space(3))) short4v lds_s4;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(p));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(p + 4 * TileLds<ROWS, KC>::STRIDE_MC));
    const short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

// Epilogue flavours, fixed at compile time so the 16 x TM x TN stores unroll into straight code.
enum { EM_STORE = 0, EM_GELU_TANH = 1, EM_DGELU_TANH = 2, EM_F32 = 3, EM_GELU_ERF = 4, EM_DGELU_ERF = 5 };

// tanh-form GELU through the logistic function: (1 + tanh z) / 2 = 1 / (1 + exp(-2 z)), one
// v_exp_f32 and one v_rcp_f32 per element, a few ulp in fp32 (the outputs are rounded to bf16).
__device__ __forceinline__ float sigmoid2z(float u) {
  const float z2 = 1.5957691216057308f * (u + 0.044715f * u * u * u);  // 2 sqrt(2/pi) (u + k u^3)
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z2));
}
__device__ __forceinline__ float gelu_tanh_fast(float u) { return u * sigmoid2z(u); }
__device__ __forceinline__ float gelu_tanh_grad_fast(float u) {
  const float sg = sigmoid2z(u);
  return sg + u * sg * (1.f - sg) * 1.5957691216057308f * (1.f + 0.134145f * u * u);
}

template <int EM>
__device__ __forceinline__ void mfma_epilogue(const EpiArgs& e, int m, int n, float acc) {
  if (EM == EM_F32) {
    float* c = (float*)e.C + (size_t)m * e.ldc + n;
    *c = e.accumulate ? *c + acc : acc;
    return;
  }
  if (EM == EM_STORE && e.C2) ((bf16_t*)e.C2)[(size_t)m * e.ldc2 + n] = (bf16_t)acc;
  if (e.bias) acc += (float)((const bf16_t*)e.bias)[n];
  if (e.R) acc += (float)((const bf16_t*)e.R)[(size_t)m * e.ldr + n];
  if (EM == EM_GELU_TANH || EM == EM_GELU_ERF) {
    ((bf16_t*)e.C)[(size_t)m * e.ldc + n] = (bf16_t)acc;
    const float a = EM == EM_GELU_TANH ? gelu_tanh_fast(acc) : gelu_f(acc, FAX_GELU_ERF);
    ((bf16_t*)e.C2)[(size_t)m * e.ldc2 + n] = (bf16_t)a;
    return;
  }
  if (EM == EM_DGELU_TANH || EM == EM_DGELU_ERF) {
    const float u = (float)((const bf16_t*)e.U)[(size_t)m * e.ldu + n];
    acc *= EM == EM_DGELU_TANH ? gelu_tanh_grad_fast(u) : gelu_grad_f(u, FAX_GELU_ERF);
  }
  ((bf16_t*)e.C)[(size_t)m * e.ldc + n] = (bf16_t)acc;
}

template <int BM, int BN, bool A_KC, bool B_KC, int EM>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(int M, int N, int K, const bf16_t* __restrict__ A, int lda,
                                                        const bf16_t* __restrict__ B, int ldb, EpiArgs e, int tiles_m,
                                                        int tiles_n) {
  using LA = TileLds<BM, A_KC>;
  using LB = TileLds<BN, B_KC>;
  constexpr int TM = BM / 64, TN = BN / 64;  // 32x32 MFMA tiles per wave in each direction
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int STAGE = LA::BYTES + LB::BYTES;  // [A slab | B slab] per buffer, two buffers

  // Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 of them, each with
  // its own L2), so id is first re-dealt so that each XCD owns a contiguous run of tiles, then
  // tiles are walked in column-major groups of 8 tile-rows to keep the working set of A and B
  // panels small.
  int id = blockIdx.x;
  const int nt = tiles_m * tiles_n;
  if (nt % 8 == 0) id = (id % 8) * (nt / 8) + id / 8;
  constexpr int GROUP = 8;
  const int per_group = GROUP * tiles_n;
  const int g = id / per_group;
  const int gm0 = g * GROUP;
  const int gsz = min(GROUP, tiles_m - gm0);
  const int tm_i = gm0 + (id % per_group) % gsz;
  const int tn_i = (id % per_group) / gsz;
  const int m0 = tm_i * BM, n0 = tn_i * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  uint4 ra[LA::NCHUNK], rb[LB::NCHUNK];
  slab_load<BM, A_KC>(ra, A, lda, m0, 0);
  slab_load<BN, B_KC>(rb, B, ldb, n0, 0);
  slab_store<BM, A_KC>(ra, smem);
  slab_store<BN, B_KC>(rb, smem + LA::BYTES);
  __syncthreads();

  auto compute = [&](const char* curA, const char* curB) {
#pragma unroll
    for (int ks = 0; ks < GK / 16; ks++) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; i++) fa[i] = frag_load<BM, A_KC>(curA, wm + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < TN; j++) fb[j] = frag_load<BN, B_KC>(curB, wn + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };

  const int nk = K / GK;
  for (int kt = 0; kt < nk - 1; kt++) {
    const char* curA = smem + (kt & 1) * STAGE;
    char* nxtA = smem + ((kt + 1) & 1) * STAGE;
    slab_load<BM, A_KC>(ra, A, lda, m0, (kt + 1) * GK);
    slab_load<BN, B_KC>(rb, B, ldb, n0, (kt + 1) * GK);
    compute(curA, curA + LA::BYTES);
    slab_store<BM, A_KC>(ra, nxtA);
    slab_store<BN, B_KC>(rb, nxtA + LA::BYTES);
    __syncthreads();
  }
  {
    const char* curA = smem + ((nk - 1) & 1) * STAGE;
    compute(curA, curA + LA::BYTES);
  }

#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++) {
      const int n = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int m = m0 + wm + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        mfma_epilogue<EM>(e, m, n, acc[i][j][v]);
      }
    }
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

static int pick_tile(const GemmArgs& g) {
  if (g.M % 256 == 0 && g.N % 256 == 0 && (size_t)(g.M / 256) * (g.N / 256) >= 128) return 256;
  if (g.M % 128 == 0 && g.N % 128 == 0) return 128;
  return 0;
}

bool gemm_mfma_supported(const GemmArgs& g) {
  if (g.dtype != FAX_BF16) return false;
  if (g.c_f32 && (g.bias || g.R || g.C2 || g.epi != EPI_NONE)) return false;  // fp32 C is the plain weight-gradient form
  // the GELU epilogues exist for the orientations the block uses them in: forward (A [M,K], B [K,N])
  // and input-gradient (A [M,K], B [N,K])
  if (g.epi == EPI_GELU && (g.ta || g.tb)) return false;
  if (g.epi == EPI_DGELU && (g.ta || !g.tb)) return false;
  if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.K % GK != 0) return false;
  if (g.lda % 8 || g.ldb % 8 || !aligned16(g.A) || !aligned16(g.B)) return false;
  return pick_tile(g) != 0;
}

template <int BT, bool A_KC, bool B_KC, int EM>
static int launch_mfma(const GemmArgs& g, const EpiArgs& e, hipStream_t s) {
  constexpr size_t lds = 2 * (size_t)(TileLds<BT, A_KC>::BYTES + TileLds<BT, B_KC>::BYTES);
  auto kern = gemm_mfma_kernel<BT, BT, A_KC, B_KC, EM>;
  static bool configured = false;  // benign race: the attribute is idempotent
  if (!configured) {
    FAX_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    configured = true;
  }
  const int tiles_m = g.M / BT, tiles_n = g.N / BT;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), lds, s, g.M, g.N, g.K, (const bf16_t*)g.A, g.lda,
                     (const bf16_t*)g.B, g.ldb, e, tiles_m, tiles_n);
  FAX_LAUNCH_CHECK("gemm_mfma");
  return FAX_OK;
}

template <int BT>
static int dispatch(const GemmArgs& g, const EpiArgs& e, hipStream_t s) {
  const bool a_kc = !g.ta, b_kc = g.tb;
  const bool erf = g.gelu_form == FAX_GELU_ERF;
  if (g.epi == EPI_GELU)
    return erf ? launch_mfma<BT, true, false, EM_GELU_ERF>(g, e, s) : launch_mfma<BT, true, false, EM_GELU_TANH>(g, e, s);
  if (g.epi == EPI_DGELU)
    return erf ? launch_mfma<BT, true, true, EM_DGELU_ERF>(g, e, s) : launch_mfma<BT, true, true, EM_DGELU_TANH>(g, e, s);
  if (g.c_f32) {
    if (a_kc && b_kc) return launch_mfma<BT, true, true, EM_F32>(g, e, s);
    if (a_kc && !b_kc) return launch_mfma<BT, true, false, EM_F32>(g, e, s);
    if (!a_kc && b_kc) return launch_mfma<BT, false, true, EM_F32>(g, e, s);
    return launch_mfma<BT, false, false, EM_F32>(g, e, s);
  }
  if (a_kc && b_kc) return launch_mfma<BT, true, true, EM_STORE>(g, e, s);
  if (a_kc && !b_kc) return launch_mfma<BT, true, false, EM_STORE>(g, e, s);
  if (!a_kc && b_kc) return launch_mfma<BT, false, true, EM_STORE>(g, e, s);
  return launch_mfma<BT, false, false, EM_STORE>(g, e, s);
}

int gemm_mfma(const GemmArgs& g, hipStream_t s) {
  EpiArgs e{g.bias, g.R, g.ldr, g.C, g.ldc, g.C2, g.ldc2, g.U, g.ldu, g.epi, g.gelu_form, g.c_f32 ? 1 : 0,
            g.accumulate ? 1 : 0};
  if (pick_tile(g) == 256) return dispatch<256>(g, e, s);
  return dispatch<128>(g, e, s);
}

}  // namespace fax
