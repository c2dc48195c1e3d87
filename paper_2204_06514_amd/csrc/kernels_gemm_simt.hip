// Scalar-FMA GEMM: true fp32 multiply-add for the fp32 workloads, and the fallback for bf16
// shapes that the MFMA kernel's tiles do not divide.  Any M, N, K, any operand orientation.
// 64x64x16 tile, 256 threads, 4x4 outputs per thread, operands staged through LDS as fp32.
#include <cstdio>

#include "fax_internal.h"

namespace fax {

template <typename T, bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_simt_kernel(int M, int N, int K, const T* __restrict__ A, int lda,
                                                        const T* __restrict__ B, int ldb, EpiArgs e) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int id = tid + i * 256;
      int m, k;
      if (TA) { m = id % 64; k = id / 64; } else { k = id % 16; m = id / 16; }
      const int gm = m0 + m, gk = k0 + k;
      float v = 0.f;
      if (gm < M && gk < K) v = to_f(TA ? A[(size_t)gk * lda + gm] : A[(size_t)gm * lda + gk]);
      As[k][m] = v;
      int n, kb;
      if (TB) { kb = id % 16; n = id / 16; } else { n = id % 64; kb = id / 64; }
      const int gn = n0 + n, gkb = k0 + kb;
      float w = 0.f;
      if (gn < N && gkb < K) w = to_f(TB ? B[(size_t)gn * ldb + gkb] : B[(size_t)gkb * ldb + gn]);
      Bs[kb][n] = w;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; k++) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; j++) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int n = n0 + tx * 4 + j;
      if (n < N) epilogue_store<T>(e, m, n, acc[i][j]);
    }
  }
}

template <typename T>
static int gemm_simt_t(const GemmArgs& g, hipStream_t s) {
  EpiArgs e{g.bias, g.R, g.ldr, g.C, g.ldc, g.C2, g.ldc2, g.U, g.ldu, g.epi, g.gelu_form, g.c_f32 ? 1 : 0,
            g.accumulate ? 1 : 0};
  dim3 grid((g.N + 63) / 64, (g.M + 63) / 64), block(256);
  const T* A = (const T*)g.A;
  const T* B = (const T*)g.B;
  if (!g.ta && !g.tb)
    hipLaunchKernelGGL((gemm_simt_kernel<T, false, false>), grid, block, 0, s, g.M, g.N, g.K, A, g.lda, B, g.ldb, e);
  else if (!g.ta && g.tb)
    hipLaunchKernelGGL((gemm_simt_kernel<T, false, true>), grid, block, 0, s, g.M, g.N, g.K, A, g.lda, B, g.ldb, e);
  else if (g.ta && !g.tb)
    hipLaunchKernelGGL((gemm_simt_kernel<T, true, false>), grid, block, 0, s, g.M, g.N, g.K, A, g.lda, B, g.ldb, e);
  else
    hipLaunchKernelGGL((gemm_simt_kernel<T, true, true>), grid, block, 0, s, g.M, g.N, g.K, A, g.lda, B, g.ldb, e);
  FAX_LAUNCH_CHECK("gemm_simt");
  return FAX_OK;
}

int gemm_simt(const GemmArgs& g, hipStream_t s) {
  if (g.M == 0 || g.N == 0) return FAX_OK;
  if (g.dtype == FAX_F32) return gemm_simt_t<float>(g, s);
  return gemm_simt_t<bf16_t>(g, s);
}

static int gemm_dispatch(const GemmArgs& g, hipStream_t s);

int gemm(const GemmArgs& g, hipStream_t s) {
  if (!timing_on()) return gemm_dispatch(g, s);
  // name the variant the way the kernel templates are instantiated: operand orientation
  // (k = contraction index contiguous, m = row/column index contiguous) and epilogue
  const bool mfma = g.path != PATH_SIMT && gemm_mfma_supported(g);
  char name[64];
  snprintf(name, sizeof(name), "gemm_%s_A%c_B%c_%s", mfma ? "mfma" : "scalar", g.ta ? 'm' : 'k', g.tb ? 'k' : 'm',
           g.c_f32 ? "f32out" : g.epi == EPI_GELU ? "gelu" : g.epi == EPI_DGELU ? "dgelu" : "store");
  Timed t(name, WORK_FLOP, 2.0 * g.M * g.N * g.K, s);
  return gemm_dispatch(g, s);
}

static int gemm_dispatch(const GemmArgs& g, hipStream_t s) {
  const bool mfma = g.path != PATH_SIMT && gemm_mfma_supported(g);
  if (g.path == PATH_MFMA && !mfma) {
    set_error("fax_gemm: shape M=%d N=%d K=%d (dtype %d) does not tile for the MFMA kernel", g.M, g.N, g.K, g.dtype);
    return FAX_ERR_UNSUPPORTED;
  }
  if (mfma) {
    return gemm_mfma(g, s);
  }
  if (g.colsum) {
    // no fused form here: take the column sums of B [K, N] in a pass of their own
    if (g.tb || !g.colsum_ws) {
      set_error("gemm: column sums need B stored [K, N] and scratch space");
      return FAX_ERR_INVALID_ARG;
    }
    FAX_TRY(colsum(g.dtype, g.K, g.N, g.B, g.ldb, g.colsum, g.accumulate, g.colsum_ws, s));
  }
  return gemm_simt(g, s);
}

}  // namespace fax
