// LayerNorm forward/backward and column sums: HBM-bound kernels.
//
// Forward reads each row once (16-byte loads, row cached in registers), writes it once.
// Backward reads dh and x once, writes dx once; the per-column sums for dgamma/dbeta are
// kept in registers across a strip of rows, written as one partial row per block and
// folded by a second small kernel, so the result does not depend on scheduling order.
#include "fax_internal.h"

namespace fax {

static constexpr int LN_MAXV = 8;      // 16-byte vectors cached per thread
static constexpr int LN_THREADS = 256;
static constexpr int RED_PARTS = 512;  // partial rows produced by strip kernels

// Sum `v` over the TPR consecutive threads that share a row.  TPR in {64,128,256}.
template <int TPR>
__device__ __forceinline__ float row_sum(float v, float* red /* [LN_THREADS/64] */) {
  v = wave_sum(v);
  if (TPR == 64) return v;
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  constexpr int WPR = TPR / 64;
  const int w0 = (wave / WPR) * WPR;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < WPR; i++) s += red[w0 + i];
  return s;
}

template <typename T, int TPR>
__global__ __launch_bounds__(LN_THREADS) void ln_fwd_kernel(int rows, int D, const T* __restrict__ x,
                                                            const T* __restrict__ gamma,
                                                            const T* __restrict__ beta, float eps,
                                                            T* __restrict__ h, float* __restrict__ mu_out,
                                                            float* __restrict__ rstd_out) {
  using V = Vec16<T>;
  __shared__ float red[LN_THREADS / 64];
  constexpr int RPB = LN_THREADS / TPR;
  const int tr = threadIdx.x % TPR;
  const int row = blockIdx.x * RPB + threadIdx.x / TPR;
  const bool live = row < rows;
  const int nvec = D / V::N;
  V xv[LN_MAXV];
  float s = 0.f;
  const T* xr = x + (size_t)(live ? row : 0) * D;
#pragma unroll
  for (int i = 0; i < LN_MAXV; i++) {
    int c = tr + i * TPR;
    if (c < nvec) {
      xv[i].load(xr + c * V::N);
#pragma unroll
      for (int e = 0; e < V::N; e++) s += xv[i].get(e);
    }
  }
  const float mean = row_sum<TPR>(s, red) / D;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXV; i++) {
    int c = tr + i * TPR;
    if (c < nvec) {
#pragma unroll
      for (int e = 0; e < V::N; e++) {
        float d = xv[i].get(e) - mean;
        q += d * d;
      }
    }
  }
  const float var = row_sum<TPR>(q, red) / D;
  const float r = rsqrtf(var + eps);
  if (!live) return;
  if (tr == 0) {
    mu_out[row] = mean;
    rstd_out[row] = r;
  }
  T* hr = h + (size_t)row * D;
#pragma unroll
  for (int i = 0; i < LN_MAXV; i++) {
    int c = tr + i * TPR;
    if (c < nvec) {
      V g, b, o;
      g.load(gamma + c * V::N);
      b.load(beta + c * V::N);
#pragma unroll
      for (int e = 0; e < V::N; e++) o.set(e, (xv[i].get(e) - mean) * r * g.get(e) + b.get(e));
      o.store(hr + c * V::N);
    }
  }
}

// Any D: one wave per row, three passes over the row (the re-reads hit cache).
template <typename T>
__global__ __launch_bounds__(LN_THREADS) void ln_fwd_generic_kernel(int rows, int D, const T* __restrict__ x,
                                                                    const T* __restrict__ gamma,
                                                                    const T* __restrict__ beta, float eps,
                                                                    T* __restrict__ h, float* __restrict__ mu_out,
                                                                    float* __restrict__ rstd_out) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (LN_THREADS / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* xr = x + (size_t)row * D;
  float s = 0.f;
  for (int c = lane; c < D; c += 64) s += to_f(xr[c]);
  const float mean = wave_sum(s) / D;
  float q = 0.f;
  for (int c = lane; c < D; c += 64) {
    float d = to_f(xr[c]) - mean;
    q += d * d;
  }
  const float r = rsqrtf(wave_sum(q) / D + eps);
  if (lane == 0) {
    mu_out[row] = mean;
    rstd_out[row] = r;
  }
  T* hr = h + (size_t)row * D;
  for (int c = lane; c < D; c += 64) hr[c] = from_f<T>((to_f(xr[c]) - mean) * r * to_f(gamma[c]) + to_f(beta[c]));
}

template <typename T>
static int ln_fwd_t(int rows, int D, const T* x, const T* gamma, const T* beta, float eps, T* h, float* mu,
                    float* rstd, hipStream_t s) {
  constexpr int VN = Vec16<T>::N;
  const int nvec = D / VN;
  if (D % VN == 0 && nvec <= 256 * LN_MAXV) {
    if (nvec <= 64 * LN_MAXV / 2) {
      hipLaunchKernelGGL((ln_fwd_kernel<T, 64>), dim3((rows + 3) / 4), dim3(LN_THREADS), 0, s, rows, D, x, gamma, beta,
                         eps, h, mu, rstd);
    } else if (nvec <= 128 * LN_MAXV / 2) {
      hipLaunchKernelGGL((ln_fwd_kernel<T, 128>), dim3((rows + 1) / 2), dim3(LN_THREADS), 0, s, rows, D, x, gamma, beta,
                         eps, h, mu, rstd);
    } else {
      hipLaunchKernelGGL((ln_fwd_kernel<T, 256>), dim3(rows), dim3(LN_THREADS), 0, s, rows, D, x, gamma, beta, eps, h, mu,
                         rstd);
    }
  } else {
    hipLaunchKernelGGL((ln_fwd_generic_kernel<T>), dim3((rows + 3) / 4), dim3(LN_THREADS), 0, s, rows, D, x, gamma, beta,
                       eps, h, mu, rstd);
  }
  FAX_LAUNCH_CHECK("ln_fwd");
  return FAX_OK;
}

int ln_fwd(int dtype, int rows, int D, const void* x, const void* gamma, const void* beta, float eps, void* h,
           float* mu, float* rstd, hipStream_t s) {
  if (rows == 0) return FAX_OK;
  Timed t_("layernorm_fwd", WORK_BYTE, 2.0 * rows * D * (dtype == FAX_F32 ? 4.0 : 2.0) + 8.0 * rows, s);
  if (dtype == FAX_F32)
    return ln_fwd_t<float>(rows, D, (const float*)x, (const float*)gamma, (const float*)beta, eps, (float*)h, mu, rstd, s);
  return ln_fwd_t<bf16_t>(rows, D, (const bf16_t*)x, (const bf16_t*)gamma, (const bf16_t*)beta, eps, (bf16_t*)h, mu, rstd, s);
}

// ---------------------------------------------------------------------------------------------
// Backward.  Block b handles rows b*RPB + k*gridDim.x*RPB ...; each thread owns the same
// columns in every row, so dgamma/dbeta partials stay in registers.
// partial layout: [gridDim.x * RPB][2][D] fp32 (dgamma then dbeta).
// ---------------------------------------------------------------------------------------------
template <typename T, int TPR>
__global__ __launch_bounds__(LN_THREADS) void ln_bwd_kernel(int rows, int D, const T* __restrict__ dh,
                                                            const T* __restrict__ x, const float* __restrict__ mu,
                                                            const float* __restrict__ rstd,
                                                            const T* __restrict__ gamma, const T* __restrict__ dres,
                                                            T* __restrict__ dx, float* __restrict__ partial) {
  using V = Vec16<T>;
  __shared__ float red[LN_THREADS / 64];
  constexpr int RPB = LN_THREADS / TPR;
  const int tr = threadIdx.x % TPR;
  const int sub = threadIdx.x / TPR;
  const int nvec = D / V::N;
  float ag[LN_MAXV][V::N], ab[LN_MAXV][V::N];
  V gv[LN_MAXV];
#pragma unroll
  for (int i = 0; i < LN_MAXV; i++) {
    int c = tr + i * TPR;
    if (c < nvec) gv[i].load(gamma + c * V::N);
#pragma unroll
    for (int e = 0; e < V::N; e++) ag[i][e] = ab[i][e] = 0.f;
  }
  const int iters = (rows + gridDim.x * RPB - 1) / (gridDim.x * RPB);
  for (int it = 0; it < iters; it++) {
    const int row = (it * gridDim.x + blockIdx.x) * RPB + sub;
    const bool live = row < rows;
    const size_t off = (size_t)(live ? row : 0) * D;
    const float m = live ? mu[row] : 0.f, r = live ? rstd[row] : 0.f;
    V dv[LN_MAXV], xv[LN_MAXV];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; i++) {
      int c = tr + i * TPR;
      if (c < nvec) {
        dv[i].load(dh + off + c * V::N);
        xv[i].load(x + off + c * V::N);
#pragma unroll
        for (int e = 0; e < V::N; e++) {
          float xh = (xv[i].get(e) - m) * r;
          float g = dv[i].get(e) * gv[i].get(e);
          s1 += g;
          s2 += g * xh;
          if (live) {
            ag[i][e] += dv[i].get(e) * xh;
            ab[i][e] += dv[i].get(e);
          }
        }
      }
    }
    const float m1 = row_sum<TPR>(s1, red) / D;
    const float m2 = row_sum<TPR>(s2, red) / D;
    if (live) {
#pragma unroll
      for (int i = 0; i < LN_MAXV; i++) {
        int c = tr + i * TPR;
        if (c < nvec) {
          V o, rv;
          if (dres) rv.load(dres + off + c * V::N);
#pragma unroll
          for (int e = 0; e < V::N; e++) {
            float xh = (xv[i].get(e) - m) * r;
            float g = dv[i].get(e) * gv[i].get(e);
            float d = r * (g - m1 - xh * m2);
            if (dres) d += rv.get(e);
            o.set(e, d);
          }
          o.store(dx + off + c * V::N);
        }
      }
    }
  }
  float* pg = partial + (size_t)(blockIdx.x * RPB + sub) * 2 * D;
#pragma unroll
  for (int i = 0; i < LN_MAXV; i++) {
    int c = tr + i * TPR;
    if (c < nvec) {
#pragma unroll
      for (int e = 0; e < V::N; e++) {
        pg[c * V::N + e] = ag[i][e];
        pg[D + c * V::N + e] = ab[i][e];
      }
    }
  }
}

// Any D: one wave per row for dx; dgamma/dbeta partials through global atomics-free strips:
// each wave owns a strip of rows and loops over columns, writing its own partial row.
template <typename T>
__global__ __launch_bounds__(LN_THREADS) void ln_bwd_generic_kernel(int rows, int D, const T* __restrict__ dh,
                                                                    const T* __restrict__ x,
                                                                    const float* __restrict__ mu,
                                                                    const float* __restrict__ rstd,
                                                                    const T* __restrict__ gamma,
                                                                    const T* __restrict__ dres, T* __restrict__ dx,
                                                                    float* __restrict__ partial) {
  const int lane = threadIdx.x & 63;
  const int wid = blockIdx.x * (LN_THREADS / 64) + (threadIdx.x >> 6);
  const int nw = gridDim.x * (LN_THREADS / 64);
  float* pg = partial + (size_t)wid * 2 * D;
  for (int c = lane; c < D; c += 64) pg[c] = pg[D + c] = 0.f;
  for (int row = wid; row < rows; row += nw) {
    const size_t off = (size_t)row * D;
    const float m = mu[row], r = rstd[row];
    float s1 = 0.f, s2 = 0.f;
    for (int c = lane; c < D; c += 64) {
      float d = to_f(dh[off + c]);
      float xh = (to_f(x[off + c]) - m) * r;
      float g = d * to_f(gamma[c]);
      s1 += g;
      s2 += g * xh;
      pg[c] += d * xh;
      pg[D + c] += d;
    }
    const float m1 = wave_sum(s1) / D, m2 = wave_sum(s2) / D;
    for (int c = lane; c < D; c += 64) {
      float xh = (to_f(x[off + c]) - m) * r;
      float g = to_f(dh[off + c]) * to_f(gamma[c]);
      float d = r * (g - m1 - xh * m2);
      if (dres) d += to_f(dres[off + c]);
      dx[off + c] = from_f<T>(d);
    }
  }
}

// out[n] (+)= sum_p partial[p*stride + n]
__global__ __launch_bounds__(256) void fold_partials_kernel(int parts, size_t stride, int N,
                                                            const float* __restrict__ partial,
                                                            float* __restrict__ out, int accumulate) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  float s = 0.f;
  for (int p = 0; p < parts; p++) s += partial[(size_t)p * stride + n];
  out[n] = accumulate ? out[n] + s : s;
}

size_t ln_bwd_ws_bytes(int D) { return (size_t)RED_PARTS * 4 * 2 * (size_t)D * sizeof(float); }

template <typename T>
static int ln_bwd_t(int rows, int D, const T* dh, const T* x, const float* mu, const float* rstd, const T* gamma,
                    const T* dres, T* dx, float* dgamma, float* dbeta, bool accumulate, float* partial,
                    hipStream_t s) {
  constexpr int VN = Vec16<T>::N;
  const int nvec = D / VN;
  int parts;
  if (D % VN == 0 && nvec <= 256 * LN_MAXV) {
    if (nvec <= 64 * LN_MAXV / 2) {
      int grid = min(RED_PARTS, (rows + 3) / 4);
      parts = grid * 4;
      hipLaunchKernelGGL((ln_bwd_kernel<T, 64>), dim3(grid), dim3(LN_THREADS), 0, s, rows, D, dh, x, mu, rstd, gamma, dres,
                         dx, partial);
    } else if (nvec <= 128 * LN_MAXV / 2) {
      int grid = min(RED_PARTS, (rows + 1) / 2);
      parts = grid * 2;
      hipLaunchKernelGGL((ln_bwd_kernel<T, 128>), dim3(grid), dim3(LN_THREADS), 0, s, rows, D, dh, x, mu, rstd, gamma,
                         dres, dx, partial);
    } else {
      int grid = min(RED_PARTS, rows);
      parts = grid;
      hipLaunchKernelGGL((ln_bwd_kernel<T, 256>), dim3(grid), dim3(LN_THREADS), 0, s, rows, D, dh, x, mu, rstd, gamma,
                         dres, dx, partial);
    }
  } else {
    int grid = min(RED_PARTS, (rows + 3) / 4);
    parts = grid * 4;
    hipLaunchKernelGGL((ln_bwd_generic_kernel<T>), dim3(grid), dim3(LN_THREADS), 0, s, rows, D, dh, x, mu, rstd, gamma,
                       dres, dx, partial);
  }
  FAX_LAUNCH_CHECK("ln_bwd");
  const int gb = (D + 255) / 256;
  hipLaunchKernelGGL(fold_partials_kernel, dim3(gb), dim3(256), 0, s, parts, (size_t)2 * D, D, partial, dgamma,
                     accumulate ? 1 : 0);
  hipLaunchKernelGGL(fold_partials_kernel, dim3(gb), dim3(256), 0, s, parts, (size_t)2 * D, D, partial + D, dbeta,
                     accumulate ? 1 : 0);
  FAX_LAUNCH_CHECK("ln_bwd_fold");
  return FAX_OK;
}

int ln_bwd(int dtype, int rows, int D, const void* dh, const void* x, const float* mu, const float* rstd,
           const void* gamma, const void* dres, void* dx, float* dgamma, float* dbeta, bool accumulate, void* ws,
           hipStream_t s) {
  if (rows == 0) return FAX_OK;
  Timed t_("layernorm_bwd", WORK_BYTE, (dres ? 4.0 : 3.0) * rows * D * (dtype == FAX_F32 ? 4.0 : 2.0) + 8.0 * rows, s);
  if (dtype == FAX_F32)
    return ln_bwd_t<float>(rows, D, (const float*)dh, (const float*)x, mu, rstd, (const float*)gamma, (const float*)dres,
                           (float*)dx, dgamma, dbeta, accumulate, (float*)ws, s);
  return ln_bwd_t<bf16_t>(rows, D, (const bf16_t*)dh, (const bf16_t*)x, mu, rstd, (const bf16_t*)gamma,
                          (const bf16_t*)dres, (bf16_t*)dx, dgamma, dbeta, accumulate, (float*)ws, s);
}

// ---------------------------------------------------------------------------------------------
// Column sums (bias gradients): block (bx, by) sums a strip of rows for 64*VN columns.
// ---------------------------------------------------------------------------------------------
static constexpr int CS_PARTS = 128;

template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(int rows, int N, const T* __restrict__ a, int lda,
                                                     float* __restrict__ partial) {
  using V = Vec16<T>;
  __shared__ float red[4][64 * V::N];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = (blockIdx.x * 64 + lane) * V::N;
  float acc[V::N];
#pragma unroll
  for (int e = 0; e < V::N; e++) acc[e] = 0.f;
  const bool vec_ok = (c0 + V::N <= N) && (lda % V::N == 0);
  for (int r = blockIdx.y * 4 + wave; r < rows; r += gridDim.y * 4) {
    const T* p = a + (size_t)r * lda + c0;
    if (vec_ok) {
      V v;
      v.load(p);
#pragma unroll
      for (int e = 0; e < V::N; e++) acc[e] += v.get(e);
    } else {
#pragma unroll
      for (int e = 0; e < V::N; e++)
        if (c0 + e < N) acc[e] += to_f(p[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < V::N; e++) red[wave][lane * V::N + e] = acc[e];
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int e = 0; e < V::N; e++) {
      int c = c0 + e;
      if (c < N) {
        int i = lane * V::N + e;
        partial[(size_t)blockIdx.y * N + c] = red[0][i] + red[1][i] + red[2][i] + red[3][i];
      }
    }
  }
}

size_t colsum_ws_bytes(int N) { return (size_t)CS_PARTS * (size_t)N * sizeof(float); }

int colsum(int dtype, int rows, int N, const void* a, int lda, float* out, bool accumulate, void* ws, hipStream_t s) {
  if (N == 0) return FAX_OK;
  Timed t_("colsum", WORK_BYTE, 1.0 * rows * N * (dtype == FAX_F32 ? 4.0 : 2.0), s);
  const int parts = max(1, min(CS_PARTS, (rows + 3) / 4));
  float* partial = (float*)ws;
  if (dtype == FAX_F32) {
    dim3 grid((N + 64 * 4 - 1) / (64 * 4), parts);
    hipLaunchKernelGGL((colsum_kernel<float>), grid, dim3(256), 0, s, rows, N, (const float*)a, lda, partial);
  } else {
    dim3 grid((N + 64 * 8 - 1) / (64 * 8), parts);
    hipLaunchKernelGGL((colsum_kernel<bf16_t>), grid, dim3(256), 0, s, rows, N, (const bf16_t*)a, lda, partial);
  }
  FAX_LAUNCH_CHECK("colsum");
  hipLaunchKernelGGL(fold_partials_kernel, dim3((N + 255) / 256), dim3(256), 0, s, parts, (size_t)N, N, partial, out,
                     accumulate ? 1 : 0);
  FAX_LAUNCH_CHECK("colsum_fold");
  return FAX_OK;
}

}  // namespace fax
