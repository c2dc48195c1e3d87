// LayerNorm forward/backward and column sums: HBM-bound kernels.
//
// Forward reads each row once (16-byte loads, row cached in registers), writes it once.
// Backward is one pass as well: a workgroup walks over row blocks, reads dh and x once, writes dx
// once and keeps running per-column sums of dh * xhat and dh in registers; each workgroup leaves
// one partial row of dgamma and of dbeta, and a second small kernel folds the partial rows in a
// fixed order, so no result depends on scheduling order.  (Row lengths the vector kernels do not
// cover fall back to a row kernel for dx plus a column-parallel pass for the two sums.)
#include "fax_internal.h"

namespace fax {

static constexpr int LN_MAXV = 8;      // 16-byte vectors cached per thread
static constexpr int LN_THREADS = 256;
static constexpr int CS_PARTS = 128;   // row strips of the column-sum kernels

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
// Backward, row part: dx = rstd (g - mean(g) - xhat mean(g xhat)) [+ dres], g = dh * gamma.
// ---------------------------------------------------------------------------------------------
// With the parameter gradients folded in: a workgroup walks over row blocks b,
// b + gridDim.x, ... and every thread keeps the running sums of dh * xhat (-> dgamma) and dh
// (-> dbeta) for the columns it owns; dh and x are read once for all three results.  At the end
// the row groups of the workgroup are combined through LDS and one partial row per workgroup is
// written: partial[0][blockIdx.x][D] (dgamma), partial[1][blockIdx.x][D] (dbeta).
// NV: 16-byte vectors per thread and row (D <= TPR * NV * V::N).
template <typename T, int TPR, int NV>
__global__ __launch_bounds__(LN_THREADS) void ln_bwd_fused_kernel(int rows, int D, const T* __restrict__ dh,
                                                                  const T* __restrict__ x, const float* __restrict__ mu,
                                                                  const float* __restrict__ rstd,
                                                                  const T* __restrict__ gamma, const T* __restrict__ dres,
                                                                  T* __restrict__ dx, float* __restrict__ partial) {
  using V = Vec16<T>;
  constexpr int RPB = LN_THREADS / TPR;
  constexpr int NACC = NV * V::N * 2;  // running sums per thread
  __shared__ float red[LN_THREADS / 64];
  __shared__ float comb[RPB > 1 ? (RPB - 1) * NACC * TPR : 1];
  const int tr = threadIdx.x % TPR, rg = threadIdx.x / TPR;
  const int nvec = D / V::N;
  float ag[NV][V::N], ab[NV][V::N];
#pragma unroll
  for (int i = 0; i < NV; i++)
#pragma unroll
    for (int e = 0; e < V::N; e++) ag[i][e] = ab[i][e] = 0.f;
  for (int rb = blockIdx.x; rb * RPB < rows; rb += gridDim.x) {  // trip count uniform over the workgroup
    const int row = rb * RPB + rg;
    const bool live = row < rows;
    const size_t off = (size_t)(live ? row : 0) * D;
    const float m = live ? mu[row] : 0.f, r = live ? rstd[row] : 0.f;
    V dv[NV], xv[NV];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NV; i++) {
      const int c = tr + i * TPR;
      if (c < nvec) {
        V gv;
        gv.load(gamma + c * V::N);
        dv[i].load(dh + off + c * V::N);
        xv[i].load(x + off + c * V::N);
#pragma unroll
        for (int e = 0; e < V::N; e++) {
          const float xh = (xv[i].get(e) - m) * r;
          const float g = dv[i].get(e) * gv.get(e);
          s1 += g;
          s2 += g * xh;
        }
      }
    }
    const float m1 = row_sum<TPR>(s1, red) / D;
    const float m2 = row_sum<TPR>(s2, red) / D;
    if (live) {
#pragma unroll
      for (int i = 0; i < NV; i++) {
        const int c = tr + i * TPR;
        if (c < nvec) {
          V gv, o, rv;
          gv.load(gamma + c * V::N);
          if (dres) rv.load(dres + off + c * V::N);
#pragma unroll
          for (int e = 0; e < V::N; e++) {
            const float xh = (xv[i].get(e) - m) * r;
            const float dhe = dv[i].get(e);
            float d = r * (dhe * gv.get(e) - m1 - xh * m2);
            if (dres) d += rv.get(e);
            o.set(e, d);
            ag[i][e] += dhe * xh;
            ab[i][e] += dhe;
          }
          o.store(dx + off + c * V::N);
        }
      }
    }
  }
  if (RPB > 1) {
    __syncthreads();
    if (rg > 0) {
#pragma unroll
      for (int i = 0; i < NV; i++)
#pragma unroll
        for (int e = 0; e < V::N; e++) {
          comb[(((rg - 1) * NV + i) * V::N * 2 + e) * TPR + tr] = ag[i][e];
          comb[(((rg - 1) * NV + i) * V::N * 2 + V::N + e) * TPR + tr] = ab[i][e];
        }
    }
    __syncthreads();
    if (rg > 0) return;
#pragma unroll
    for (int g = 0; g < RPB - 1; g++)
#pragma unroll
      for (int i = 0; i < NV; i++)
#pragma unroll
        for (int e = 0; e < V::N; e++) {
          ag[i][e] += comb[((g * NV + i) * V::N * 2 + e) * TPR + tr];
          ab[i][e] += comb[((g * NV + i) * V::N * 2 + V::N + e) * TPR + tr];
        }
  }
  float* pg = partial + (size_t)blockIdx.x * D;
  float* pb = partial + ((size_t)gridDim.x + blockIdx.x) * D;
#pragma unroll
  for (int i = 0; i < NV; i++) {
    const int c = tr + i * TPR;
    if (c < nvec) {
#pragma unroll
      for (int e = 0; e < V::N; e += 4) {
        *reinterpret_cast<float4*>(pg + c * V::N + e) = make_float4(ag[i][e], ag[i][e + 1], ag[i][e + 2], ag[i][e + 3]);
        *reinterpret_cast<float4*>(pb + c * V::N + e) = make_float4(ab[i][e], ab[i][e + 1], ab[i][e + 2], ab[i][e + 3]);
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(LN_THREADS) void ln_bwd_dx_generic_kernel(int rows, int D, const T* __restrict__ dh,
                                                                       const T* __restrict__ x,
                                                                       const float* __restrict__ mu,
                                                                       const float* __restrict__ rstd,
                                                                       const T* __restrict__ gamma,
                                                                       const T* __restrict__ dres, T* __restrict__ dx) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (LN_THREADS / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const size_t off = (size_t)row * D;
  const float m = mu[row], r = rstd[row];
  float s1 = 0.f, s2 = 0.f;
  for (int c = lane; c < D; c += 64) {
    const float xh = (to_f(x[off + c]) - m) * r;
    const float g = to_f(dh[off + c]) * to_f(gamma[c]);
    s1 += g;
    s2 += g * xh;
  }
  const float m1 = wave_sum(s1) / D, m2 = wave_sum(s2) / D;
  for (int c = lane; c < D; c += 64) {
    const float xh = (to_f(x[off + c]) - m) * r;
    const float g = to_f(dh[off + c]) * to_f(gamma[c]);
    float d = r * (g - m1 - xh * m2);
    if (dres) d += to_f(dres[off + c]);
    dx[off + c] = from_f<T>(d);
  }
}

// ---------------------------------------------------------------------------------------------
// Column sums.  Block (bx, by): 64*VN columns, row strip by; its four waves take every fourth
// row of the strip, sum in registers, combine through LDS and write one partial row.
// MODE 0: out = sum_r a[r, n]                      (bias gradients)
// MODE 1: out0 = sum_r a[r, n] xhat[r, n], out1 = sum_r a[r, n]   (dgamma, dbeta; a = dh)
// partial layout: [MODE + 1][gridDim.y][N]
// ---------------------------------------------------------------------------------------------
template <typename T, int MODE>
__global__ __launch_bounds__(256) void colsum_kernel(int rows, int N, const T* __restrict__ a, int lda,
                                                     const T* __restrict__ x, const float* __restrict__ mu,
                                                     const float* __restrict__ rstd, float* __restrict__ partial) {
  using V = Vec16<T>;
  __shared__ float red[4][(MODE + 1) * 64 * V::N];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = (blockIdx.x * 64 + lane) * V::N;
  float acc[MODE + 1][V::N];
#pragma unroll
  for (int k = 0; k <= MODE; k++)
#pragma unroll
    for (int e = 0; e < V::N; e++) acc[k][e] = 0.f;
  const bool vec_ok = (c0 + V::N <= N) && (lda % V::N == 0);
  for (int r = blockIdx.y * 4 + wave; r < rows; r += gridDim.y * 4) {
    const T* p = a + (size_t)r * lda + c0;
    float m = 0.f, rs = 0.f;
    if (MODE == 1) {
      m = mu[r];
      rs = rstd[r];
    }
    if (vec_ok) {
      V v, xv;
      v.load(p);
      if (MODE == 1) xv.load(x + (size_t)r * lda + c0);
#pragma unroll
      for (int e = 0; e < V::N; e++) {
        if (MODE == 1) {
          acc[0][e] += v.get(e) * ((xv.get(e) - m) * rs);
          acc[MODE][e] += v.get(e);
        } else {
          acc[0][e] += v.get(e);
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < V::N; e++)
        if (c0 + e < N) {
          const float d = to_f(p[e]);
          if (MODE == 1) {
            acc[0][e] += d * ((to_f(x[(size_t)r * lda + c0 + e]) - m) * rs);
            acc[MODE][e] += d;
          } else {
            acc[0][e] += d;
          }
        }
    }
  }
#pragma unroll
  for (int k = 0; k <= MODE; k++)
#pragma unroll
    for (int e = 0; e < V::N; e++) red[wave][(k * 64 + lane) * V::N + e] = acc[k][e];
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int k = 0; k <= MODE; k++)
#pragma unroll
      for (int e = 0; e < V::N; e++) {
        const int c = c0 + e;
        if (c < N) {
          const int i = (k * 64 + lane) * V::N + e;
          partial[((size_t)k * gridDim.y + blockIdx.y) * N + c] = red[0][i] + red[1][i] + red[2][i] + red[3][i];
        }
      }
  }
}

// The same for N a multiple of 4 and many parts: a block takes 64 columns as 16 float4 lanes and
// splits the parts 16 ways (thread = 16 * part group + column group), combining through LDS.
__global__ __launch_bounds__(256) void fold_partials4_kernel(int parts, int N, const float* __restrict__ partial,
                                                             float* __restrict__ out0, float* __restrict__ out1,
                                                             int accumulate) {
  __shared__ float4 red[16][16];
  const int cg = threadIdx.x & 15, pgp = threadIdx.x >> 4;
  const int n = blockIdx.x * 64 + cg * 4;
  partial += (size_t)blockIdx.y * parts * N;
  float* out = blockIdx.y ? out1 : out0;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (n < N) {
#pragma unroll 4
    for (int p = pgp; p < parts; p += 16) {
      const float4 v = *reinterpret_cast<const float4*>(partial + (size_t)p * N + n);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
  }
  red[pgp][cg] = s;
  __syncthreads();
  if (pgp == 0 && n < N) {
#pragma unroll
    for (int g = 1; g < 16; g++) {
      const float4 v = red[g][cg];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    float4* o = reinterpret_cast<float4*>(out + n);
    if (accumulate) {
      const float4 v = *o;
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *o = s;
  }
}

// out[n] (+)= sum_p partial[p * N + n], p < parts: 64 columns per block, 4 waves split the parts.
// blockIdx.y = 1 folds a second stack of partials, stored right behind the first, into out1.
__global__ __launch_bounds__(256) void fold_partials_kernel(int parts, int N, const float* __restrict__ partial,
                                                            float* __restrict__ out0, float* __restrict__ out1,
                                                            int accumulate) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + lane;
  partial += (size_t)blockIdx.y * parts * N;
  float* out = blockIdx.y ? out1 : out0;
  float s = 0.f;
  if (n < N)
    for (int p = wave; p < parts; p += 4) s += partial[(size_t)p * N + n];
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && n < N) {
    s = red[0][lane] + red[1][lane] + red[2][lane] + red[3][lane];
    out[n] = accumulate ? out[n] + s : s;
  }
}

// The same for long vectors, four elements per thread: out[i] (+)= (partial[0][i] + partial[1][i] + ...).
// The blocks from `blocks_a` on fold a second, short stack of partials (nb elements each, any nb) into out_b,
// one element per thread, in the same launch.
__global__ __launch_bounds__(256) void fold_partials_vec_kernel(int parts, size_t n4, const float4* __restrict__ partial,
                                                                float4* __restrict__ out, int accumulate, unsigned blocks_a,
                                                                int nb, const float* __restrict__ partial_b,
                                                                float* __restrict__ out_b) {
  if (blockIdx.x >= blocks_a) {
    const int j = (int)(blockIdx.x - blocks_a) * 256 + (int)threadIdx.x;
    if (j >= nb) return;
    float sb = partial_b[j];
    for (int p = 1; p < parts; p++) sb += partial_b[(size_t)p * nb + j];
    out_b[j] = accumulate ? out_b[j] + sb : sb;
    return;
  }
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  float4 s = partial[i];
#pragma unroll 4
  for (int p = 1; p < parts; p++) {
    const float4 v = partial[(size_t)p * n4 + i];
    s.x += v.x;
    s.y += v.y;
    s.z += v.z;
    s.w += v.w;
  }
  if (accumulate) {
    const float4 o = out[i];
    s.x += o.x;
    s.y += o.y;
    s.z += o.z;
    s.w += o.w;
  }
  out[i] = s;
}

int fold_partials(int parts, size_t n, const float* partial, float* out, bool accumulate, hipStream_t s, int nb,
                  const float* partial_b, float* out_b) {
  if (n == 0) return nb > 0 ? fold_partials(parts, (size_t)nb, partial_b, out_b, accumulate, s) : FAX_OK;
  if (n % 4 == 0 && n >= 4096 && ((reinterpret_cast<uintptr_t>(partial) | reinterpret_cast<uintptr_t>(out)) & 15) == 0 &&
      n / 4 / 256 < 0x7ff00000) {
    const unsigned blocks_a = (unsigned)((n / 4 + 255) / 256);
    const unsigned blocks_b = nb > 0 ? (unsigned)((nb + 255) / 256) : 0u;
    hipLaunchKernelGGL(fold_partials_vec_kernel, dim3(blocks_a + blocks_b), dim3(256), 0, s, parts, n / 4,
                       (const float4*)partial, (float4*)out, accumulate ? 1 : 0, blocks_a, nb, partial_b, out_b);
    FAX_LAUNCH_CHECK("fold_partials");
    return FAX_OK;
  }
  if (nb > 0) FAX_TRY(fold_partials(parts, (size_t)nb, partial_b, out_b, accumulate, s));
  if (n > (size_t)0x7fffffff) {
    set_error("fold_partials: %zu elements", n);
    return FAX_ERR_UNSUPPORTED;
  }
  hipLaunchKernelGGL(fold_partials_kernel, dim3((unsigned)((n + 63) / 64)), dim3(256), 0, s, parts, (int)n, partial, out,
                     (float*)nullptr, accumulate ? 1 : 0);
  FAX_LAUNCH_CHECK("fold_partials");
  return FAX_OK;
}

static int strips(int rows) { return max(1, min(CS_PARTS, (rows + 3) / 4)); }

static constexpr int LN_BWD_PARTS = 1024;  // workgroups (= partial rows) of the fused LayerNorm backward
size_t ln_bwd_ws_bytes(int D) { return (size_t)2 * LN_BWD_PARTS * (size_t)D * sizeof(float); }
size_t colsum_ws_bytes(int N) { return (size_t)CS_PARTS * (size_t)N * sizeof(float); }

template <typename T>
static int ln_bwd_t(int rows, int D, const T* dh, const T* x, const float* mu, const float* rstd, const T* gamma,
                    const T* dres, T* dx, float* dgamma, float* dbeta, bool accumulate, float* partial,
                    hipStream_t s, hipStream_t fold_s, hipEvent_t handover) {
  constexpr int VN = Vec16<T>::N;
  const int nvec = D / VN;
  const int gb = (D + 63) / 64;
  if (D % VN == 0 && nvec <= 256 * LN_MAXV) {
    // one pass: dx and, per workgroup, a partial row of dgamma and of dbeta
    int parts;
    // Each workgroup writes two fp32 partial rows, which the fold reads back: with R rows per
    // workgroup that is 2 / R on top of the rows' own traffic.  Eight row blocks per workgroup, fewer
    // (down to two) while that leaves less than two workgroups per CU: with few tokens the
    // parallelism is worth more than the partial rows cost (2048 x 5120: 43 -> 31 us).
    auto grid = [&](int rpb) {
      int per_wg = 8;
      while (per_wg > 2 && rows / (per_wg * rpb) < 512) per_wg /= 2;
      return parts = max(1, min(LN_BWD_PARTS, (rows + per_wg * rpb - 1) / (per_wg * rpb)));
    };
    // threads per row and vectors per thread: as few registers as the row length allows, so that
    // several workgroups fit on a CU
#define FAX_LN_BWD_FUSED(TPR, NV)                                                                                   \
  hipLaunchKernelGGL((ln_bwd_fused_kernel<T, TPR, NV>), dim3(grid(LN_THREADS / TPR)), dim3(LN_THREADS), 0, s, rows, D, \
                     dh, x, mu, rstd, gamma, dres, dx, partial)
    if (nvec <= 64 * 2) FAX_LN_BWD_FUSED(64, 2);
    else if (nvec <= 128 * 2) FAX_LN_BWD_FUSED(128, 2);  // D = 2048: twice the workgroups of (64, 4) at two thirds of its registers
    else if (nvec <= 256 * 2) FAX_LN_BWD_FUSED(256, 2);
    else if (nvec <= 256 * 3) FAX_LN_BWD_FUSED(256, 3);
    else if (nvec <= 256 * 4) FAX_LN_BWD_FUSED(256, 4);
    else if (nvec <= 256 * 5) FAX_LN_BWD_FUSED(256, 5);
    else if (nvec <= 256 * 6) FAX_LN_BWD_FUSED(256, 6);
    else FAX_LN_BWD_FUSED(256, LN_MAXV);
#undef FAX_LN_BWD_FUSED
    FAX_LAUNCH_CHECK("ln_bwd_fused");
    // The fold only feeds the parameter gradients, nothing further down the backward pass: given a
    // second stream it goes there, behind an event that marks the partial rows complete.
    hipStream_t fs = s;
    if (fold_s && fold_s != s && handover) {
      FAX_HIP(hipEventRecord(handover, s));
      FAX_HIP(hipStreamWaitEvent(fold_s, handover, 0));
      fs = fold_s;
    }
    if (D % 4 == 0 && ((reinterpret_cast<uintptr_t>(dgamma) | reinterpret_cast<uintptr_t>(dbeta)) & 15) == 0)
      hipLaunchKernelGGL(fold_partials4_kernel, dim3(gb, 2), dim3(256), 0, fs, parts, D, partial, dgamma, dbeta, accumulate ? 1 : 0);
    else
      hipLaunchKernelGGL(fold_partials_kernel, dim3(gb, 2), dim3(256), 0, fs, parts, D, partial, dgamma, dbeta, accumulate ? 1 : 0);
    FAX_LAUNCH_CHECK("ln_bwd_fold");
    return FAX_OK;
  }
  hipLaunchKernelGGL((ln_bwd_dx_generic_kernel<T>), dim3((rows + 3) / 4), dim3(LN_THREADS), 0, s, rows, D, dh, x, mu,
                     rstd, gamma, dres, dx);
  FAX_LAUNCH_CHECK("ln_bwd_dx");
  const int parts = strips(rows);
  hipLaunchKernelGGL((colsum_kernel<T, 1>), dim3((D + 64 * VN - 1) / (64 * VN), parts), dim3(256), 0, s, rows, D, dh, D, x,
                     mu, rstd, partial);
  FAX_LAUNCH_CHECK("ln_bwd_dgamma_dbeta");
  hipLaunchKernelGGL(fold_partials_kernel, dim3(gb, 2), dim3(256), 0, s, parts, D, partial, dgamma, dbeta, accumulate ? 1 : 0);
  FAX_LAUNCH_CHECK("ln_bwd_fold");
  return FAX_OK;
}

int ln_bwd(int dtype, int rows, int D, const void* dh, const void* x, const float* mu, const float* rstd,
           const void* gamma, const void* dres, void* dx, float* dgamma, float* dbeta, bool accumulate, void* ws,
           hipStream_t s, hipStream_t fold_s, hipEvent_t handover) {
  if (rows == 0) return FAX_OK;
  Timed t_("layernorm_bwd", WORK_BYTE, (dres ? 4.0 : 3.0) * rows * D * (dtype == FAX_F32 ? 4.0 : 2.0) + 8.0 * rows, s);
  if (dtype == FAX_F32)
    return ln_bwd_t<float>(rows, D, (const float*)dh, (const float*)x, mu, rstd, (const float*)gamma, (const float*)dres,
                           (float*)dx, dgamma, dbeta, accumulate, (float*)ws, s, fold_s, handover);
  return ln_bwd_t<bf16_t>(rows, D, (const bf16_t*)dh, (const bf16_t*)x, mu, rstd, (const bf16_t*)gamma,
                          (const bf16_t*)dres, (bf16_t*)dx, dgamma, dbeta, accumulate, (float*)ws, s, fold_s, handover);
}

int colsum(int dtype, int rows, int N, const void* a, int lda, float* out, bool accumulate, void* ws, hipStream_t s) {
  if (N == 0) return FAX_OK;
  Timed t_("colsum", WORK_BYTE, 1.0 * rows * N * (dtype == FAX_F32 ? 4.0 : 2.0), s);
  const int parts = strips(rows);
  float* partial = (float*)ws;
  if (dtype == FAX_F32) {
    dim3 grid((N + 64 * 4 - 1) / (64 * 4), parts);
    hipLaunchKernelGGL((colsum_kernel<float, 0>), grid, dim3(256), 0, s, rows, N, (const float*)a, lda, (const float*)nullptr,
                       (const float*)nullptr, (const float*)nullptr, partial);
  } else {
    dim3 grid((N + 64 * 8 - 1) / (64 * 8), parts);
    hipLaunchKernelGGL((colsum_kernel<bf16_t, 0>), grid, dim3(256), 0, s, rows, N, (const bf16_t*)a, lda,
                       (const bf16_t*)nullptr, (const float*)nullptr, (const float*)nullptr, partial);
  }
  FAX_LAUNCH_CHECK("colsum");
  hipLaunchKernelGGL(fold_partials_kernel, dim3((N + 63) / 64), dim3(256), 0, s, parts, N, partial, out, (float*)nullptr,
                     accumulate ? 1 : 0);
  FAX_LAUNCH_CHECK("colsum_fold");
  return FAX_OK;
}

}  // namespace fax
