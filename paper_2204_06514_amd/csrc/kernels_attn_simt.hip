// Causal attention with scalar FMAs: the fp32 path, and the fallback for head widths the MFMA
// kernel does not cover.  One wavefront per query row (forward, dQ) or per key row (dK, dV);
// scores are never materialised: a 64-key chunk at a time with a running max and sum.
// No atomics: every output element has exactly one writer.
#include "fax_internal.h"

namespace fax {

static constexpr int AT_MAXDH = 256;  // lane owns d = lane + 64 r, r < 4

template <typename T>
__device__ __forceinline__ float dot_row(const float* __restrict__ a, const T* __restrict__ row, int dh) {
  float s = 0.f;
  for (int d = 0; d < dh; d++) s = fmaf(a[d], to_f(row[d]), s);
  return s;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_simt_kernel(int S, int H, int dh, const T* __restrict__ qkv,
                                                            T* __restrict__ ctx, float* __restrict__ lse) {
  __shared__ float qs[4][AT_MAXDH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int Hd = H * dh, ld = 3 * Hd;
  const int i = blockIdx.x * 4 + wave;
  const T* base = qkv + (size_t)b * S * ld + h * dh;
  if (i < S)
    for (int d = lane; d < dh; d += 64) qs[wave][d] = to_f(base[(size_t)i * ld + d]);
  __syncthreads();
  if (i >= S) return;
  const float scale = rsqrtf((float)dh);
  float m = -INFINITY, l = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    const bool ok = j <= i;
    float sc = ok ? dot_row<T>(qs[wave], base + (size_t)j * ld + Hd, dh) * scale : -INFINITY;
    const float mn = fmaxf(m, wave_max(sc));
    const float p = ok ? expf(sc - mn) : 0.f;
    const float corr = expf(m - mn);
    l = l * corr + wave_sum(p);
#pragma unroll
    for (int r = 0; r < 4; r++) acc[r] *= corr;
    const int nj = min(64, i - j0 + 1);
    for (int jj = 0; jj < nj; jj++) {
      const float pj = __shfl(p, jj, 64);
      const T* vr = base + (size_t)(j0 + jj) * ld + 2 * Hd;
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int d = lane + 64 * r;
        if (d < dh) acc[r] = fmaf(pj, to_f(vr[d]), acc[r]);
      }
    }
    m = mn;
  }
  T* out = ctx + ((size_t)b * S + i) * Hd + h * dh;
  const float inv = 1.f / l;
#pragma unroll
  for (int r = 0; r < 4; r++) {
    const int d = lane + 64 * r;
    if (d < dh) out[d] = from_f<T>(acc[r] * inv);
  }
  if (lane == 0) lse[((size_t)b * H + h) * S + i] = m + logf(l);
}

// delta[b,h,i] = sum_d dO[i,d] O[i,d]
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(int S, int H, int dh, const T* __restrict__ ctx,
                                                         const T* __restrict__ dctx, float* __restrict__ delta) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int i = blockIdx.x * 4 + wave;
  if (i >= S) return;
  const size_t off = ((size_t)b * S + i) * H * dh + h * dh;
  float s = 0.f;
  for (int d = lane; d < dh; d += 64) s += to_f(ctx[off + d]) * to_f(dctx[off + d]);
  s = wave_sum(s);
  if (lane == 0) delta[((size_t)b * H + h) * S + i] = s;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_simt_kernel(int S, int H, int dh, const T* __restrict__ qkv,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ delta,
                                                               const T* __restrict__ dctx, T* __restrict__ dqkv) {
  __shared__ float qs[4][AT_MAXDH];
  __shared__ float dos[4][AT_MAXDH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int Hd = H * dh, ld = 3 * Hd;
  const int i = blockIdx.x * 4 + wave;
  const T* base = qkv + (size_t)b * S * ld + h * dh;
  if (i < S)
    for (int d = lane; d < dh; d += 64) {
      qs[wave][d] = to_f(base[(size_t)i * ld + d]);
      dos[wave][d] = to_f(dctx[((size_t)b * S + i) * Hd + h * dh + d]);
    }
  __syncthreads();
  if (i >= S) return;
  const float scale = rsqrtf((float)dh);
  const float li = lse[((size_t)b * H + h) * S + i], di = delta[((size_t)b * H + h) * S + i];
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    float ds = 0.f;
    if (j <= i) {
      const float sc = dot_row<T>(qs[wave], base + (size_t)j * ld + Hd, dh) * scale;
      const float p = expf(sc - li);
      const float dp = dot_row<T>(dos[wave], base + (size_t)j * ld + 2 * Hd, dh);
      ds = p * (dp - di);
    }
    const int nj = min(64, i - j0 + 1);
    for (int jj = 0; jj < nj; jj++) {
      const float dsj = __shfl(ds, jj, 64);
      const T* kr = base + (size_t)(j0 + jj) * ld + Hd;
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int d = lane + 64 * r;
        if (d < dh) acc[r] = fmaf(dsj, to_f(kr[d]), acc[r]);
      }
    }
  }
  T* out = dqkv + ((size_t)b * S + i) * ld + h * dh;
#pragma unroll
  for (int r = 0; r < 4; r++) {
    const int d = lane + 64 * r;
    if (d < dh) out[d] = from_f<T>(acc[r] * scale);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_simt_kernel(int S, int H, int dh, const T* __restrict__ qkv,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ delta,
                                                                const T* __restrict__ dctx, T* __restrict__ dqkv) {
  __shared__ float ks[4][AT_MAXDH];
  __shared__ float vs[4][AT_MAXDH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int Hd = H * dh, ld = 3 * Hd;
  const int j = blockIdx.x * 4 + wave;
  const T* base = qkv + (size_t)b * S * ld + h * dh;
  const T* dob = dctx + (size_t)b * S * Hd + h * dh;
  if (j < S)
    for (int d = lane; d < dh; d += 64) {
      ks[wave][d] = to_f(base[(size_t)j * ld + Hd + d]);
      vs[wave][d] = to_f(base[(size_t)j * ld + 2 * Hd + d]);
    }
  __syncthreads();
  if (j >= S) return;
  const float scale = rsqrtf((float)dh);
  const float* lrow = lse + ((size_t)b * H + h) * S;
  const float* drow = delta + ((size_t)b * H + h) * S;
  float ak[4] = {0.f, 0.f, 0.f, 0.f}, av[4] = {0.f, 0.f, 0.f, 0.f};
  for (int i0 = j; i0 < S; i0 += 64) {
    const int i = i0 + lane;
    float p = 0.f, ds = 0.f;
    if (i < S) {
      const float sc = dot_row<T>(ks[wave], base + (size_t)i * ld, dh) * scale;
      p = expf(sc - lrow[i]);
      const float dp = dot_row<T>(vs[wave], dob + (size_t)i * Hd, dh);
      ds = p * (dp - drow[i]);
    }
    const int ni = min(64, S - i0);
    for (int ii = 0; ii < ni; ii++) {
      const float pi = __shfl(p, ii, 64), dsi = __shfl(ds, ii, 64);
      const T* qr = base + (size_t)(i0 + ii) * ld;
      const T* dor = dob + (size_t)(i0 + ii) * Hd;
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int d = lane + 64 * r;
        if (d < dh) {
          av[r] = fmaf(pi, to_f(dor[d]), av[r]);
          ak[r] = fmaf(dsi, to_f(qr[d]), ak[r]);
        }
      }
    }
  }
  T* out = dqkv + ((size_t)b * S + j) * ld + h * dh;
#pragma unroll
  for (int r = 0; r < 4; r++) {
    const int d = lane + 64 * r;
    if (d < dh) {
      out[Hd + d] = from_f<T>(ak[r] * scale);
      out[2 * Hd + d] = from_f<T>(av[r]);
    }
  }
}

int attn_delta(int dtype, int B, int S, int H, int dh, const void* ctx, const void* dctx, float* delta, hipStream_t s) {
  dim3 grid((S + 3) / 4, B * H);
  if (dtype == FAX_F32)
    hipLaunchKernelGGL((attn_delta_kernel<float>), grid, dim3(256), 0, s, S, H, dh, (const float*)ctx, (const float*)dctx,
                       delta);
  else
    hipLaunchKernelGGL((attn_delta_kernel<bf16_t>), grid, dim3(256), 0, s, S, H, dh, (const bf16_t*)ctx,
                       (const bf16_t*)dctx, delta);
  FAX_LAUNCH_CHECK("attn_delta");
  return FAX_OK;
}

template <typename T>
static int attn_fwd_simt_t(int B, int S, int H, int dh, const T* qkv, T* ctx, float* lse, hipStream_t s) {
  dim3 grid((S + 3) / 4, B * H);
  hipLaunchKernelGGL((attn_fwd_simt_kernel<T>), grid, dim3(256), 0, s, S, H, dh, qkv, ctx, lse);
  FAX_LAUNCH_CHECK("attn_fwd_simt");
  return FAX_OK;
}

int attn_fwd_simt(int dtype, int B, int S, int H, int dh, const void* qkv, void* ctx, float* lse, hipStream_t s) {
  if (dh > AT_MAXDH) {
    set_error("attention: head width %d exceeds %d", dh, AT_MAXDH);
    return FAX_ERR_UNSUPPORTED;
  }
  if (B * H == 0 || S == 0) return FAX_OK;
  if (dtype == FAX_F32) return attn_fwd_simt_t<float>(B, S, H, dh, (const float*)qkv, (float*)ctx, lse, s);
  return attn_fwd_simt_t<bf16_t>(B, S, H, dh, (const bf16_t*)qkv, (bf16_t*)ctx, lse, s);
}

template <typename T>
static int attn_bwd_simt_t(int B, int S, int H, int dh, const T* qkv, const T* ctx, const float* lse, const T* dctx,
                           T* dqkv, float* delta, hipStream_t s) {
  dim3 grid((S + 3) / 4, B * H);
  hipLaunchKernelGGL((attn_delta_kernel<T>), grid, dim3(256), 0, s, S, H, dh, ctx, dctx, delta);
  hipLaunchKernelGGL((attn_bwd_dq_simt_kernel<T>), grid, dim3(256), 0, s, S, H, dh, qkv, lse, delta, dctx, dqkv);
  hipLaunchKernelGGL((attn_bwd_dkv_simt_kernel<T>), grid, dim3(256), 0, s, S, H, dh, qkv, lse, delta, dctx, dqkv);
  FAX_LAUNCH_CHECK("attn_bwd_simt");
  return FAX_OK;
}

int attn_bwd_simt(int dtype, int B, int S, int H, int dh, const void* qkv, const void* ctx, const float* lse,
                  const void* dctx, void* dqkv, float* delta, hipStream_t s) {
  if (dh > AT_MAXDH) {
    set_error("attention: head width %d exceeds %d", dh, AT_MAXDH);
    return FAX_ERR_UNSUPPORTED;
  }
  if (B * H == 0 || S == 0) return FAX_OK;
  if (dtype == FAX_F32)
    return attn_bwd_simt_t<float>(B, S, H, dh, (const float*)qkv, (const float*)ctx, lse, (const float*)dctx,
                                  (float*)dqkv, delta, s);
  return attn_bwd_simt_t<bf16_t>(B, S, H, dh, (const bf16_t*)qkv, (const bf16_t*)ctx, lse, (const bf16_t*)dctx,
                                 (bf16_t*)dqkv, delta, s);
}

}  // namespace fax
