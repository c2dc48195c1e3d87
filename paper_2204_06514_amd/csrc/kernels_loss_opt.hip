// HBM-bound kernels around the blocks: softmax cross-entropy (forward + gradient in one pass
// over the logits), embedding gather / scatter, and the AdamW update.
#include <mutex>

#include "fax_internal.h"

namespace fax {

// ---------------------------------------------------------------------------------------------
// Cross-entropy.  One workgroup per row.  The row is read from HBM once and kept in registers as
// the raw 16-byte vectors it arrived in; the gradient grad_scale (softmax - onehot)/N is written
// over it (or anywhere else; nowhere when dlogits is NULL: loss only), so the logits cross HBM
// once in each direction.
//
// What bounds it besides HBM is the vector unit (one exponential per logit and pass, quarter
// rate), so the arithmetic is kept short: the exponentials are single v_exp_f32 instructions on
// (z - maximum) log2(e); each thread first reduces its
// own elements to a (maximum, sum of 2^(t - maximum)) pair and the pairs are then combined across
// the workgroup in one step (one barrier instead of one per reduction); the one element that
// carries the label is patched by the thread that holds it instead of every element being
// compared with the label.  The workgroup size is chosen on the host so that the row divides
// evenly over the threads (51200 bf16 logits: 640 threads x 10 vectors).
// ---------------------------------------------------------------------------------------------
static constexpr int CE_MAX_THREADS = 1024;
static constexpr int CE_MAX_NV = 16;
static constexpr float CE_LOG2E = 1.4426950408889634f;
static constexpr float CE_LN2 = 0.6931471805599453f;

__device__ __forceinline__ float block_reduce(float v, float* red, bool is_max) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
  for (int i = 1; i < nw; i++) r = is_max ? fmaxf(r, red[i]) : r + red[i];
  return r;
}

// NV: 16-byte vectors per thread (V <= blockDim.x * NV * elements per vector, V a multiple of the latter).
template <typename T, int NV>
__global__ __launch_bounds__(CE_MAX_THREADS) void ce_cached_kernel(int N, int V, const T* __restrict__ logits,
                                                                   const int32_t* __restrict__ labels,
                                                                   T* __restrict__ dlogits, float* __restrict__ row_loss,
                                                                   float grad_scale) {
  using Vv = Vec16<T>;
  __shared__ float red_m[CE_MAX_THREADS / 64], red_s[CE_MAX_THREADS / 64];
  const int row = blockIdx.x;
  const T* z = logits + (size_t)row * V;
  const int nvec = V / Vv::N;
  const int nt = blockDim.x;
  const int label = labels[row];
  // read before the barrier below, i.e. before any thread of the workgroup overwrites the row (dz may alias z)
  const float z_label = threadIdx.x == 0 ? to_f(z[label]) : 0.f;
  Vv zv[NV];
#pragma unroll
  for (int i = 0; i < NV; i++) {
    const int c = threadIdx.x + i * nt;
    if (c < nvec) zv[i].load(z + (size_t)c * Vv::N);
  }
  // this thread's maximum, then its sum of e^(z - maximum) (differences first, then the scale to base 2)
  float mt = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV; i++) {
    if (threadIdx.x + i * nt < nvec) {
#pragma unroll
      for (int e = 0; e < Vv::N; e++) mt = fmaxf(mt, zv[i].get(e));
    }
  }
  float se = 0.f;
#pragma unroll
  for (int i = 0; i < NV; i++) {
    if (threadIdx.x + i * nt < nvec) {
#pragma unroll
      for (int e = 0; e < Vv::N; e++) se += __builtin_amdgcn_exp2f((zv[i].get(e) - mt) * CE_LOG2E);
    }
  }
  // combine the (maximum, sum) pairs: within the wave, then across waves through LDS.  A thread
  // without elements has maximum -inf and sum 0 and drops out.
  const float mw = wave_max(mt);
  const float sw = wave_sum(mt == -INFINITY ? 0.f : se * __builtin_amdgcn_exp2f((mt - mw) * CE_LOG2E));
  const int wave = threadIdx.x >> 6, nw = nt >> 6;
  if ((threadIdx.x & 63) == 0) {
    red_m[wave] = mw;
    red_s[wave] = sw;
  }
  __syncthreads();
  float M = red_m[0];
  for (int i = 1; i < nw; i++) M = fmaxf(M, red_m[i]);
  float S = 0.f;
  for (int i = 0; i < nw; i++)  // fixed order
    S += red_m[i] == -INFINITY ? 0.f : red_s[i] * __builtin_amdgcn_exp2f((red_m[i] - M) * CE_LOG2E);
  if (threadIdx.x == 0) row_loss[row] = (M + __builtin_amdgcn_logf(S) * CE_LN2) - z_label;  // v_log_f32 is log2
  if (!dlogits) return;
  const float invN = grad_scale / (float)N;
  const float inv = invN / S;
  T* dz = dlogits + (size_t)row * V;
#pragma unroll
  for (int i = 0; i < NV; i++) {
    const int c = threadIdx.x + i * nt;
    if (c < nvec) {
      float g[Vv::N];
#pragma unroll
      for (int e = 0; e < Vv::N; e++) g[e] = __builtin_amdgcn_exp2f((zv[i].get(e) - M) * CE_LOG2E) * inv;
      const int k = label - c * Vv::N;
      if (k >= 0 && k < Vv::N) {  // rare: the vector that holds the label's column
#pragma unroll
        for (int e = 0; e < Vv::N; e++)
          if (e == k) g[e] -= invN;
      }
      Vv o;
#pragma unroll
      for (int e = 0; e < Vv::N; e++) o.set(e, g[e]);
      o.store_nt(dz + (size_t)c * Vv::N);  // gigabytes of gradient: streaming (-3 % on this kernel; the same store for LayerNorm's output cost the next GEMM more than it saved)
    }
  }
}

// Any V: three passes over the row in memory (the re-reads hit cache).
template <typename T>
__global__ __launch_bounds__(CE_MAX_THREADS) void ce_generic_kernel(int N, int V, const T* __restrict__ logits,
                                                                    const int32_t* __restrict__ labels,
                                                                    T* __restrict__ dlogits, float* __restrict__ row_loss,
                                                                    float grad_scale) {
  __shared__ float red[CE_MAX_THREADS / 64];
  const int row = blockIdx.x;
  const T* z = logits + (size_t)row * V;
  T* dz = dlogits + (size_t)row * V;
  const int label = labels[row];
  const float invN = grad_scale / (float)N;
  float mx = -INFINITY;
  for (int c = threadIdx.x; c < V; c += blockDim.x) mx = fmaxf(mx, to_f(z[c]));
  mx = block_reduce(mx, red, true);
  float se = 0.f;
  for (int c = threadIdx.x; c < V; c += blockDim.x) se += expf(to_f(z[c]) - mx);
  se = block_reduce(se, red, false);
  const float inv = invN / se;
  if (threadIdx.x == 0) row_loss[row] = (mx + logf(se)) - to_f(z[label]);
  if (!dlogits) return;
  __syncthreads();  // z[label] is read before anyone overwrites it (dz may alias z)
  for (int c = threadIdx.x; c < V; c += blockDim.x) {
    float g = expf(to_f(z[c]) - mx) * inv;
    if (c == label) g -= invN;
    dz[c] = from_f<T>(g);
  }
}

// loss = mean(row_loss), summed in a fixed order by one block.
__global__ __launch_bounds__(1024) void mean_kernel(int N, const float* __restrict__ v, float* __restrict__ out) {
  __shared__ float red[16];
  float s = 0.f;
  for (int i = threadIdx.x; i < N; i += 1024) s += v[i];
  s = block_reduce(s, red, false);
  if (threadIdx.x == 0) *out = s / (float)N;
}

// Threads per row and vectors per thread for a row of `nvec` 16-byte vectors: the pair with the
// fewest idle vector slots among workgroups of 4 to 16 waves; of equals, the larger workgroup.
static bool ce_shape(int nvec, int* threads, int* nv) {
  long best = -1;
  for (int nt = CE_MAX_THREADS; nt >= 256; nt -= 64) {
    const int v = (nvec + nt - 1) / nt;
    if (v > CE_MAX_NV) continue;
    const int vt = v <= 2 ? 2 : v <= 4 ? 4 : v <= 6 ? 6 : v <= 8 ? 8 : v <= 10 ? 10 : v <= 12 ? 12 : 16;  // instantiated sizes
    const long waste = (long)nt * vt - nvec;
    if (best < 0 || waste < best) {
      best = waste;
      *threads = nt;
      *nv = vt;
    }
  }
  return best >= 0;
}

template <typename T>
static int ce_t(int N, int V, const T* logits, const int32_t* labels, T* dlogits, float* row_loss, float* loss_out,
                float grad_scale, hipStream_t s) {
  constexpr int VN = Vec16<T>::N;
  int nt = 0, nv = 0;
  if (V % VN == 0 && ce_shape(V / VN, &nt, &nv)) {
#define FAX_CE(NVT)                                                                                                  \
  case NVT:                                                                                                          \
    hipLaunchKernelGGL((ce_cached_kernel<T, NVT>), dim3(N), dim3(nt), 0, s, N, V, logits, labels, dlogits, row_loss, \
                       grad_scale);                                                                                  \
    break
    switch (nv) {
      FAX_CE(2); FAX_CE(4); FAX_CE(6); FAX_CE(8); FAX_CE(10); FAX_CE(12); FAX_CE(16);
    }
#undef FAX_CE
  } else {
    hipLaunchKernelGGL((ce_generic_kernel<T>), dim3(N), dim3(CE_MAX_THREADS), 0, s, N, V, logits, labels, dlogits, row_loss,
                       grad_scale);
  }
  FAX_LAUNCH_CHECK("cross_entropy");
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(1024), 0, s, N, row_loss, loss_out);
  FAX_LAUNCH_CHECK("cross_entropy_mean");
  return FAX_OK;
}

int cross_entropy(int dtype, int N, int V, const void* logits, const int32_t* labels, void* dlogits, float* row_loss,
                  float* loss_out, float grad_scale, hipStream_t s) {
  if (N == 0) return FAX_OK;
  Timed t_("cross_entropy", WORK_BYTE, (dlogits ? 2.0 : 1.0) * N * V * (dtype == FAX_F32 ? 4.0 : 2.0), s);
  if (dtype == FAX_F32)
    return ce_t<float>(N, V, (const float*)logits, labels, (float*)dlogits, row_loss, loss_out, grad_scale, s);
  return ce_t<bf16_t>(N, V, (const bf16_t*)logits, labels, (bf16_t*)dlogits, row_loss, loss_out, grad_scale, s);
}

// The same with the per-row losses in a buffer that belongs to the library instead of the caller:
// for callers that cannot allocate (code under graph capture, loops that must not call the
// allocator).  `ce_scratch` is device memory of this code object, one copy per GPU, alive until
// the process ends.  Its name is only a handle on the host: the device address is looked up once
// per device, with that device current, and only that address is passed to kernels.
static __device__ __align__(256) float ce_scratch[CE_STATIC_MAX_ROWS];
static constexpr int MAX_DEVICES = 64;
static float* g_ce_scratch_addr[MAX_DEVICES];  // per device; written once under the mutex
static std::mutex g_ce_scratch_mu;

int cross_entropy_static(int dtype, int N, int V, const void* logits, const int32_t* labels, void* dlogits,
                         float* loss_out, hipStream_t s) {
  if (N > CE_STATIC_MAX_ROWS) {
    set_error("fax_cross_entropy_static: %d rows exceed the built-in scratch of %d rows; use fax_cross_entropy "
              "with a row_loss buffer of your own", N, CE_STATIC_MAX_ROWS);
    return FAX_ERR_WORKSPACE;
  }
  int dev = -1;
  FAX_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) {
    set_error("fax_cross_entropy_static: device ordinal %d not in [0, %d)", dev, MAX_DEVICES);
    return FAX_ERR_UNSUPPORTED;
  }
  float* row_loss;
  {
    std::lock_guard<std::mutex> lk(g_ce_scratch_mu);
    if (!g_ce_scratch_addr[dev]) {
      void* addr = nullptr;
      FAX_HIP(hipGetSymbolAddress(&addr, HIP_SYMBOL(ce_scratch)));
      if (!addr) {
        set_error("fax_cross_entropy_static: no device address for the scratch array on device %d", dev);
        return FAX_ERR_HIP;
      }
      g_ce_scratch_addr[dev] = (float*)addr;
    }
    row_loss = g_ce_scratch_addr[dev];
  }
  // Every row < N of the scratch is written by the row kernel before the mean reads it, and no row
  // >= N is read: nothing has to be cleared between calls.
  return cross_entropy(dtype, N, V, logits, labels, dlogits, row_loss, loss_out, 1.0f, s);
}

// ---------------------------------------------------------------------------------------------
// Embedding
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(int S, int D, const int32_t* __restrict__ tokens,
                                                        const T* __restrict__ tok_emb, const T* __restrict__ pos_emb,
                                                        T* __restrict__ x0) {
  const int t = blockIdx.x;  // token position b*S + s
  const int s = t % S;
  const T* e = tok_emb + (size_t)tokens[t] * D;
  const T* p = pos_emb + (size_t)s * D;
  T* o = x0 + (size_t)t * D;
  for (int d = threadIdx.x; d < D; d += 256) o[d] = from_f<T>(to_f(e[d]) + to_f(p[d]));
}

template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_tok_kernel(int D, const int32_t* __restrict__ tokens,
                                                            const T* __restrict__ dx0, float* __restrict__ g_tok) {
  const int t = blockIdx.x;
  float* g = g_tok + (size_t)tokens[t] * D;
  const T* dx = dx0 + (size_t)t * D;
  for (int d = threadIdx.x; d < D; d += 256) atomicAdd(g + d, to_f(dx[d]));
}

template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_pos_kernel(int B, int S, int D, const T* __restrict__ dx0,
                                                            float* __restrict__ g_pos, int accumulate) {
  const int s = blockIdx.x;
  for (int d = threadIdx.x; d < D; d += 256) {
    float a = accumulate ? g_pos[(size_t)s * D + d] : 0.f;
    for (int b = 0; b < B; b++) a += to_f(dx0[((size_t)b * S + s) * D + d]);
    g_pos[(size_t)s * D + d] = a;
  }
}

int embed_fwd(int dtype, int B, int S, int D, const int32_t* tokens, const void* tok_emb, const void* pos_emb, void* x0,
              hipStream_t s) {
  if (B * S == 0) return FAX_OK;
  Timed t_("embed_fwd", WORK_BYTE, 3.0 * B * S * D * (dtype == FAX_F32 ? 4.0 : 2.0), s);
  if (dtype == FAX_F32)
    hipLaunchKernelGGL((embed_fwd_kernel<float>), dim3(B * S), dim3(256), 0, s, S, D, tokens, (const float*)tok_emb,
                       (const float*)pos_emb, (float*)x0);
  else
    hipLaunchKernelGGL((embed_fwd_kernel<bf16_t>), dim3(B * S), dim3(256), 0, s, S, D, tokens, (const bf16_t*)tok_emb,
                       (const bf16_t*)pos_emb, (bf16_t*)x0);
  FAX_LAUNCH_CHECK("embed_fwd");
  return FAX_OK;
}

// Ordered variant of the token scatter (no floating-point atomics).  Two integer tables over the
// vocabulary are built first: first[v] = the smallest position holding token v, count[v] = how many
// positions hold it (integer min and add commute, so the tables do not depend on the order in
// which the atomics are served).  Then one workgroup per position: the workgroup of first[v] owns
// row v of the gradient and adds the rows of dx0 of all count[v] positions in ascending order.
// It finds them by walking the token array from its own position on in windows of 1024: every
// thread compares four ids and marks its matches in a 1024-bit map in LDS, and the set bits are
// then taken in ascending order by all threads alike.  Columns: a thread keeps EMB_ACC running sums
// (columns tid, tid + 256, ...); rows wider than 256 * EMB_ACC take several passes over the list.
static constexpr int EMB_ACC = 8;
static constexpr int EMB_WIN = 1024;

__global__ __launch_bounds__(256) void embed_index_init_kernel(int V, int* __restrict__ first, int* __restrict__ count) {
  const int v = blockIdx.x * 256 + threadIdx.x;
  if (v < V) {
    first[v] = 0x7fffffff;
    count[v] = 0;
  }
}

__global__ __launch_bounds__(256) void embed_index_kernel(int T, const int32_t* __restrict__ tokens, int* __restrict__ first,
                                                          int* __restrict__ count) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < T) {
    const int v = tokens[t];
    atomicMin(first + v, t);
    atomicAdd(count + v, 1);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_tok_ordered_kernel(int Tn, int D, const int32_t* __restrict__ tokens,
                                                                    const T* __restrict__ dx0, float* __restrict__ g_tok,
                                                                    const int* __restrict__ first,
                                                                    const int* __restrict__ count) {
  __shared__ unsigned map[EMB_WIN / 32];
  const int t = blockIdx.x;
  const int v = tokens[t];
  if (first[v] != t) return;  // uniform over the workgroup: some earlier position owns this row
  const int n = count[v];
  float* g = g_tok + (size_t)v * D;
  for (int d0 = 0; d0 < D; d0 += 256 * EMB_ACC) {
    float acc[EMB_ACC];
#pragma unroll
    for (int k = 0; k < EMB_ACC; k++) acc[k] = 0.f;
    int found = 0;
    for (int base = t; found < n && base < Tn; base += EMB_WIN) {  // uniform; the n positions all lie at or after t
      if (threadIdx.x < EMB_WIN / 32) map[threadIdx.x] = 0u;
      __syncthreads();
#pragma unroll
      for (int j = 0; j < EMB_WIN / 256; j++) {
        const int i = j * 256 + threadIdx.x;
        if (base + i < Tn && tokens[base + i] == v) atomicOr(&map[i >> 5], 1u << (i & 31));
      }
      __syncthreads();
      for (int w = 0; w < EMB_WIN / 32; w++) {
        unsigned bits = map[w];
        while (bits) {
          const int pos = base + w * 32 + __ffs(bits) - 1;
          bits &= bits - 1;
          found++;
          const T* dx = dx0 + (size_t)pos * D + d0;
#pragma unroll
          for (int k = 0; k < EMB_ACC; k++) {
            const int d = threadIdx.x + 256 * k;
            if (d0 + d < D) acc[k] += to_f(dx[d]);
          }
        }
      }
      __syncthreads();  // everyone has read the map before the next window clears it
    }
#pragma unroll
    for (int k = 0; k < EMB_ACC; k++) {
      const int d = d0 + threadIdx.x + 256 * k;
      if (d < D) g[d] += acc[k];
    }
  }
}

size_t embed_index_ws_bytes(int V) { return (size_t)2 * (size_t)V * sizeof(int); }

int embed_bwd(int dtype, int B, int S, int D, int V, const int32_t* tokens, const void* dx0, float* g_tok, float* g_pos,
              bool accumulate_pos, void* index_ws, hipStream_t s) {
  if (B * S == 0) return FAX_OK;
  Timed t_("embed_bwd", WORK_BYTE, 2.0 * B * S * D * (dtype == FAX_F32 ? 4.0 : 2.0) + 8.0 * B * S * D + 4.0 * S * D, s);
  const int T = B * S;
  if (index_ws) {  // ordered reduction
    int* first = (int*)index_ws;
    int* count = first + V;
    hipLaunchKernelGGL(embed_index_init_kernel, dim3((V + 255) / 256), dim3(256), 0, s, V, first, count);
    hipLaunchKernelGGL(embed_index_kernel, dim3((T + 255) / 256), dim3(256), 0, s, T, tokens, first, count);
    if (dtype == FAX_F32)
      hipLaunchKernelGGL((embed_bwd_tok_ordered_kernel<float>), dim3(T), dim3(256), 0, s, T, D, tokens, (const float*)dx0,
                         g_tok, first, count);
    else
      hipLaunchKernelGGL((embed_bwd_tok_ordered_kernel<bf16_t>), dim3(T), dim3(256), 0, s, T, D, tokens, (const bf16_t*)dx0,
                         g_tok, first, count);
  } else if (dtype == FAX_F32) {
    hipLaunchKernelGGL((embed_bwd_tok_kernel<float>), dim3(T), dim3(256), 0, s, D, tokens, (const float*)dx0, g_tok);
  } else {
    hipLaunchKernelGGL((embed_bwd_tok_kernel<bf16_t>), dim3(T), dim3(256), 0, s, D, tokens, (const bf16_t*)dx0, g_tok);
  }
  if (dtype == FAX_F32)
    hipLaunchKernelGGL((embed_bwd_pos_kernel<float>), dim3(S), dim3(256), 0, s, B, S, D, (const float*)dx0, g_pos,
                       accumulate_pos ? 1 : 0);
  else
    hipLaunchKernelGGL((embed_bwd_pos_kernel<bf16_t>), dim3(S), dim3(256), 0, s, B, S, D, (const bf16_t*)dx0, g_pos,
                       accumulate_pos ? 1 : 0);
  FAX_LAUNCH_CHECK("embed_bwd");
  return FAX_OK;
}

// ---------------------------------------------------------------------------------------------
// AdamW: 16 B/param read (g, p, m, v) + 12 B/param written (+2 for the bf16 copy).
// ---------------------------------------------------------------------------------------------
// Streaming stores for values this kernel does not read again.
__device__ __forceinline__ void nt_store4(float4* p, float4 v) {
  typedef __attribute__((ext_vector_type(4))) float f4;
  const f4 x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<f4*>(p));
}
__device__ __forceinline__ void nt_store2(uint2* p, uint2 v) {
  typedef __attribute__((ext_vector_type(2))) unsigned u2;
  const u2 x = {v.x, v.y};
  __builtin_nontemporal_store(x, reinterpret_cast<u2*>(p));
}

struct AdamScalars {
  float b1, b2, one_m_b1, one_m_b2, inv_bc1, inv_bc2, lr, eps, decay;
};

__device__ __forceinline__ void adam_one(float g, float& p, float& m, float& v, const AdamScalars& a) {
  m = a.b1 * m + a.one_m_b1 * g;
  v = a.b2 * v + a.one_m_b2 * g * g;
  const float mh = m * a.inv_bc1;
  const float vh = v * a.inv_bc2;
  p = p * a.decay - a.lr * mh / (sqrtf(vh) + a.eps);
}

// G: the gradient's type, float or bf16_t (a caller that keeps its gradients in the compute precision)
template <typename G>
__global__ __launch_bounds__(256) void adamw_kernel(size_t n, float* __restrict__ p, float* __restrict__ m,
                                                    float* __restrict__ v, const G* __restrict__ g,
                                                    bf16_t* __restrict__ lowp, AdamScalars a) {
  const size_t nvec = n / 4;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride) {
    float4 pv = reinterpret_cast<float4*>(p)[i], mv = reinterpret_cast<float4*>(m)[i];
    float4 vv = reinterpret_cast<float4*>(v)[i];
    float4 gv;
    if constexpr (sizeof(G) == 4) {
      gv = reinterpret_cast<const float4*>(g)[i];
    } else {
      union { uint2 u; bf16_t h[4]; } gk;
      gk.u = reinterpret_cast<const uint2*>(g)[i];
      gv = make_float4((float)gk.h[0], (float)gk.h[1], (float)gk.h[2], (float)gk.h[3]);
    }
    adam_one(gv.x, pv.x, mv.x, vv.x, a);
    adam_one(gv.y, pv.y, mv.y, vv.y, a);
    adam_one(gv.z, pv.z, mv.z, vv.z, a);
    adam_one(gv.w, pv.w, mv.w, vv.w, a);
    nt_store4(reinterpret_cast<float4*>(p) + i, pv);
    nt_store4(reinterpret_cast<float4*>(m) + i, mv);
    nt_store4(reinterpret_cast<float4*>(v) + i, vv);
    if (lowp) {
      union { bf16_t h[4]; uint2 u; } pk;
      pk.h[0] = (bf16_t)pv.x; pk.h[1] = (bf16_t)pv.y; pk.h[2] = (bf16_t)pv.z; pk.h[3] = (bf16_t)pv.w;
      nt_store2(reinterpret_cast<uint2*>(lowp) + i, pk.u);
    }
  }
  // ragged tail
  for (size_t i = nvec * 4 + (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    float pp = p[i], mm = m[i], vv = v[i];
    adam_one((float)g[i], pp, mm, vv, a);
    p[i] = pp; m[i] = mm; v[i] = vv;
    if (lowp) lowp[i] = (bf16_t)pp;
  }
}

static AdamScalars adam_scalars(const FaxAdamW& hp, int step);

int adamw(float* master, float* m, float* v, const void* grad, int grad_dtype, void* lowp, size_t n, const FaxAdamW& hp,
          int step, hipStream_t s) {
  if (n == 0) return FAX_OK;
  Timed t_("adamw", WORK_BYTE, ((lowp ? 30.0 : 28.0) - (grad_dtype == FAX_BF16 ? 2.0 : 0.0)) * (double)n, s);
  const AdamScalars a = adam_scalars(hp, step);
  size_t blocks = (n / 4 + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (grad_dtype == FAX_BF16)
    hipLaunchKernelGGL(adamw_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, s, n, master, m, v, (const bf16_t*)grad,
                       (bf16_t*)lowp, a);
  else
    hipLaunchKernelGGL(adamw_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s, n, master, m, v, (const float*)grad,
                       (bf16_t*)lowp, a);
  FAX_LAUNCH_CHECK("adamw");
  return FAX_OK;
}

// Several tensors per launch: a model has a dozen tensors per layer, most of them a few KB, and a
// launch per tensor costs more than their update.  Workgroup w works on chunk w - first[t] (4096
// elements) of the tensor t whose range of workgroups contains w.
__global__ __launch_bounds__(256) void adamw_multi_kernel(AdamWBatch b, AdamScalars a) {
  int t = 0;
  while (t + 1 < b.count && blockIdx.x >= b.first[t + 1]) t++;  // uniform over the workgroup
  const size_t n = b.n[t], nvec = n / 4;
  float* const p = b.p[t];
  float* const m = b.m[t];
  float* const v = b.v[t];
  const float* const g = b.g[t];
  bf16_t* const lowp = b.lowp[t];
  const size_t chunk = blockIdx.x - b.first[t];
#pragma unroll
  for (int k = 0; k < ADAM_CHUNK / 1024; k++) {
    const size_t i = chunk * (ADAM_CHUNK / 4) + k * 256 + threadIdx.x;
    if (i < nvec) {
      float4 pv = reinterpret_cast<float4*>(p)[i], mv = reinterpret_cast<float4*>(m)[i];
      float4 vv = reinterpret_cast<float4*>(v)[i];
      const float4 gv = reinterpret_cast<const float4*>(g)[i];
      adam_one(gv.x, pv.x, mv.x, vv.x, a);
      adam_one(gv.y, pv.y, mv.y, vv.y, a);
      adam_one(gv.z, pv.z, mv.z, vv.z, a);
      adam_one(gv.w, pv.w, mv.w, vv.w, a);
      nt_store4(reinterpret_cast<float4*>(p) + i, pv);
      nt_store4(reinterpret_cast<float4*>(m) + i, mv);
      nt_store4(reinterpret_cast<float4*>(v) + i, vv);
      if (lowp) {
        union { bf16_t h[4]; uint2 u; } pk;
        pk.h[0] = (bf16_t)pv.x; pk.h[1] = (bf16_t)pv.y; pk.h[2] = (bf16_t)pv.z; pk.h[3] = (bf16_t)pv.w;
        nt_store2(reinterpret_cast<uint2*>(lowp) + i, pk.u);
      }
    }
  }
  // ragged tail (at most three elements), by the tensor's last workgroup
  const size_t i = nvec * 4 + threadIdx.x;
  if (blockIdx.x + 1 == b.first[t + 1] && i < n) {
    float pp = p[i], mm = m[i], vv = v[i];
    adam_one(g[i], pp, mm, vv, a);
    p[i] = pp; m[i] = mm; v[i] = vv;
    if (lowp) lowp[i] = (bf16_t)pp;
  }
}

static AdamScalars adam_scalars(const FaxAdamW& hp, int step) {
  AdamScalars a;
  a.b1 = (float)hp.beta1; a.b2 = (float)hp.beta2;
  a.one_m_b1 = (float)(1.0 - hp.beta1); a.one_m_b2 = (float)(1.0 - hp.beta2);
  a.inv_bc1 = (float)(1.0 / (1.0 - pow(hp.beta1, (double)step)));
  a.inv_bc2 = (float)(1.0 / (1.0 - pow(hp.beta2, (double)step)));
  a.lr = (float)hp.lr; a.eps = (float)hp.eps;
  a.decay = (float)(1.0 - hp.lr * hp.wd);
  return a;
}

int AdamWQueue::add(float* master, float* m, float* v, const float* grad, void* lowp, size_t n) {
  if (n == 0) return FAX_OK;
  const size_t chunks = (n + ADAM_CHUNK - 1) / ADAM_CHUNK;
  if (chunks > 0x7fffffffu) {
    set_error("adamw: tensor of %zu elements", n);
    return FAX_ERR_UNSUPPORTED;
  }
  if (b.count == ADAM_BATCH || (size_t)b.first[b.count] + chunks > 0x7fffffffu) FAX_TRY(flush());
  const int t = b.count++;
  b.p[t] = master; b.m[t] = m; b.v[t] = v; b.g[t] = grad; b.lowp[t] = (bf16_t*)lowp; b.n[t] = n;
  b.first[t + 1] = b.first[t] + (unsigned)chunks;
  bytes += (lowp ? 30.0 : 28.0) * (double)n;
  return FAX_OK;
}

int AdamWQueue::flush() {
  if (b.count == 0) return FAX_OK;
  {
    Timed t_("adamw", WORK_BYTE, bytes, s);
    hipLaunchKernelGGL(adamw_multi_kernel, dim3(b.first[b.count]), dim3(256), 0, s, b, adam_scalars(hp, step));
    FAX_LAUNCH_CHECK("adamw");
  }
  b.count = 0;
  b.first[0] = 0;
  bytes = 0;
  return FAX_OK;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* __restrict__ p, size_t nvec, size_t bytes) {
  const size_t stride = (size_t)gridDim.x * 256;
  const size_t first = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (size_t i = first; i < nvec; i += stride) p[i] = make_uint4(0, 0, 0, 0);
  unsigned char* tail = reinterpret_cast<unsigned char*>(p);
  for (size_t i = nvec * 16 + first; i < bytes; i += stride) tail[i] = 0;
}

// p must be 16-byte aligned; any byte count.
int fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return FAX_OK;
  size_t nvec = bytes / 16;
  size_t blocks = (nvec + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)p, nvec, bytes);
  FAX_LAUNCH_CHECK("fill_zero");
  return FAX_OK;
}

}  // namespace fax
