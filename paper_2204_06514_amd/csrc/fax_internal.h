// Internal declarations shared by the kernel files and the C-ABI layer of libfax.
// Target: gfx950 (CDNA4) only; wavefront = 64 lanes.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/fax.h"

namespace fax {

typedef __bf16 bf16_t;

// ---- error text for the calling thread -------------------------------------------------
void set_error(const char* fmt, ...);
int hip_fail(hipError_t e, const char* what);

#define FAX_HIP(call)                                   \
  do {                                                  \
    hipError_t e_ = (call);                             \
    if (e_ != hipSuccess) return fax::hip_fail(e_, #call); \
  } while (0)
#define FAX_TRY(call)          \
  do {                         \
    int s_ = (call);           \
    if (s_ != FAX_OK) return s_; \
  } while (0)
#define FAX_LAUNCH_CHECK(name) FAX_HIP(hipGetLastError())

// ---- GEMM -------------------------------------------------------------------------------
enum { EPI_NONE = 0, EPI_GELU = 1, EPI_DGELU = 2 };
enum { PATH_AUTO = 0, PATH_SIMT = 1, PATH_MFMA = 2 };

// C[M,N] = op(A) op(B) in fp32, then (in this order):
//   C2 = acc                       (EPI_NONE with C2: the pre-bias partial product)
//   acc += bias[n]; acc += R[m,n]
//   EPI_GELU : C = gelu'(acc), C2 = gelu(acc)   (the backward pass needs the derivative, never acc itself)
//   EPI_DGELU: C = acc * U[m,n]                 (U: the derivative stored by EPI_GELU)
//   otherwise: C = acc (fp32 C may accumulate)
struct GemmArgs {
  int dtype = FAX_BF16;
  bool ta = false, tb = false;
  int M = 0, N = 0, K = 0;
  const void* A = nullptr; int lda = 0;
  const void* B = nullptr; int ldb = 0;
  void* C = nullptr; int ldc = 0;
  bool c_f32 = false, accumulate = false;
  const void* bias = nullptr;
  const void* R = nullptr; int ldr = 0;
  int epi = EPI_NONE;
  void* C2 = nullptr; int ldc2 = 0;
  const void* U = nullptr; int ldu = 0;
  int gelu_form = FAX_GELU_TANH;
  int path = PATH_AUTO;
  // Optional by-product, B stored [K, N] only: colsum[n] (+)= sum over k of B[k, n] (`accumulate`
  // applies to it as well).  colsum_ws: colsum_ws_bytes(N) of scratch for the paths that take the
  // sums in a separate pass.
  float* colsum = nullptr;
  void* colsum_ws = nullptr;
  // Scratch for splitting the contraction (fp32-output form only): gemm_split_ws_bytes(M, N, K)
  // bytes, or NULL to forbid the split.
  void* split_ws = nullptr;
};
int gemm(const GemmArgs& g, hipStream_t s);
int gemm_simt(const GemmArgs& g, hipStream_t s);
bool gemm_mfma_supported(const GemmArgs& g);
// A weight-gradient product of a narrow model has few output tiles and a very long contraction
// (K = all tokens): it is then cut into K ranges, each a full set of tiles writing its own fp32
// partial product (and partial column sums), summed afterwards in a fixed order.  The plan (tile
// class, number of ranges; 1 = no split) comes from a small cost model of the kernel.
struct GemmSplitPlan {
  int tile_m, tile_n;  // 256 x 256, 256 x 128 or 128 x 128; 0: no tile class divides the shape
  int splits;
};
GemmSplitPlan gemm_split_plan(int M, int N, int K);
size_t gemm_split_ws_bytes(int M, int N, int K);
GemmSplitPlan gemm_plan_query(int M, int N, int K, bool f32_out, int* tail);
int gemm_tile_walk_query(int M, int N, int K, bool f32_out, int* tm, int* tn, int capacity, int* count, int* group);
// Predicted duration of gemm() on this shape from the same cost model (host only), microseconds.
double gemm_time_estimate_us(int M, int N, int K, bool f32_out);
int gemm_mfma(const GemmArgs& g, hipStream_t s);

// ---- LayerNorm, column sums ---------------------------------------------------------------
int ln_fwd(int dtype, int rows, int D, const void* x, const void* gamma, const void* beta, float eps,
           void* h, float* mu, float* rstd, hipStream_t s);
size_t ln_bwd_ws_bytes(int D);
int ln_bwd(int dtype, int rows, int D, const void* dh, const void* x, const float* mu, const float* rstd,
           const void* gamma, const void* dres, void* dx, float* dgamma, float* dbeta, bool accumulate,
           void* ws, hipStream_t s, hipStream_t fold_s = nullptr, hipEvent_t handover = nullptr);
// (fold_s, handover: optionally a second stream for the fold of the partial rows, which feeds only
// dgamma / dbeta, and an event to order it behind the row kernel; `ws` then stays in use until that
// stream has run the fold)
size_t colsum_ws_bytes(int N);
// out[i] (+)= sum_p partial[p * n + i], p < parts, in that order
// out[i] (+)= sum over p < parts of partial[p * n + i]; optionally a second stack (nb elements per part) into
// out_b in the same launch.  Fixed summation order.
int fold_partials(int parts, size_t n, const float* partial, float* out, bool accumulate, hipStream_t s, int nb = 0,
                  const float* partial_b = nullptr, float* out_b = nullptr);
// out[n] (+)= sum over rows of a[r, n]; a in dtype with leading dimension lda.
int colsum(int dtype, int rows, int N, const void* a, int lda, float* out, bool accumulate, void* ws,
           hipStream_t s);

// ---- attention ------------------------------------------------------------------------------
int attn_fwd_simt(int dtype, int B, int S, int H, int dh, const void* qkv, void* ctx, float* lse, hipStream_t s);
int attn_bwd_simt(int dtype, int B, int S, int H, int dh, const void* qkv, const void* ctx, const float* lse,
                  const void* dctx, void* dqkv, float* delta, hipStream_t s);
// delta[b,h,i] = sum_d dctx[b,i,h,d] ctx[b,i,h,d]
int attn_delta(int dtype, int B, int S, int H, int dh, const void* ctx, const void* dctx, float* delta, hipStream_t s);
bool attn_mfma_supported(int dtype, int B, int S, int H, int dh);
int attn_fwd_mfma(int B, int S, int H, int dh, const void* qkv, void* ctx, float* lse, hipStream_t s);
// Optional: scratch for the dQ kernel's own copy of delta ([B,H,S] fp32) and a second stream with two
// events; given them, and few enough workgroups (attn_bwd_side_by_side), dQ and dK/dV run side by side.
struct AttnBwdSplit {
  float* delta_scratch;
  hipStream_t side;
  hipEvent_t fork, join;
};
bool attn_bwd_side_by_side(int B, int S, int H);
int attn_bwd_mfma(int B, int S, int H, int dh, const void* qkv, const void* ctx, const float* lse,
                  const void* dctx, void* dqkv, float* delta, hipStream_t s, const AttnBwdSplit* split = nullptr);

// ---- loss, embedding, optimizer ---------------------------------------------------------------
// dlogits = grad_scale (softmax - onehot) / N, may alias logits, NULL for the loss alone
int cross_entropy(int dtype, int N, int V, const void* logits, const int32_t* labels, void* dlogits,
                  float* row_loss, float* loss_out, float grad_scale, hipStream_t s);
// Per-row losses in a file-scope device array of the library (CE_STATIC_MAX_ROWS floats, 1 MiB per GPU).
constexpr int CE_STATIC_MAX_ROWS = 1 << 18;
int cross_entropy_static(int dtype, int N, int V, const void* logits, const int32_t* labels, void* dlogits,
                         float* loss_out, hipStream_t s);
int embed_fwd(int dtype, int B, int S, int D, const int32_t* tokens, const void* tok_emb, const void* pos_emb,
              void* x0, hipStream_t s);
// g_tok[tokens[b,s]] += dx0[b,s]; g_pos[s] (+)= sum_b dx0[b,s]; rows of g_pos beyond S untouched.
// index_ws = NULL: fp32 atomics (the order of the additions into a row is the hardware's).
// index_ws = embed_index_ws_bytes(V) bytes of scratch: one writer per row, positions in ascending order.
size_t embed_index_ws_bytes(int V);
int embed_bwd(int dtype, int B, int S, int D, int V, const int32_t* tokens, const void* dx0, float* g_tok, float* g_pos,
              bool accumulate_pos, void* index_ws, hipStream_t s);
// Up to ADAM_BATCH tensors per launch.  add() queues a tensor (launching what is queued when the
// batch is full), flush() launches the rest; nothing is kept beyond flush().
constexpr int ADAM_BATCH = 16;
constexpr int ADAM_CHUNK = 4096;  // elements per workgroup
struct AdamWBatch {
  float* p[ADAM_BATCH];
  float* m[ADAM_BATCH];
  float* v[ADAM_BATCH];
  const float* g[ADAM_BATCH];
  bf16_t* lowp[ADAM_BATCH];
  size_t n[ADAM_BATCH];
  unsigned first[ADAM_BATCH + 1];  // first workgroup of each tensor; first[count] = grid size
  int count;
};
struct AdamWQueue {
  AdamWQueue(const FaxAdamW& hp_, int step_, hipStream_t s_) : hp(hp_), step(step_), s(s_) {
    b.count = 0;
    b.first[0] = 0;
  }
  int add(float* master, float* m, float* v, const float* grad, void* lowp, size_t n);
  int flush();
  AdamWBatch b;
  FaxAdamW hp;
  int step;
  hipStream_t s;
  double bytes = 0;
};
int adamw(float* master, float* m, float* v, const void* grad, int grad_dtype, void* lowp, size_t n, const FaxAdamW& hp,
          int step, hipStream_t s);
int fill_zero(void* p, size_t bytes, hipStream_t s);

// ---- measured ceilings (probes.hip) ---------------------------------------------------------------
int probe_mfma(int workgroups, int iters, unsigned seed, float* sink, hipStream_t s);
int probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s);

// ---- optional per-kernel timing (see fax_timing_enable) ------------------------------------
enum { WORK_FLOP = 0, WORK_BYTE = 1 };
bool timing_on();
void timing_begin(const char* name, int unit, double work, hipStream_t s, void** token);
void timing_end(void* token, hipStream_t s);
struct Timed {
  void* token = nullptr;
  hipStream_t s;
  Timed(const char* name, int unit, double work, hipStream_t stream) : s(stream) {
    if (timing_on()) timing_begin(name, unit, work, s, &token);
  }
  ~Timed() {
    if (token) timing_end(token, s);
  }
};

// ---- device helpers -----------------------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return (bf16_t)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// 16-byte vector of T: 4 floats or 8 bf16.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ __forceinline__ void load(const float* p) { raw = *reinterpret_cast<const float4*>(p); }
  __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<float4*>(p) = raw; }
  // streaming store: for values that are too large to be found in a cache by whoever reads them next
  __device__ __forceinline__ void store_nt(float* p) const {
    typedef __attribute__((ext_vector_type(4))) float f4;
    const f4 x = {raw.x, raw.y, raw.z, raw.w};
    __builtin_nontemporal_store(x, reinterpret_cast<f4*>(p));
  }
  __device__ __forceinline__ float get(int i) const { return reinterpret_cast<const float*>(&raw)[i]; }
  __device__ __forceinline__ void set(int i, float v) { reinterpret_cast<float*>(&raw)[i] = v; }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ __forceinline__ void load(const bf16_t* p) { raw = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void store(bf16_t* p) const { *reinterpret_cast<uint4*>(p) = raw; }
  __device__ __forceinline__ void store_nt(bf16_t* p) const {
    typedef __attribute__((ext_vector_type(4))) unsigned u4;
    const u4 x = {raw.x, raw.y, raw.z, raw.w};
    __builtin_nontemporal_store(x, reinterpret_cast<u4*>(p));
  }
  __device__ __forceinline__ float get(int i) const {
    uint32_t w = reinterpret_cast<const uint32_t*>(&raw)[i >> 1];
    return __uint_as_float((i & 1) ? (w & 0xffff0000u) : (w << 16));
  }
  __device__ __forceinline__ void set(int i, float v) { reinterpret_cast<bf16_t*>(&raw)[i] = (bf16_t)v; }
};

// GELU, both forms, and its derivative.
__device__ __forceinline__ float gelu_f(float u, int form) {
  if (form == FAX_GELU_TANH) {
    float t = tanhf(0.7978845608028654f * (u + 0.044715f * u * u * u));
    return 0.5f * u * (1.0f + t);
  }
  return 0.5f * u * (1.0f + erff(u * 0.7071067811865476f));
}
__device__ __forceinline__ float gelu_grad_f(float u, int form) {
  if (form == FAX_GELU_TANH) {
    float t = tanhf(0.7978845608028654f * (u + 0.044715f * u * u * u));
    return 0.5f * (1.0f + t) + 0.5f * u * (1.0f - t * t) * 0.7978845608028654f * (1.0f + 0.134145f * u * u);
  }
  float cdf = 0.5f * (1.0f + erff(u * 0.7071067811865476f));
  float pdf = 0.3989422804014327f * expf(-0.5f * u * u);
  return cdf + u * pdf;
}
// ---- direct global -> LDS loads ---------------------------------------------------------------
// global_load_lds_dwordx4: each lane names 16 bytes of global memory; the wave's 1024 bytes land
// in LDS at M0 + 16 * lane.  No destination registers and no LDS store instructions.  Issued
// through inline assembly because the compiler, given the builtin, waits for every outstanding
// load of this kind before each later LDS read that it cannot prove disjoint -- here all of them,
// which would expose the full memory latency.  In exchange the completion wait is explicit:
// lds_dma_wait() (vmcnt drains when the data is in LDS) must precede the barrier that publishes
// the buffer.  `lds_segment` must be wave-uniform.  M0 is not otherwise used by these kernels.
// lds_addr(): the 32-bit LDS address of a pointer into shared memory (take it once per kernel).
__device__ __forceinline__ unsigned lds_addr(const void* shared_ptr) {
  return (unsigned)(__UINTPTR_TYPE__)(__attribute__((address_space(3))) const char*)shared_ptr;
}
__device__ __forceinline__ void lds_dma16(const void* global_src, unsigned lds_segment_addr) {
  const unsigned dst = __builtin_amdgcn_readfirstlane(lds_segment_addr);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(dst), "v"(global_src) : "memory");
}
// Same, with the address split into a wave-uniform base (scalar registers) and a 32-bit per-lane
// byte offset: a loop that walks the base forward then needs no vector arithmetic per load.
__device__ __forceinline__ void lds_dma16(const void* uniform_base, unsigned lane_byte_offset, unsigned lds_segment_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               : : "s"(lds_segment_addr), "v"(lane_byte_offset), "s"(uniform_base) : "memory");
}
// 4 bytes per lane: the wave's 256 bytes land at M0 + 4 * lane.
__device__ __forceinline__ void lds_dma4(const void* global_src, unsigned lds_segment_addr) {
  const unsigned dst = __builtin_amdgcn_readfirstlane(lds_segment_addr);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" : : "s"(dst), "v"(global_src) : "memory");
}
__device__ __forceinline__ void lds_dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---- GEMM epilogue shared by the scalar and MFMA kernels ----
struct EpiArgs {
  const void* bias;
  const void* R; int ldr;
  void* C; int ldc;
  void* C2; int ldc2;
  const void* U; int ldu;
  int epi, gelu_form, c_f32, accumulate;
  float* colsum;
  int splits;           // K ranges (fp32-output form); range r writes to C + r * split_stride
  size_t split_stride;  // in elements
  size_t colsum_stride; // likewise for the column sums: range r writes colsum + r * colsum_stride
  int group;            // tile rows per column-major group of the tile walk (MFMA kernel)
};

template <typename T>
__device__ __forceinline__ void epilogue_store(const EpiArgs& e, int m, int n, float acc) {
  if (e.epi == EPI_NONE && e.C2) ((T*)e.C2)[(size_t)m * e.ldc2 + n] = from_f<T>(acc);
  if (e.bias) acc += to_f(((const T*)e.bias)[n]);
  if (e.R) acc += to_f(((const T*)e.R)[(size_t)m * e.ldr + n]);
  if (e.epi == EPI_GELU) {
    ((T*)e.C)[(size_t)m * e.ldc + n] = from_f<T>(gelu_grad_f(acc, e.gelu_form));
    ((T*)e.C2)[(size_t)m * e.ldc2 + n] = from_f<T>(gelu_f(acc, e.gelu_form));
  } else {
    if (e.epi == EPI_DGELU) acc *= to_f(((const T*)e.U)[(size_t)m * e.ldu + n]);
    if (e.c_f32) {
      float* c = (float*)e.C + (size_t)m * e.ldc + n;
      *c = e.accumulate ? *c + acc : acc;
    } else {
      ((T*)e.C)[(size_t)m * e.ldc + n] = from_f<T>(acc);
    }
  }
}

#endif  // __HIPCC__

}  // namespace fax
