// C-ABI layer: argument validation, buffer layouts, and the order in which kernels are enqueued.
// Everything here runs on the host; validation precedes the first launch.
#include <cstdarg>
#include <cstdio>
#include <atomic>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "fax_internal.h"

namespace fax {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int hip_fail(hipError_t e, const char* what) {
  set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
  return FAX_ERR_HIP;
}

// ---- per-kernel timing ------------------------------------------------------------------------
struct TimingRecord {
  std::string name;
  int unit;
  double work;
  hipEvent_t start, stop;
};
static std::mutex g_timing_mu;
static std::atomic<bool> g_timing_on{false};
static std::vector<TimingRecord*> g_timing;

bool timing_on() { return g_timing_on.load(std::memory_order_relaxed); }

void timing_begin(const char* name, int unit, double work, hipStream_t s, void** token) {
  TimingRecord* r = new TimingRecord{name, unit, work, nullptr, nullptr};
  if (hipEventCreate(&r->start) != hipSuccess || hipEventCreate(&r->stop) != hipSuccess ||
      hipEventRecord(r->start, s) != hipSuccess) {
    if (r->start) (void)hipEventDestroy(r->start);
    if (r->stop) (void)hipEventDestroy(r->stop);
    delete r;
    return;
  }
  *token = r;
}

void timing_end(void* token, hipStream_t s) {
  TimingRecord* r = static_cast<TimingRecord*>(token);
  (void)hipEventRecord(r->stop, s);
  std::lock_guard<std::mutex> lk(g_timing_mu);
  g_timing.push_back(r);
}

static void timing_clear() {
  std::lock_guard<std::mutex> lk(g_timing_mu);
  for (TimingRecord* r : g_timing) {
    (void)hipEventDestroy(r->start);
    (void)hipEventDestroy(r->stop);
    delete r;
  }
  g_timing.clear();
}

static inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
static inline size_t esize(int dtype) { return dtype == FAX_F32 ? 4 : 2; }
static inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

static int check_dims(const FaxBlockDims* d) {
  if (!d) {
    set_error("dims is NULL");
    return FAX_ERR_INVALID_ARG;
  }
  if (d->B <= 0 || d->S <= 0 || d->D <= 0 || d->H <= 0 || d->dh <= 0 || d->F <= 0) {
    set_error("non-positive dimension: B=%d S=%d D=%d H=%d dh=%d F=%d", d->B, d->S, d->D, d->H, d->dh, d->F);
    return FAX_ERR_INVALID_ARG;
  }
  if (d->dtype != FAX_F32 && d->dtype != FAX_BF16) {
    set_error("dtype %d is neither FAX_F32 nor FAX_BF16", d->dtype);
    return FAX_ERR_INVALID_ARG;
  }
  if (d->gelu != FAX_GELU_TANH && d->gelu != FAX_GELU_ERF) {
    set_error("gelu %d is neither FAX_GELU_TANH nor FAX_GELU_ERF", d->gelu);
    return FAX_ERR_INVALID_ARG;
  }
  if (!(d->ln_eps >= 0.f)) {
    set_error("ln_eps must be >= 0");
    return FAX_ERR_INVALID_ARG;
  }
  if ((long long)d->B * d->S > (1ll << 30) || (long long)d->H * d->dh * 3 > (1ll << 30)) {
    set_error("B*S or 3*H*dh exceeds 2^30");
    return FAX_ERR_INVALID_ARG;
  }
  if (d->dh > 256) {
    set_error("head width %d exceeds 256", d->dh);
    return FAX_ERR_UNSUPPORTED;
  }
  return FAX_OK;
}

struct Sizes {
  size_t T, D, Hd, F, es;
  explicit Sizes(const FaxBlockDims& d)
      : T((size_t)d.B * d.S), D(d.D), Hd((size_t)d.H * d.dh), F(d.F), es(esize(d.dtype)) {}
};

static void saved_layout(const FaxBlockDims& d, FaxSavedLayout* L) {
  Sizes z(d);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += align_up(bytes); return r; };
  L->h1 = take(z.T * z.D * z.es);
  L->qkv = take(z.T * 3 * z.Hd * z.es);
  L->ctx = take(z.T * z.Hd * z.es);
  L->lse = take((size_t)d.B * d.H * d.S * 4);
  L->x1 = take(z.T * z.D * z.es);
  L->h2 = take(z.T * z.D * z.es);
  L->dgelu = take(z.T * z.F * z.es);
  L->a = take(z.T * z.F * z.es);
  L->mu1 = take(z.T * 4);
  L->rstd1 = take(z.T * 4);
  L->mu2 = take(z.T * 4);
  L->rstd2 = take(z.T * 4);
  L->total = o;
}

struct BwdWs {
  FaxBwdLayout pub;
  size_t delta, delta2, red, red_ln1, red_side, splitk, total;
};

static void bwd_layout(const FaxBlockDims& d, BwdWs* W) {
  Sizes z(d);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += align_up(bytes); return r; };
  W->pub.du = take(z.T * z.F * z.es);
  W->pub.dh2 = take(z.T * z.D * z.es);
  W->pub.dx1 = take(z.T * z.D * z.es);
  W->pub.dctx = take(z.T * z.Hd * z.es);
  W->pub.dqkv = take(z.T * 3 * z.Hd * z.es);
  W->pub.dh1 = take(z.T * z.D * z.es);
  W->delta = take((size_t)d.B * d.H * d.S * 4);
  W->delta2 = take((size_t)d.B * d.H * d.S * 4);  // the dQ kernel's own copy when delta comes from a kernel of its own
  size_t widest = z.D;
  if (z.F > widest) widest = z.F;
  if (3 * z.Hd > widest) widest = 3 * z.Hd;
  size_t red = ln_bwd_ws_bytes(d.D);
  if (colsum_ws_bytes((int)widest) > red) red = colsum_ws_bytes((int)widest);
  W->red = take(red);
  W->red_ln1 = take(ln_bwd_ws_bytes(d.D));  // LN1's partial rows: LN2's may still await their fold on the second stream
  W->red_side = take(colsum_ws_bytes((int)widest));  // column-sum scratch of the weight-gradient stream
  // scratch for the weight-gradient products whose contraction gets split (narrow models)
  const int T = (int)z.T, D = (int)z.D, Hd = (int)z.Hd, F = (int)z.F;
  size_t sk = gemm_split_ws_bytes(F, D, T);
  sk = std::max(sk, gemm_split_ws_bytes(D, F, T));
  sk = std::max(sk, gemm_split_ws_bytes(Hd, D, T));
  sk = std::max(sk, gemm_split_ws_bytes(D, 3 * Hd, T));
  W->splitk = take(sk);
  W->total = o;
  W->pub.total = o;
}

static const void* const* tensor_list(const FaxBlockTensors* t) { return reinterpret_cast<const void* const*>(t); }
static const char* const kTensorNames[12] = {"ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
                                              "ln2_g", "ln2_b", "w1",   "b1",   "w2", "b2"};

static void tensor_counts(const FaxBlockDims& d, size_t n[12]) {
  Sizes z(d);
  n[0] = z.D; n[1] = z.D; n[2] = z.D * 3 * z.Hd; n[3] = 3 * z.Hd; n[4] = z.Hd * z.D; n[5] = z.D;
  n[6] = z.D; n[7] = z.D; n[8] = z.D * z.F; n[9] = z.F; n[10] = z.F * z.D; n[11] = z.D;
}

static int check_tensors(const FaxBlockTensors* t, const char* what) {
  if (!t) {
    set_error("%s is NULL", what);
    return FAX_ERR_INVALID_ARG;
  }
  const void* const* p = tensor_list(t);
  for (int i = 0; i < 12; i++) {
    if (!p[i]) {
      set_error("%s.%s is NULL", what, kTensorNames[i]);
      return FAX_ERR_INVALID_ARG;
    }
    if (misaligned(p[i])) {
      set_error("%s.%s is not 16-byte aligned", what, kTensorNames[i]);
      return FAX_ERR_INVALID_ARG;
    }
  }
  return FAX_OK;
}

static int check_ptr(const void* p, const char* name) {
  if (!p) {
    set_error("%s is NULL", name);
    return FAX_ERR_INVALID_ARG;
  }
  if (misaligned(p)) {
    set_error("%s is not 16-byte aligned", name);
    return FAX_ERR_INVALID_ARG;
  }
  return FAX_OK;
}

static int check_adamw(const FaxAdamW* hp, int step) {
  if (!hp) {
    set_error("hp is NULL");
    return FAX_ERR_INVALID_ARG;
  }
  if (step < 1) {
    set_error("step must be >= 1, got %d", step);
    return FAX_ERR_INVALID_ARG;
  }
  if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0 && hp->beta2 >= 0.0 && hp->beta2 < 1.0)) {
    set_error("betas must lie in [0, 1)");  // beta = 1 would make the bias correction infinite
    return FAX_ERR_INVALID_ARG;
  }
  if (!(hp->eps >= 0.0) || hp->lr != hp->lr || hp->wd != hp->wd) {
    set_error("eps must be >= 0 and lr, wd must be numbers");
    return FAX_ERR_INVALID_ARG;
  }
  return FAX_OK;
}

static int attention_fwd(int dtype, int B, int S, int H, int dh, const void* qkv, void* ctx, float* lse, int path,
                         hipStream_t s) {
  const bool ok = attn_mfma_supported(dtype, B, S, H, dh);
  if (path == PATH_MFMA && !ok) {
    set_error("attention: dtype %d, S=%d, dh=%d is not covered by the MFMA kernel", dtype, S, dh);
    return FAX_ERR_UNSUPPORTED;
  }
  const bool mfma = ok && path != PATH_SIMT;
  Timed t_(mfma ? "attention_fwd_mfma" : "attention_fwd_scalar", WORK_FLOP, 2.0 * B * H * (double)S * S * dh, s);
  if (mfma) return attn_fwd_mfma(B, S, H, dh, qkv, ctx, lse, s);
  return attn_fwd_simt(dtype, B, S, H, dh, qkv, ctx, lse, s);
}

static int attention_bwd(int dtype, int B, int S, int H, int dh, const void* qkv, const void* ctx, const float* lse,
                         const void* dctx, void* dqkv, float* delta, int path, hipStream_t s,
                         const AttnBwdSplit* split = nullptr) {
  const bool ok = attn_mfma_supported(dtype, B, S, H, dh);
  if (path == PATH_MFMA && !ok) {
    set_error("attention: dtype %d, S=%d, dh=%d is not covered by the MFMA kernel", dtype, S, dh);
    return FAX_ERR_UNSUPPORTED;
  }
  const bool mfma = ok && path != PATH_SIMT;
  Timed t_(mfma ? "attention_bwd_mfma" : "attention_bwd_scalar", WORK_FLOP, 4.0 * B * H * (double)S * S * dh, s);
  if (mfma) return attn_bwd_mfma(B, S, H, dh, qkv, ctx, lse, dctx, dqkv, delta, s, split);
  return attn_bwd_simt(dtype, B, S, H, dh, qkv, ctx, lse, dctx, dqkv, delta, s);
}

// ---- block forward --------------------------------------------------------------------------
static int block_fwd_impl(const FaxBlockDims& d, const FaxBlockTensors& p, const void* x, void* y, char* saved,
                          void* p_attn, void* p_mlp, hipStream_t s) {
  Sizes z(d);
  FaxSavedLayout L;
  saved_layout(d, &L);
  const int T = (int)z.T, D = d.D, Hd = (int)z.Hd, F = d.F;
  const bool partial = (d.flags & FAX_FLAG_TP_PARTIAL) != 0;
  FAX_TRY(ln_fwd(d.dtype, T, D, x, p.ln1_g, p.ln1_b, d.ln_eps, saved + L.h1, (float*)(saved + L.mu1),
                 (float*)(saved + L.rstd1), s));
  GemmArgs g;
  g.dtype = d.dtype;
  g.gelu_form = d.gelu;
  // qkv = h1 Wqkv + bqkv
  g.M = T; g.N = 3 * Hd; g.K = D;
  g.A = saved + L.h1; g.lda = D; g.B = p.wqkv; g.ldb = 3 * Hd; g.C = saved + L.qkv; g.ldc = 3 * Hd; g.bias = p.bqkv;
  FAX_TRY(gemm(g, s));
  FAX_TRY(attention_fwd(d.dtype, d.B, d.S, d.H, d.dh, saved + L.qkv, saved + L.ctx, (float*)(saved + L.lse), PATH_AUTO, s));
  // x1 = x + ctx Wo + bo
  g = GemmArgs(); g.dtype = d.dtype; g.gelu_form = d.gelu;
  g.M = T; g.N = D; g.K = Hd;
  g.A = saved + L.ctx; g.lda = Hd; g.B = p.wo; g.ldb = D; g.C = saved + L.x1; g.ldc = D; g.bias = p.bo;
  g.R = x; g.ldr = D;
  if (partial) { g.C2 = p_attn; g.ldc2 = D; }
  FAX_TRY(gemm(g, s));
  FAX_TRY(ln_fwd(d.dtype, T, D, saved + L.x1, p.ln2_g, p.ln2_b, d.ln_eps, saved + L.h2, (float*)(saved + L.mu2),
                 (float*)(saved + L.rstd2), s));
  // u = h2 W1 + b1 ; a = gelu(u), kept together with gelu'(u)
  g = GemmArgs(); g.dtype = d.dtype; g.gelu_form = d.gelu;
  g.M = T; g.N = F; g.K = D;
  g.A = saved + L.h2; g.lda = D; g.B = p.w1; g.ldb = F; g.C = saved + L.dgelu; g.ldc = F; g.bias = p.b1;
  g.epi = EPI_GELU; g.C2 = saved + L.a; g.ldc2 = F;
  FAX_TRY(gemm(g, s));
  // y = x1 + a W2 + b2
  g = GemmArgs(); g.dtype = d.dtype; g.gelu_form = d.gelu;
  g.M = T; g.N = D; g.K = F;
  g.A = saved + L.a; g.lda = F; g.B = p.w2; g.ldb = D; g.C = y; g.ldc = D; g.bias = p.b2;
  g.R = saved + L.x1; g.ldr = D;
  if (partial) { g.C2 = p_mlp; g.ldc2 = D; }
  FAX_TRY(gemm(g, s));
  return FAX_OK;
}

// ---- a second stream for the weight gradients --------------------------------------------------
// In the backward pass the weight-gradient product of a projection and its input-gradient product
// read the same upstream gradient and do not depend on each other; only the input gradients are on
// the path to the next kernel.  With few tokens (the 2048-token shares) neither fills the chip: a
// GEMM has 80 to 160 tiles for 256 CUs and attention a few dozen workgroups.  The four weight
// gradients are then enqueued on a stream of the library's own, forked from and joined back into
// the caller's stream with events inside the same call, so that they run beside the chain of
// input gradients.  Seen from the caller nothing changes: everything the call enqueues is
// ordered after earlier work on the caller's stream and before later work on it.
struct SideStream {
  std::mutex mu;  // held while one call enqueues: the events are shared, so record/wait pairs of two host threads must not interleave
  hipStream_t s = nullptr;
  hipEvent_t fork = nullptr, du = nullptr, dx1 = nullptr, dqkv = nullptr, ln2 = nullptr, ln1 = nullptr, w2_done = nullptr, join = nullptr,
             attn_fork = nullptr, attn_join = nullptr;
};
static std::mutex g_side_mu;
static SideStream* g_side[64];

static int side_stream(SideStream** out) {
  int dev = -1;
  FAX_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) { *out = nullptr; return FAX_OK; }
  std::lock_guard<std::mutex> lk(g_side_mu);
  if (!g_side[dev]) {
    SideStream* n = new SideStream;
    FAX_HIP(hipStreamCreateWithFlags(&n->s, hipStreamNonBlocking));  // default priority
    for (hipEvent_t* e : {&n->fork, &n->du, &n->dx1, &n->dqkv, &n->ln2, &n->ln1, &n->w2_done, &n->join, &n->attn_fork, &n->attn_join})
      FAX_HIP(hipEventCreateWithFlags(e, hipEventDisableTiming));
    g_side[dev] = n;
  }
  *out = g_side[dev];
  return FAX_OK;
}

// When every product of the backward pass is a whole number of rounds of one workgroup per CU
// (the 4096-wide block: 256 to 2048 tiles each), the second stream has nothing to fill and the
// kernels would only take turns: everything then stays on the caller's stream.
static bool use_side_stream(const FaxBlockDims& d) {
  if (d.flags & FAX_FLAG_SINGLE_STREAM) return false;
  if (d.dtype != FAX_BF16) return true;
  Sizes z(d);
  const int T = (int)z.T, D = d.D, Hd = (int)z.Hd, F = d.F;
  const int shapes[8][4] = {{F, D, T, 1}, {D, F, T, 1}, {Hd, D, T, 1}, {D, 3 * Hd, T, 1},
                            {T, F, D, 0}, {T, D, F, 0}, {T, Hd, D, 0}, {T, D, 3 * Hd, 0}};
  constexpr long long kCUs = 256;
  for (const auto& g : shapes) {
    int tail = 0;
    const GemmSplitPlan p = gemm_plan_query(g[0], g[1], g[2], g[3] != 0, &tail);
    if (tail || p.tile_m == 0) return true;
    const long long items = (long long)(g[0] / p.tile_m) * (g[1] / p.tile_n) * p.splits;
    if (items % kCUs) return true;
  }
  return false;
}

// ---- block backward -------------------------------------------------------------------------
static int block_bwd_impl(const FaxBlockDims& d, const FaxBlockTensors& p, const void* x, const void* dy,
                          const char* saved, void* dx, const FaxBlockTensors& gr, bool acc, void* dh1_out,
                          void* dh2_out, char* ws, hipStream_t s) {
  Sizes z(d);
  FaxSavedLayout L;
  saved_layout(d, &L);
  BwdWs W;
  bwd_layout(d, &W);
  const int T = (int)z.T, D = d.D, Hd = (int)z.Hd, F = d.F;
  // dh1, dh2 (the input-gradient partial sums of a tensor-parallel rank) go where the caller wants
  // them, else into their workspace slots
  char* du = ws + W.pub.du; char* dh2 = dh2_out ? (char*)dh2_out : ws + W.pub.dh2; char* dx1 = ws + W.pub.dx1;
  char* dctx = ws + W.pub.dctx; char* dqkv = ws + W.pub.dqkv; char* dh1 = dh1_out ? (char*)dh1_out : ws + W.pub.dh1;
  float* delta = (float*)(ws + W.delta);
  void* red = ws + W.red;

  SideStream* side = nullptr;
  if (use_side_stream(d)) FAX_TRY(side_stream(&side));
  std::unique_lock<std::mutex> side_lock;
  if (side) side_lock = std::unique_lock<std::mutex>(side->mu);
  hipStream_t sw = side ? side->s : s;  // where the weight gradients go
  void* red_w = side ? (void*)(ws + W.red_side) : red;
  auto wgrad = [&](const void* act, int lda, int Kdim, const void* grad, int ldb, int Ndim, void* out, void* bias_grad) {
    GemmArgs g;  // out[Kdim, Ndim] (+)= act^T grad, contraction over the T rows; bias_grad[Ndim] (+)= column sums of grad
    g.dtype = d.dtype; g.ta = true; g.tb = false;
    g.M = Kdim; g.N = Ndim; g.K = T;
    g.A = act; g.lda = lda; g.B = grad; g.ldb = ldb; g.C = out; g.ldc = Ndim; g.c_f32 = true; g.accumulate = acc;
    g.colsum = (float*)bias_grad; g.colsum_ws = red_w;
    g.split_ws = W.splitk < W.total ? ws + W.splitk : nullptr;
    return gemm(g, sw);
  };
  auto dgrad = [&](const void* grad, int lda, int Ndim, const void* w, int ldw, int Kdim, void* out) {
    GemmArgs g;  // out[T, Kdim] = grad[T, Ndim] w[Kdim, Ndim]^T
    g.dtype = d.dtype; g.ta = false; g.tb = true;
    g.M = T; g.N = Kdim; g.K = Ndim;
    g.A = grad; g.lda = lda; g.B = w; g.ldb = ldw; g.C = out; g.ldc = Kdim;
    return g;
  };
  // main stream records `e` once the tensor the next weight gradient reads is complete; the side stream waits for it
  auto hand_over = [&](hipEvent_t SideStream::*e) -> int {
    if (!side) return FAX_OK;
    FAX_HIP(hipEventRecord(side->*e, s));
    FAX_HIP(hipStreamWaitEvent(side->s, side->*e, 0));
    return FAX_OK;
  };

  // feed-forward output projection
  FAX_TRY(hand_over(&SideStream::fork));  // everything enqueued before this call (dy, saved, ...) is visible to the side stream
  FAX_TRY(wgrad(saved + L.a, F, F, dy, D, D, gr.w2, gr.b2));
  if (side) FAX_HIP(hipEventRecord(side->w2_done, side->s));
  {
    GemmArgs g = dgrad(dy, D, D, p.w2, D, F, du);  // du = (dy W2^T) * gelu'(u)
    g.epi = EPI_DGELU; g.U = saved + L.dgelu; g.ldu = F;
    FAX_TRY(gemm(g, s));
  }
  // feed-forward input projection
  FAX_TRY(hand_over(&SideStream::du));
  FAX_TRY(wgrad(saved + L.h2, D, D, du, F, F, gr.w1, gr.b1));
  FAX_TRY(gemm(dgrad(du, F, F, p.w1, F, D, dh2), s));
  // LN2 and the residual branch: dx1 = dy + LN2'(dh2)
  FAX_TRY(ln_bwd(d.dtype, T, D, dh2, saved + L.x1, (const float*)(saved + L.mu2), (const float*)(saved + L.rstd2),
                 p.ln2_g, dy, dx1, (float*)gr.ln2_g, (float*)gr.ln2_b, acc, red, s, side ? side->s : nullptr,
                 side ? side->ln2 : nullptr));
  // attention output projection
  FAX_TRY(hand_over(&SideStream::dx1));
  FAX_TRY(wgrad(saved + L.ctx, Hd, Hd, dx1, D, D, gr.wo, gr.bo));
  FAX_TRY(gemm(dgrad(dx1, D, D, p.wo, D, Hd, dctx), s));
  // attention
  const AttnBwdSplit split{(float*)(ws + W.delta2), side ? side->s : nullptr, side ? side->attn_fork : nullptr,
                           side ? side->attn_join : nullptr};
  FAX_TRY(attention_bwd(d.dtype, d.B, d.S, d.H, d.dh, saved + L.qkv, saved + L.ctx, (const float*)(saved + L.lse), dctx,
                        dqkv, delta, PATH_AUTO, s, &split));
  // QKV projection
  FAX_TRY(hand_over(&SideStream::dqkv));
  FAX_TRY(wgrad(saved + L.h1, D, D, dqkv, 3 * Hd, 3 * Hd, gr.wqkv, gr.bqkv));
  FAX_TRY(gemm(dgrad(dqkv, 3 * Hd, 3 * Hd, p.wqkv, 3 * Hd, D, dh1), s));
  // LN1 and the residual branch: dx = dx1 + LN1'(dh1).  dx may be the buffer dy came in: the first
  // weight gradient, which reads dy, has to be through with it.
  if (side) FAX_HIP(hipStreamWaitEvent(s, side->w2_done, 0));
  FAX_TRY(ln_bwd(d.dtype, T, D, dh1, x, (const float*)(saved + L.mu1), (const float*)(saved + L.rstd1), p.ln1_g, dx1,
                 dx, (float*)gr.ln1_g, (float*)gr.ln1_b, acc, side ? (void*)(ws + W.red_ln1) : red, s, side ? side->s : nullptr,
                 side ? side->ln1 : nullptr));
  // join: later work on the caller's stream (the next block, the update) sees every gradient, and the
  // workspace is free again
  if (side) {
    FAX_HIP(hipEventRecord(side->join, side->s));
    FAX_HIP(hipStreamWaitEvent(s, side->join, 0));
  }
  return FAX_OK;
}

// ---- model ----------------------------------------------------------------------------------
struct TrainWs {
  size_t xs, saved, hf, muf, rstdf, logits, row_loss, dcur, dhf, blk, headsplit, embidx, total;
  size_t x_stride, saved_stride;
};

static void train_layout(const FaxModelDims& m, TrainWs* W) {
  const FaxBlockDims& d = m.blk;
  Sizes z(d);
  FaxSavedLayout L;
  saved_layout(d, &L);
  BwdWs B;
  bwd_layout(d, &B);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += align_up(bytes); return r; };
  W->x_stride = align_up(z.T * z.D * z.es);
  W->saved_stride = L.total;
  W->xs = take(W->x_stride * (size_t)(m.L + 1));
  W->saved = take(W->saved_stride * (size_t)m.L);
  W->hf = take(z.T * z.D * z.es);
  W->muf = take(z.T * 4);
  W->rstdf = take(z.T * 4);
  W->logits = take(z.T * (size_t)m.V * z.es);
  W->row_loss = take(z.T * 4);
  W->dcur = take(z.T * z.D * z.es);
  W->dhf = take(z.T * z.D * z.es);
  W->blk = take(B.total);
  W->headsplit = take(gemm_split_ws_bytes(m.V, (int)z.D, (int)z.T));  // the embedding gradient's product may split K
  W->embidx = take(embed_index_ws_bytes(m.V));  // first position and count per token id (FAX_FLAG_DETERMINISTIC)
  W->total = o;
}

static int check_model_tensors(const FaxModelTensors* t, int L, const char* what) {
  if (!t) {
    set_error("%s is NULL", what);
    return FAX_ERR_INVALID_ARG;
  }
  char name[64];
  snprintf(name, sizeof(name), "%s.tok_emb", what); FAX_TRY(check_ptr(t->tok_emb, name));
  snprintf(name, sizeof(name), "%s.pos_emb", what); FAX_TRY(check_ptr(t->pos_emb, name));
  snprintf(name, sizeof(name), "%s.lnf_g", what); FAX_TRY(check_ptr(t->lnf_g, name));
  snprintf(name, sizeof(name), "%s.lnf_b", what); FAX_TRY(check_ptr(t->lnf_b, name));
  if (!t->blocks) {
    set_error("%s.blocks is NULL", what);
    return FAX_ERR_INVALID_ARG;
  }
  for (int l = 0; l < L; l++) {
    snprintf(name, sizeof(name), "%s.blocks[%d]", what, l);
    FAX_TRY(check_tensors(&t->blocks[l], name));
  }
  return FAX_OK;
}

}  // namespace fax

using namespace fax;

extern "C" {

const char* fax_version(void) { return "libfax 0.1 (gfx950, HIP)"; }
const char* fax_last_error(void) { return g_err; }

int fax_block_dims_check(const FaxBlockDims* dims) { return check_dims(dims); }

int fax_gemm_plan(int M, int N, int K, int c_f32, FaxGemmPlan* out) {
  if (!out) { set_error("out is NULL"); return FAX_ERR_INVALID_ARG; }
  if (M <= 0 || N <= 0 || K <= 0) { set_error("non-positive GEMM size %d x %d x %d", M, N, K); return FAX_ERR_INVALID_ARG; }
  int tail = 0;
  const GemmSplitPlan p = gemm_plan_query(M, N, K, c_f32 != 0, &tail);
  out->tail = tail; out->tile_m = p.tile_m; out->tile_n = p.tile_n; out->splits = p.splits;
  return FAX_OK;
}

int fax_gemm_tile_walk(int M, int N, int K, int c_f32, int32_t* tile_row, int32_t* tile_col, int capacity, int* count,
                       int* group) {
  if (!count || !group) { set_error("count or group is NULL"); return FAX_ERR_INVALID_ARG; }
  if (capacity < 0 || (capacity > 0 && (!tile_row || !tile_col))) { set_error("tile_row / tile_col missing"); return FAX_ERR_INVALID_ARG; }
  if (M <= 0 || N <= 0 || K <= 0) { set_error("non-positive GEMM size %d x %d x %d", M, N, K); return FAX_ERR_INVALID_ARG; }
  gemm_tile_walk_query(M, N, K, c_f32 != 0, tile_row, tile_col, capacity, count, group);
  return FAX_OK;
}

int fax_block_saved_layout(const FaxBlockDims* dims, FaxSavedLayout* out) {
  FAX_TRY(check_dims(dims));
  if (!out) { set_error("out is NULL"); return FAX_ERR_INVALID_ARG; }
  saved_layout(*dims, out);
  return FAX_OK;
}

int fax_block_bwd_layout(const FaxBlockDims* dims, FaxBwdLayout* out) {
  FAX_TRY(check_dims(dims));
  if (!out) { set_error("out is NULL"); return FAX_ERR_INVALID_ARG; }
  BwdWs W;
  bwd_layout(*dims, &W);
  *out = W.pub;
  return FAX_OK;
}

int fax_block_workspace_bytes(const FaxBlockDims* dims, size_t* out) {
  FAX_TRY(check_dims(dims));
  if (!out) { set_error("out is NULL"); return FAX_ERR_INVALID_ARG; }
  BwdWs W;
  bwd_layout(*dims, &W);
  *out = W.total;
  return FAX_OK;
}

int fax_train_workspace_bytes(const FaxModelDims* dims, size_t* out) {
  if (!dims) { set_error("dims is NULL"); return FAX_ERR_INVALID_ARG; }
  FAX_TRY(check_dims(&dims->blk));
  if (!out) { set_error("out is NULL"); return FAX_ERR_INVALID_ARG; }
  if (dims->L <= 0 || dims->V <= 0 || dims->S_max < dims->blk.S) {
    set_error("model dims: L=%d V=%d S_max=%d (S=%d)", dims->L, dims->V, dims->S_max, dims->blk.S);
    return FAX_ERR_INVALID_ARG;
  }
  TrainWs W;
  train_layout(*dims, &W);
  *out = W.total;
  return FAX_OK;
}

int fax_block_fwd(const FaxBlockDims* dims, const FaxBlockTensors* params, const void* x, void* y, void* saved,
                  void* p_attn, void* p_mlp, void* ws, size_t ws_bytes, void* stream) {
  FAX_TRY(check_dims(dims));
  FAX_TRY(check_tensors(params, "params"));
  FAX_TRY(check_ptr(x, "x"));
  FAX_TRY(check_ptr(y, "y"));
  FAX_TRY(check_ptr(saved, "saved"));
  if (x == y) { set_error("y must not alias x"); return FAX_ERR_INVALID_ARG; }
  if (dims->flags & FAX_FLAG_TP_PARTIAL) {
    FAX_TRY(check_ptr(p_attn, "p_attn"));
    FAX_TRY(check_ptr(p_mlp, "p_mlp"));
  }
  (void)ws; (void)ws_bytes;  // the forward pass needs no scratch beyond `saved`
  return block_fwd_impl(*dims, *params, x, y, (char*)saved, p_attn, p_mlp, (hipStream_t)stream);
}

int fax_block_bwd(const FaxBlockDims* dims, const FaxBlockTensors* params, const void* x, const void* dy,
                  const void* saved, void* dx, const FaxBlockTensors* grads, int accumulate, void* dh1_partial,
                  void* dh2_partial, void* ws, size_t ws_bytes, void* stream) {
  FAX_TRY(check_dims(dims));
  FAX_TRY(check_tensors(params, "params"));
  FAX_TRY(check_tensors(grads, "grads"));
  FAX_TRY(check_ptr(x, "x"));
  FAX_TRY(check_ptr(dy, "dy"));
  FAX_TRY(check_ptr(saved, "saved"));
  FAX_TRY(check_ptr(dx, "dx"));
  FAX_TRY(check_ptr(ws, "ws"));
  if (dh1_partial) FAX_TRY(check_ptr(dh1_partial, "dh1_partial"));
  if (dh2_partial) FAX_TRY(check_ptr(dh2_partial, "dh2_partial"));
  BwdWs W;
  bwd_layout(*dims, &W);
  if (ws_bytes < W.total) {
    set_error("workspace of %zu bytes is smaller than the %zu required", ws_bytes, W.total);
    return FAX_ERR_WORKSPACE;
  }
  return block_bwd_impl(*dims, *params, x, dy, (const char*)saved, dx, *grads, accumulate != 0, dh1_partial, dh2_partial,
                        (char*)ws, (hipStream_t)stream);
}

int fax_adamw_step(void* master, void* m, void* v, const void* grad, int grad_dtype, void* lowp, size_t n,
                   const FaxAdamW* hp, int step, void* stream) {
  if (grad_dtype != FAX_F32 && grad_dtype != FAX_BF16) { set_error("grad_dtype must be FAX_F32 or FAX_BF16"); return FAX_ERR_INVALID_ARG; }
  if (n == 0) return FAX_OK;
  FAX_TRY(check_ptr(master, "master"));
  FAX_TRY(check_ptr(m, "m"));
  FAX_TRY(check_ptr(v, "v"));
  FAX_TRY(check_ptr(grad, "grad"));
  if (lowp && misaligned(lowp)) { set_error("lowp is not 16-byte aligned"); return FAX_ERR_INVALID_ARG; }
  FAX_TRY(check_adamw(hp, step));
  return adamw((float*)master, (float*)m, (float*)v, grad, grad_dtype, lowp, n, *hp, step, (hipStream_t)stream);
}

int fax_adamw_block_step(const FaxBlockDims* dims, const FaxBlockTensors* master, const FaxBlockTensors* m,
                         const FaxBlockTensors* v, const FaxBlockTensors* grads, const FaxBlockTensors* lowp,
                         const FaxAdamW* hp, int step, void* stream) {
  FAX_TRY(check_dims(dims));
  FAX_TRY(check_tensors(master, "master"));
  FAX_TRY(check_tensors(m, "m"));
  FAX_TRY(check_tensors(v, "v"));
  FAX_TRY(check_tensors(grads, "grads"));
  if (lowp) FAX_TRY(check_tensors(lowp, "lowp"));
  FAX_TRY(check_adamw(hp, step));
  size_t n[12];
  tensor_counts(*dims, n);
  void* const* Ms = (void* const*)tensor_list(master);
  void* const* Mo = (void* const*)tensor_list(m);
  void* const* Vo = (void* const*)tensor_list(v);
  void* const* G = (void* const*)tensor_list(grads);
  void* const* P = lowp ? (void* const*)tensor_list(lowp) : nullptr;
  AdamWQueue q(*hp, step, (hipStream_t)stream);
  for (int i = 0; i < 12; i++)
    FAX_TRY(q.add((float*)Ms[i], (float*)Mo[i], (float*)Vo[i], (const float*)G[i], P ? P[i] : nullptr, n[i]));
  return q.flush();
}

// Evaluation: two activation buffers that take turns, one block's worth of saved tensors that every
// layer overwrites, the final LayerNorm, the logits, per-row losses.
struct EvalWs {
  size_t x[2], saved, hf, muf, rstdf, logits, row_loss, total;
};

static void eval_layout(const FaxModelDims& m, EvalWs* W) {
  const FaxBlockDims& d = m.blk;
  Sizes z(d);
  FaxSavedLayout L;
  saved_layout(d, &L);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += align_up(bytes); return r; };
  W->x[0] = take(z.T * z.D * z.es);
  W->x[1] = take(z.T * z.D * z.es);
  W->saved = take(L.total);
  W->hf = take(z.T * z.D * z.es);
  W->muf = take(z.T * 4);
  W->rstdf = take(z.T * 4);
  W->logits = take(z.T * (size_t)m.V * z.es);
  W->row_loss = take(z.T * 4);
  W->total = o;
}

int fax_eval_workspace_bytes(const FaxModelDims* dims, size_t* out) {
  size_t train = 0;
  FAX_TRY(fax_train_workspace_bytes(dims, &train));  // same validation of dims
  if (!out) { set_error("out is NULL"); return FAX_ERR_INVALID_ARG; }
  EvalWs W;
  eval_layout(*dims, &W);
  *out = W.total;
  return FAX_OK;
}

int fax_eval_step(const FaxModelDims* dims, const FaxModelTensors* params, const int32_t* tokens, const int32_t* labels,
                  float* loss_out, void* ws, size_t ws_bytes, void* stream) {
  size_t need = 0;
  FAX_TRY(fax_eval_workspace_bytes(dims, &need));
  FAX_TRY(check_model_tensors(params, dims->L, "params"));
  FAX_TRY(check_ptr(tokens, "tokens"));
  FAX_TRY(check_ptr(labels, "labels"));
  FAX_TRY(check_ptr(loss_out, "loss_out"));
  FAX_TRY(check_ptr(ws, "ws"));
  if (ws_bytes < need) {
    set_error("workspace of %zu bytes is smaller than the %zu required", ws_bytes, need);
    return FAX_ERR_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)stream;
  const FaxBlockDims& d = dims->blk;
  EvalWs W;
  eval_layout(*dims, &W);
  Sizes z(d);
  char* w = (char*)ws;
  const int T = (int)z.T, D = d.D, V = dims->V;
  FaxBlockDims bd = d;
  bd.flags &= ~FAX_FLAG_TP_PARTIAL;
  FAX_TRY(embed_fwd(d.dtype, d.B, d.S, D, tokens, params->tok_emb, params->pos_emb, w + W.x[0], s));
  for (int l = 0; l < dims->L; l++)
    FAX_TRY(block_fwd_impl(bd, params->blocks[l], w + W.x[l & 1], w + W.x[(l + 1) & 1], w + W.saved, nullptr, nullptr, s));
  FAX_TRY(ln_fwd(d.dtype, T, D, w + W.x[dims->L & 1], params->lnf_g, params->lnf_b, d.ln_eps, w + W.hf,
                 (float*)(w + W.muf), (float*)(w + W.rstdf), s));
  GemmArgs g;  // logits = hf E^T
  g.dtype = d.dtype; g.ta = false; g.tb = true;
  g.M = T; g.N = V; g.K = D;
  g.A = w + W.hf; g.lda = D; g.B = params->tok_emb; g.ldb = D; g.C = w + W.logits; g.ldc = V;
  FAX_TRY(gemm(g, s));
  return cross_entropy(d.dtype, T, V, w + W.logits, labels, nullptr, (float*)(w + W.row_loss), loss_out, 1.0f, s);
}

int fax_train_step(const FaxModelDims* dims, const FaxModelTensors* params, const FaxModelTensors* master,
                   const FaxModelTensors* m, const FaxModelTensors* v, const FaxModelTensors* grads,
                   const int32_t* tokens, const int32_t* labels, const FaxAdamW* hp, int step, float* loss_out, void* ws,
                   size_t ws_bytes, void* stream) {
  size_t need = 0;
  FAX_TRY(fax_train_workspace_bytes(dims, &need));
  const FaxBlockDims& d = dims->blk;
  const bool update = !(dims->flags & FAX_FLAG_SKIP_UPDATE);
  const bool acc = (dims->flags & FAX_FLAG_ACCUMULATE) != 0;
  if (dims->micro_batches < 0) { set_error("micro_batches must be >= 0, got %d", dims->micro_batches); return FAX_ERR_INVALID_ARG; }
  const float grad_scale = dims->micro_batches > 1 ? 1.0f / (float)dims->micro_batches : 1.0f;
  FAX_TRY(check_model_tensors(params, dims->L, "params"));
  FAX_TRY(check_model_tensors(grads, dims->L, "grads"));
  if (update) {
    FAX_TRY(check_model_tensors(master, dims->L, "master"));
    FAX_TRY(check_model_tensors(m, dims->L, "m"));
    FAX_TRY(check_model_tensors(v, dims->L, "v"));
    FAX_TRY(check_adamw(hp, step));
    if (d.dtype == FAX_F32) {
      bool same = params->tok_emb == master->tok_emb && params->pos_emb == master->pos_emb &&
                  params->lnf_g == master->lnf_g && params->lnf_b == master->lnf_b;
      for (int l = 0; l < dims->L && same; l++)
        same = memcmp(&params->blocks[l], &master->blocks[l], sizeof(FaxBlockTensors)) == 0;
      if (!same) {
        set_error("FAX_F32: master must be the same buffers as params (one fp32 copy, updated in place)");
        return FAX_ERR_INVALID_ARG;
      }
    }
  }
  FAX_TRY(check_ptr(tokens, "tokens"));
  FAX_TRY(check_ptr(labels, "labels"));
  FAX_TRY(check_ptr(loss_out, "loss_out"));
  FAX_TRY(check_ptr(ws, "ws"));
  if (ws_bytes < need) {
    set_error("workspace of %zu bytes is smaller than the %zu required", ws_bytes, need);
    return FAX_ERR_WORKSPACE;
  }
  hipStream_t s = (hipStream_t)stream;
  TrainWs W;
  train_layout(*dims, &W);
  Sizes z(d);
  char* w = (char*)ws;
  const int T = (int)z.T, D = d.D, V = dims->V, L = dims->L;
  FaxBlockDims bd = d;
  bd.flags &= ~FAX_FLAG_TP_PARTIAL;

  // The three phases the paper times separately (Fig. 4), then the update; with fax_timing_enable
  // each gets a record of its own ("phase_*") around the per-kernel ones.
  const double fwd_flop = (double)L * (2.0 * T * (3.0 * D * z.Hd + (double)z.Hd * D + 2.0 * D * d.F) +
                                       2.0 * d.B * d.H * (double)d.S * d.S * d.dh) + 2.0 * T * (double)D * V;
  const char* xL = w + W.xs + W.x_stride * L;
  // forward
  {
  Timed phase_("phase_forward", WORK_FLOP, fwd_flop, s);
  FAX_TRY(embed_fwd(d.dtype, d.B, d.S, D, tokens, params->tok_emb, params->pos_emb, w + W.xs, s));
  for (int l = 0; l < L; l++)
    FAX_TRY(block_fwd_impl(bd, params->blocks[l], w + W.xs + W.x_stride * l, w + W.xs + W.x_stride * (l + 1),
                           w + W.saved + W.saved_stride * l, nullptr, nullptr, s));
  FAX_TRY(ln_fwd(d.dtype, T, D, xL, params->lnf_g, params->lnf_b, d.ln_eps, w + W.hf, (float*)(w + W.muf),
                 (float*)(w + W.rstdf), s));
  GemmArgs g;  // logits = hf E^T
  g.dtype = d.dtype; g.ta = false; g.tb = true;
  g.M = T; g.N = V; g.K = D;
  g.A = w + W.hf; g.lda = D; g.B = params->tok_emb; g.ldb = D; g.C = w + W.logits; g.ldc = V;
  FAX_TRY(gemm(g, s));
  }
  // loss and its gradient, in place over the logits
  {
  Timed phase_("phase_loss", WORK_BYTE, 2.0 * T * (double)V * z.es, s);
  FAX_TRY(cross_entropy(d.dtype, T, V, w + W.logits, labels, w + W.logits, (float*)(w + W.row_loss), loss_out, grad_scale,
                        s));
  }
  {
  Timed phase_("phase_backward", WORK_FLOP, 2.0 * fwd_flop, s);
  // output projection backward: dE = dlogits^T hf ; dhf = dlogits E
  GemmArgs g; g.dtype = d.dtype; g.ta = true; g.tb = false;
  g.M = V; g.N = D; g.K = T;
  g.A = w + W.logits; g.lda = V; g.B = w + W.hf; g.ldb = D; g.C = grads->tok_emb; g.ldc = D; g.c_f32 = true;
  g.accumulate = acc;
  g.split_ws = W.headsplit < W.total ? w + W.headsplit : nullptr;
  FAX_TRY(gemm(g, s));
  g = GemmArgs(); g.dtype = d.dtype;
  g.M = T; g.N = D; g.K = V;
  g.A = w + W.logits; g.lda = V; g.B = params->tok_emb; g.ldb = D; g.C = w + W.dhf; g.ldc = D;
  FAX_TRY(gemm(g, s));
  FAX_TRY(ln_bwd(d.dtype, T, D, w + W.dhf, xL, (const float*)(w + W.muf), (const float*)(w + W.rstdf), params->lnf_g,
                 nullptr, w + W.dcur, (float*)grads->lnf_g, (float*)grads->lnf_b, acc, w + W.blk, s));
  for (int l = L - 1; l >= 0; l--)
    FAX_TRY(block_bwd_impl(bd, params->blocks[l], w + W.xs + W.x_stride * l, w + W.dcur,
                           w + W.saved + W.saved_stride * l, w + W.dcur, grads->blocks[l], acc, nullptr, nullptr,
                           w + W.blk, s));
  // embedding backward: token rows add onto the output projection's share; positions beyond S get zero
  if (!acc) FAX_TRY(fill_zero(grads->pos_emb, (size_t)dims->S_max * D * 4, s));
  FAX_TRY(embed_bwd(d.dtype, d.B, d.S, D, V, tokens, w + W.dcur, (float*)grads->tok_emb, (float*)grads->pos_emb, acc,
                    (dims->flags & FAX_FLAG_DETERMINISTIC) ? w + W.embidx : nullptr, s));
  }
  if (!update) return FAX_OK;
  const bool lowp = d.dtype == FAX_BF16;
  size_t n[12];
  tensor_counts(d, n);
  double n_params = (double)V * D + (double)dims->S_max * D + 2.0 * D;
  for (int i = 0; i < 12; i++) n_params += (double)L * (double)n[i];
  Timed phase_("phase_update", WORK_BYTE, (lowp ? 30.0 : 28.0) * n_params, s);

  AdamWQueue q(*hp, step, s);
  auto upd = [&](void* P, void* Mst, void* Mo, void* Vo, const void* G, size_t n) {
    return q.add((float*)Mst, (float*)Mo, (float*)Vo, (const float*)G, lowp ? P : nullptr, n);
  };
  FAX_TRY(upd(params->tok_emb, master->tok_emb, m->tok_emb, v->tok_emb, grads->tok_emb, (size_t)V * D));
  FAX_TRY(upd(params->pos_emb, master->pos_emb, m->pos_emb, v->pos_emb, grads->pos_emb, (size_t)dims->S_max * D));
  FAX_TRY(upd(params->lnf_g, master->lnf_g, m->lnf_g, v->lnf_g, grads->lnf_g, (size_t)D));
  FAX_TRY(upd(params->lnf_b, master->lnf_b, m->lnf_b, v->lnf_b, grads->lnf_b, (size_t)D));
  for (int l = 0; l < L; l++) {
    void* const* P = (void* const*)tensor_list(&params->blocks[l]);
    void* const* Ms = (void* const*)tensor_list(&master->blocks[l]);
    void* const* Mo = (void* const*)tensor_list(&m->blocks[l]);
    void* const* Vo = (void* const*)tensor_list(&v->blocks[l]);
    void* const* G = (void* const*)tensor_list(&grads->blocks[l]);
    for (int i = 0; i < 12; i++) FAX_TRY(upd(P[i], Ms[i], Mo[i], Vo[i], G[i], n[i]));
  }
  return q.flush();
}

int fax_timing_enable(int on) {
  if (on) timing_clear();
  g_timing_on.store(on != 0);
  return FAX_OK;
}

int fax_timing_report(FaxKernelTime* out, int capacity, int* count) {
  if (!out || !count || capacity <= 0) { set_error("fax_timing_report: bad arguments"); return FAX_ERR_INVALID_ARG; }
  std::lock_guard<std::mutex> lk(g_timing_mu);
  std::map<std::string, FaxKernelTime> rows;
  for (TimingRecord* r : g_timing) {
    FAX_HIP(hipEventSynchronize(r->stop));
    float ms = 0.f;
    FAX_HIP(hipEventElapsedTime(&ms, r->start, r->stop));
    FaxKernelTime& k = rows[r->name];
    if (k.launches == 0) {
      memset(&k, 0, sizeof(k));
      snprintf(k.name, sizeof(k.name), "%s", r->name.c_str());
      k.unit = r->unit;
    }
    k.launches += 1;
    k.ms += ms;
    k.work += r->work;
  }
  int n = 0;
  for (auto& kv : rows) {
    if (n == capacity) break;
    out[n++] = kv.second;
  }
  *count = n;
  return FAX_OK;
}

// ---- building blocks --------------------------------------------------------------------------
int fax_gemm(int dtype, int ta, int tb, int M, int N, int K, const void* A, int lda, const void* B, int ldb, void* C,
             int ldc, int c_f32, int accumulate, const void* bias, const void* residual, int ldr, int path,
             void* stream) {
  if (dtype != FAX_F32 && dtype != FAX_BF16) { set_error("bad dtype %d", dtype); return FAX_ERR_INVALID_ARG; }
  if (M < 0 || N < 0 || K < 0) { set_error("negative GEMM size"); return FAX_ERR_INVALID_ARG; }
  if (M == 0 || N == 0) return FAX_OK;
  if (K > 0) { FAX_TRY(check_ptr(A, "A")); FAX_TRY(check_ptr(B, "B")); }
  FAX_TRY(check_ptr(C, "C"));
  if (lda < (ta ? M : K) || ldb < (tb ? K : N) || ldc < N || (residual && ldr < N)) {
    set_error("leading dimension smaller than the row length");
    return FAX_ERR_INVALID_ARG;
  }
  if (accumulate && !c_f32) { set_error("accumulate needs an fp32 C"); return FAX_ERR_INVALID_ARG; }
  if (path < 0 || path > 2) { set_error("bad path %d", path); return FAX_ERR_INVALID_ARG; }
  GemmArgs g;
  g.dtype = dtype; g.ta = ta != 0; g.tb = tb != 0;
  g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
  g.c_f32 = c_f32 != 0; g.accumulate = accumulate != 0; g.bias = bias; g.R = residual; g.ldr = ldr; g.path = path;
  return gemm(g, (hipStream_t)stream);
}

int fax_layernorm_fwd(int dtype, int rows, int D, const void* x, const void* gamma, const void* beta, float eps, void* h,
                      float* mu, float* rstd, void* stream) {
  if (rows < 0 || D <= 0) { set_error("bad LayerNorm size rows=%d D=%d", rows, D); return FAX_ERR_INVALID_ARG; }
  if (rows == 0) return FAX_OK;
  FAX_TRY(check_ptr(x, "x")); FAX_TRY(check_ptr(gamma, "gamma")); FAX_TRY(check_ptr(beta, "beta"));
  FAX_TRY(check_ptr(h, "h")); FAX_TRY(check_ptr(mu, "mu")); FAX_TRY(check_ptr(rstd, "rstd"));
  return ln_fwd(dtype, rows, D, x, gamma, beta, eps, h, mu, rstd, (hipStream_t)stream);
}

size_t fax_layernorm_bwd_workspace_bytes(int D) { return D > 0 ? ln_bwd_ws_bytes(D) : 0; }

int fax_layernorm_bwd(int dtype, int rows, int D, const void* dh, const void* x, const float* mu, const float* rstd,
                      const void* gamma, const void* dres, void* dx, float* dgamma, float* dbeta, int accumulate,
                      void* ws, size_t ws_bytes, void* stream) {
  if (rows < 0 || D <= 0) { set_error("bad LayerNorm size rows=%d D=%d", rows, D); return FAX_ERR_INVALID_ARG; }
  if (rows == 0) return FAX_OK;
  FAX_TRY(check_ptr(dh, "dh")); FAX_TRY(check_ptr(x, "x")); FAX_TRY(check_ptr(mu, "mu")); FAX_TRY(check_ptr(rstd, "rstd"));
  FAX_TRY(check_ptr(gamma, "gamma")); FAX_TRY(check_ptr(dx, "dx")); FAX_TRY(check_ptr(dgamma, "dgamma"));
  FAX_TRY(check_ptr(dbeta, "dbeta")); FAX_TRY(check_ptr(ws, "ws"));
  if (ws_bytes < ln_bwd_ws_bytes(D)) { set_error("LayerNorm backward workspace too small"); return FAX_ERR_WORKSPACE; }
  return ln_bwd(dtype, rows, D, dh, x, mu, rstd, gamma, dres, dx, dgamma, dbeta, accumulate != 0, ws, (hipStream_t)stream);
}

int fax_attention_fwd(int dtype, int B, int S, int H, int dh, const void* qkv, void* ctx, float* lse, int path,
                      void* stream) {
  if (B <= 0 || S <= 0 || H <= 0 || dh <= 0) { set_error("bad attention size"); return FAX_ERR_INVALID_ARG; }
  FAX_TRY(check_ptr(qkv, "qkv")); FAX_TRY(check_ptr(ctx, "ctx")); FAX_TRY(check_ptr(lse, "lse"));
  return attention_fwd(dtype, B, S, H, dh, qkv, ctx, lse, path, (hipStream_t)stream);
}

int fax_attention_bwd(int dtype, int B, int S, int H, int dh, const void* qkv, const void* ctx, const float* lse,
                      const void* dctx, void* dqkv, float* delta, int path, void* stream) {
  if (B <= 0 || S <= 0 || H <= 0 || dh <= 0) { set_error("bad attention size"); return FAX_ERR_INVALID_ARG; }
  FAX_TRY(check_ptr(qkv, "qkv")); FAX_TRY(check_ptr(ctx, "ctx")); FAX_TRY(check_ptr(lse, "lse"));
  FAX_TRY(check_ptr(dctx, "dctx")); FAX_TRY(check_ptr(dqkv, "dqkv")); FAX_TRY(check_ptr(delta, "delta"));
  return attention_bwd(dtype, B, S, H, dh, qkv, ctx, lse, dctx, dqkv, delta, path, (hipStream_t)stream);
}

int fax_cross_entropy(int dtype, int N, int V, const void* logits, const int32_t* labels, void* dlogits, float* row_loss,
                      float* loss_out, void* stream) {
  if (N <= 0 || V <= 0) { set_error("bad cross-entropy size N=%d V=%d", N, V); return FAX_ERR_INVALID_ARG; }
  FAX_TRY(check_ptr(logits, "logits")); FAX_TRY(check_ptr(labels, "labels")); FAX_TRY(check_ptr(dlogits, "dlogits"));
  FAX_TRY(check_ptr(row_loss, "row_loss")); FAX_TRY(check_ptr(loss_out, "loss_out"));
  return cross_entropy(dtype, N, V, logits, labels, dlogits, row_loss, loss_out, 1.0f, (hipStream_t)stream);
}

int fax_probe_mfma(int workgroups, int iters, unsigned seed, float* sink, void* stream) {
  if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || iters > (1 << 24)) {
    set_error("fax_probe_mfma: workgroups=%d iters=%d out of range", workgroups, iters);
    return FAX_ERR_INVALID_ARG;
  }
  FAX_TRY(check_ptr(sink, "sink"));
  return probe_mfma(workgroups, iters, seed, sink, (hipStream_t)stream);
}

int fax_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (bytes == 0 || bytes % 16) { set_error("fax_probe_copy: bytes must be a positive multiple of 16"); return FAX_ERR_INVALID_ARG; }
  FAX_TRY(check_ptr(src, "src")); FAX_TRY(check_ptr(dst, "dst"));
  return probe_copy(src, dst, bytes, (hipStream_t)stream);
}

int fax_cross_entropy_static(int dtype, int N, int V, const void* logits, const int32_t* labels, void* dlogits,
                             float* loss_out, void* stream) {
  if (dtype != FAX_F32 && dtype != FAX_BF16) { set_error("bad dtype %d", dtype); return FAX_ERR_INVALID_ARG; }
  if (N <= 0 || V <= 0) { set_error("bad cross-entropy size N=%d V=%d", N, V); return FAX_ERR_INVALID_ARG; }
  FAX_TRY(check_ptr(logits, "logits")); FAX_TRY(check_ptr(labels, "labels")); FAX_TRY(check_ptr(dlogits, "dlogits"));
  FAX_TRY(check_ptr(loss_out, "loss_out"));
  return cross_entropy_static(dtype, N, V, logits, labels, dlogits, loss_out, (hipStream_t)stream);
}

int fax_cross_entropy_static_max_rows(void) { return CE_STATIC_MAX_ROWS; }

}  // extern "C"
