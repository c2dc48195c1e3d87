/*
 * fax.h -- C ABI of the per-device Transformer training step for MI355X (gfx950).
 *
 * The paper's framework compiles one function per device: the training step of
 * a decoder-only Transformer (Fig. 1), whose phases are the forward pass, the
 * loss and the backward pass (Fig. 4), followed by the Adam update (Table 1
 * caption), on that device's shard of the data-parallel x tensor-parallel mesh
 * (Sec. 2.2, Sec. 3.2).  This library is that per-device function as
 * hand-written HIP kernels.
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers unless a comment says "host".
 *     Structs (dims, pointer tables) are HOST memory, read during the call only.
 *   - The caller owns every buffer: inputs, outputs, saved activations,
 *     gradients, optimizer state, workspace.  The library allocates nothing
 *     and keeps no pointer after a call returns.
 *   - Work is enqueued on the caller's hipStream_t (passed as void*, NULL = the
 *     default stream); the calls do not synchronise.  Outputs are valid once
 *     the caller has synchronised the stream.
 *   - Return value: FAX_OK or a negative FaxStatus; fax_last_error() gives the
 *     text for the calling thread.  Arguments are validated on the host before
 *     the first launch, so a failed call has enqueued nothing.
 *   - Tensors are row-major.  Activations are [B, S, D] = [T, D] with T = B*S.
 *     Weight matrices are [in, out], applied as y = x W + b.  The fused QKV
 *     projection has 3*H*dh columns ordered [Q | K | V], head-major within each.
 *   - dtype FAX_BF16: activations, parameters and activation gradients are
 *     bfloat16, every accumulation, statistic and softmax is fp32.
 *     dtype FAX_F32: everything is fp32 with true fp32 multiply-add.
 *     Parameter GRADIENTS are fp32 for both dtypes.
 *   - Pointers must be 16-byte aligned.
 */
#ifndef FAX_H
#define FAX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum FaxStatus {
  FAX_OK = 0,
  FAX_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, inconsistent dims, misalignment */
  FAX_ERR_UNSUPPORTED = -2, /* a shape or option no kernel here covers */
  FAX_ERR_WORKSPACE = -3,   /* workspace smaller than fax_*_workspace_bytes() */
  FAX_ERR_HIP = -4          /* a HIP runtime or launch error */
} FaxStatus;

enum { FAX_F32 = 0, FAX_BF16 = 1 };
enum { FAX_GELU_TANH = 0, FAX_GELU_ERF = 1 };

/* FaxBlockDims.flags */
#define FAX_FLAG_TP_PARTIAL 1u /* also emit the pre-reduction partial sums (Sec. 3.2) */
/* fax_block_bwd (and the backward pass inside fax_train_step) by default enqueues the four
 * weight-gradient products and the folds of the LayerNorm parameter gradients on a stream of the
 * library's own, forked from the caller's stream when the call begins and joined back into it
 * before the call returns: they depend on nothing later in the chain of input gradients and run
 * beside it.  To the caller the call behaves as if everything were on its stream (ordered after
 * what was enqueued before, before what is enqueued after).  The stream and its events are
 * created once per device, on first use (not under stream capture: make one call before
 * capturing), and live until the process ends; no device memory is involved.  Host threads that
 * call into the library on the same device share that stream: their calls are enqueued one after
 * the other on it.  (When every product of
 * the backward pass fills the chip a whole number of times there is nothing to run beside, and
 * the library keeps to the caller's stream by itself.)  With this flag everything is enqueued on
 * the caller's stream only. */
#define FAX_FLAG_SINGLE_STREAM 2u

/* FaxModelDims.flags */
#define FAX_FLAG_SKIP_UPDATE 1u /* fax_train_step: stop after the gradients */
#define FAX_FLAG_ACCUMULATE 2u  /* fax_train_step: add this call's gradients to `grads` instead of overwriting */
/* fax_train_step: no floating-point atomics anywhere.  The one kernel that uses them, the
 * scatter-add of the token-embedding gradient (rows of equal token ids add up in the order the
 * hardware happens to serve them), is replaced by an ordered reduction: one writer per vocabulary
 * row, positions added in ascending order.  Every other kernel of the library already has one
 * writer per output element and fixed-order reductions, with or without the flag: two calls on the
 * same inputs then return identical bits. */
#define FAX_FLAG_DETERMINISTIC 4u

/* Shape of one decoder block as one device holds it.  H and F are the LOCAL
 * head count and feed-forward width; H*dh need not equal D (a tensor-parallel
 * share, Sec. 3.2). */
typedef struct FaxBlockDims {
  int32_t B, S, D, H, dh, F;
  int32_t dtype;  /* FAX_F32 | FAX_BF16 */
  int32_t gelu;   /* FAX_GELU_TANH | FAX_GELU_ERF */
  float ln_eps;   /* LayerNorm epsilon, added to the biased variance */
  uint32_t flags; /* FAX_FLAG_TP_PARTIAL | FAX_FLAG_SINGLE_STREAM */
} FaxBlockDims;

/* The twelve parameter tensors of a block, or twelve buffers shaped like them
 * (fp32 master copies, Adam moments, gradients).
 *   ln1_g, ln1_b [D]; wqkv [D, 3*H*dh]; bqkv [3*H*dh]; wo [H*dh, D]; bo [D];
 *   ln2_g, ln2_b [D]; w1 [D, F]; b1 [F]; w2 [F, D]; b2 [D]. */
typedef struct FaxBlockTensors {
  void *ln1_g, *ln1_b, *wqkv, *bqkv, *wo, *bo, *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
} FaxBlockTensors;

/* Byte offsets of each tensor inside the saved-activation buffer that
 * fax_block_fwd fills and fax_block_bwd reads.  Element type is dims.dtype
 * except the four LayerNorm statistics and lse, which are fp32. */
typedef struct FaxSavedLayout {
  size_t h1;    /* [T, D]      LN1(x) */
  size_t qkv;   /* [T, 3*H*dh] */
  size_t ctx;   /* [T, H*dh]   attention output, heads concatenated */
  size_t lse;   /* [B, H, S]   fp32 log-sum-exp of the scaled masked scores */
  size_t x1;    /* [T, D]      x + ctx Wo + bo */
  size_t h2;    /* [T, D]      LN2(x1) */
  size_t dgelu; /* [T, F]      gelu'(u), u = h2 W1 + b1: all the backward pass needs of u */
  size_t a;     /* [T, F]      gelu(u) */
  size_t mu1, rstd1, mu2, rstd2; /* [T] fp32 each */
  size_t total; /* bytes to allocate */
} FaxSavedLayout;

/* Byte offsets of the activation gradients fax_block_bwd leaves in its
 * workspace (valid after the call; element type dims.dtype).  Exposed so a
 * caller or test can inspect them; not needed for normal use. */
typedef struct FaxBwdLayout {
  size_t du;    /* [T, F]      gradient at u */
  size_t dh2;   /* [T, D]      du W1^T: the MLP input-gradient partial sum */
  size_t dx1;   /* [T, D]      gradient at x1 */
  size_t dctx;  /* [T, H*dh] */
  size_t dqkv;  /* [T, 3*H*dh] */
  size_t dh1;   /* [T, D]      dqkv Wqkv^T: the attention input-gradient partial sum */
  size_t total; /* == fax_block_workspace_bytes */
} FaxBwdLayout;

/* Hyper-parameters are doubles so that 1 - beta2 and the bias corrections are formed
 * from the intended decimal values and rounded to fp32 once. */
typedef struct FaxAdamW {
  double lr, beta1, beta2, eps, wd;
} FaxAdamW;

/* Full model (final LayerNorm, tied output projection, learned positions). */
typedef struct FaxModelDims {
  FaxBlockDims blk; /* blk.B, blk.S give the batch */
  int32_t L;        /* layers */
  int32_t V;        /* vocabulary */
  int32_t S_max;    /* rows of the position table, >= blk.S */
  uint32_t flags;
  int32_t micro_batches; /* 0 or 1: this call's batch is the whole step's.  n > 1: it is one of n equal
                          * micro-batches of the step; its loss gradient is scaled by 1/n so that the
                          * accumulated gradients are those of the mean loss over the whole batch. */
} FaxModelDims;

/* Pointer table of the model's parameters, or buffers shaped like them.
 *   tok_emb [V, D]; pos_emb [S_max, D]; lnf_g, lnf_b [D];
 *   blocks: HOST array of L FaxBlockTensors. */
typedef struct FaxModelTensors {
  void *tok_emb, *pos_emb, *lnf_g, *lnf_b;
  const FaxBlockTensors* blocks;
} FaxModelTensors;

/* Build id; names the GPU target the kernels were compiled for ("gfx950"). */
const char* fax_version(void);
/* Text of the calling thread's most recent error ("" if none). */
const char* fax_last_error(void);

/* Host-only size queries. */
int fax_block_saved_layout(const FaxBlockDims* dims, FaxSavedLayout* out);
int fax_block_bwd_layout(const FaxBlockDims* dims, FaxBwdLayout* out);
int fax_block_workspace_bytes(const FaxBlockDims* dims, size_t* out); /* covers fwd and bwd */
int fax_train_workspace_bytes(const FaxModelDims* dims, size_t* out);

/* Host-only argument check used by every entry point; exposed for tests. */
int fax_block_dims_check(const FaxBlockDims* dims);

/* Host-only: the launch plan the library would use for a bf16 product C[M,N] = A B with a
 * contraction of K (c_f32 != 0: the fp32-output weight-gradient form, which may split K when
 * the caller provides scratch, as fax_block_bwd and fax_train_step do).
 *   tail          0: one launch.  1 / 2: the last 128 rows / columns run as a launch of their own
 *                 (a dimension that is an odd multiple of 128); tile_* and splits then describe
 *                 the bulk.
 *   tile_m/tile_n the tile class; 0 when no class divides the shape (the scalar kernel runs).
 *   splits        K ranges, each writing a partial product that a fold kernel sums (1: none).
 * Exposed so that a test can assert that a cut-down workload runs the plans of the full one. */
typedef struct FaxGemmPlan {
  int32_t tail, tile_m, tile_n, splits;
} FaxGemmPlan;
int fax_gemm_plan(int M, int N, int K, int c_f32, FaxGemmPlan* out);

/* Host-only: the order in which the bulk launch of that plan hands out its output tiles.  Work item
 * number i (workgroup b of the persistent kernel takes i = b, b + grid, ...) is the tile at tile
 * row tile_row[i], tile column tile_col[i]; *count receives the number of tiles (at most
 * `capacity` entries are written), *group the kind of walk: 8 or 4 tile rows per column-major
 * group, or 0 for the walk that lays the eight XCDs' blocks of a round side by side in a 16 x 16
 * block of tiles.  count = 0 and group = -1 when no tile class divides the shape.
 * Exposed so that a test can check that every walk visits every tile exactly once. */
int fax_gemm_tile_walk(int M, int N, int K, int c_f32, int32_t* tile_row, int32_t* tile_col, int capacity,
                       int* count, int* group);

/*
 * Forward pass of one pre-LayerNorm decoder block (Fig. 1; forward phase of Fig. 4):
 *   h1 = LN(x; ln1);  qkv = h1 Wqkv + bqkv;  ctx = causal softmax(Q K^T / sqrt(dh)) V per head;
 *   x1 = x + ctx Wo + bo;  h2 = LN(x1; ln2);  u = h2 W1 + b1;  a = gelu(u);  y = x1 + a W2 + b2.
 * params: tensors in dims.dtype.  x, y: [B,S,D] in dims.dtype; y must not alias x.
 * saved: buffer of fax_block_saved_layout().total bytes, filled for fax_block_bwd.
 * p_attn, p_mlp: with FAX_FLAG_TP_PARTIAL, [B,S,D] outputs receiving ctx Wo and a W2
 *   (no bias, no residual): the partial sums a tensor-parallel rank holds before the
 *   reduction over the model axis (Sec. 3.2).  Ignored (may be NULL) without the flag.
 * ws: workspace of at least fax_block_workspace_bytes().
 */
int fax_block_fwd(const FaxBlockDims* dims, const FaxBlockTensors* params, const void* x, void* y,
                  void* saved, void* p_attn, void* p_mlp, void* ws, size_t ws_bytes, void* stream);

/*
 * Backward pass of the same block (backward phase of Fig. 4).
 * dy: [B,S,D] upstream gradient; x: the forward input; saved: as filled by fax_block_fwd.
 * dx: [B,S,D] gradient at x (may alias dy).
 * grads: twelve fp32 buffers; accumulate != 0 adds into them, 0 overwrites.
 * dh1_partial, dh2_partial: optional [B,S,D] outputs in dims.dtype (device, 16-byte aligned, not
 *   aliasing any other argument) for the gradients at the outputs of the two LayerNorms,
 *   dh1 = dqkv Wqkv^T and dh2 = du W1^T: on a tensor-parallel rank these are the partial sums
 *   that are reduced over the model axis before the LayerNorm backward of the full model
 *   (Sec. 3.2).  NULL: they are left in the workspace instead, at the offsets of
 *   fax_block_bwd_layout(), like the other activation gradients of the call.
 */
int fax_block_bwd(const FaxBlockDims* dims, const FaxBlockTensors* params, const void* x, const void* dy,
                  const void* saved, void* dx, const FaxBlockTensors* grads, int accumulate,
                  void* dh1_partial, void* dh2_partial, void* ws, size_t ws_bytes, void* stream);

/*
 * Adam with decoupled weight decay on one tensor of n elements (Table 1 caption: Adam;
 * wd = 0 is plain Adam), step >= 1:
 *   m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
 *   p = p (1 - lr wd) - lr (m / (1-b1^step)) / (sqrt(v / (1-b2^step)) + eps).
 * master, m, v: fp32, updated in place (parameters are kept in fp32, Sec. 3).
 * grad: n gradients of type grad_dtype, FAX_F32 (what fax_block_bwd and fax_train_step produce)
 *   or FAX_BF16 (a caller that keeps or communicates gradients in the compute precision); the
 *   arithmetic is fp32 either way.  FAX_ERR_INVALID_ARG for any other value.
 * lowp: optional bf16 buffer receiving the rounded new parameters (NULL to skip).
 * All pointers device, 16-byte aligned.
 */
int fax_adamw_step(void* master, void* m, void* v, const void* grad, int grad_dtype, void* lowp, size_t n,
                   const FaxAdamW* hp, int step, void* stream);

/* The same update on the twelve tensors of a block in one launch (most of them are a few KB: a
 * launch each costs more than their update).  Tensor sizes follow from dims.  lowp: the bf16
 * compute copies to refresh, or NULL (fp32 models: the master tensors are the parameters). */
int fax_adamw_block_step(const FaxBlockDims* dims, const FaxBlockTensors* master, const FaxBlockTensors* m,
                         const FaxBlockTensors* v, const FaxBlockTensors* grads, const FaxBlockTensors* lowp,
                         const FaxAdamW* hp, int step, void* stream);

/*
 * One training step of the full model (forward, loss, backward, update: Fig. 4 + Table 1):
 *   x0 = tok_emb[tokens] + pos_emb[s];  L blocks;  hf = LN(x_L; lnf);  logits = hf tok_emb^T;
 *   loss = mean over B*S positions of logsumexp(logits) - logits[label];
 *   gradients of every tensor; then fax_adamw_step on every tensor unless FAX_FLAG_SKIP_UPDATE.
 * Gradient accumulation over micro-batches: call once per micro-batch with dims.micro_batches = n,
 * FAX_FLAG_ACCUMULATE on every call but the first and FAX_FLAG_SKIP_UPDATE on every call but the last.
 * loss_out is always the mean loss of the call's own batch.
 * params: compute copy in dims.blk.dtype (rewritten by the update when bf16).
 * master, m, v: fp32 state (for FAX_F32, master may equal params: one copy, updated in place).
 * grads: fp32, overwritten.  tokens, labels: int32 [B,S], values in [0,V) (caller validates).
 * loss_out: one fp32 on the device.
 */
int fax_train_step(const FaxModelDims* dims, const FaxModelTensors* params, const FaxModelTensors* master,
                   const FaxModelTensors* m, const FaxModelTensors* v, const FaxModelTensors* grads,
                   const int32_t* tokens, const int32_t* labels, const FaxAdamW* hp, int step,
                   float* loss_out, void* ws, size_t ws_bytes, void* stream);

/*
 * The validation step, one of the functions the framework compiles besides the training step
 * (Sec. 2.1): forward pass and mean loss as in fax_train_step, nothing kept for a backward pass,
 * no gradient written.  Workspace: fax_eval_workspace_bytes() (activations of one layer, not L).
 */
int fax_eval_workspace_bytes(const FaxModelDims* dims, size_t* out);
int fax_eval_step(const FaxModelDims* dims, const FaxModelTensors* params, const int32_t* tokens,
                  const int32_t* labels, float* loss_out, void* ws, size_t ws_bytes, void* stream);

/*
 * Static analysis of a model on a device mesh (host only: no GPU is touched, none is needed).
 * Sec. 2.1 points out that memory requirements and latency estimates can be computed from
 * the model's description before anything runs; Sec. 2.2 maps tensor axes onto the axes of a
 * logical device mesh.  The mesh here has the paper's two axes: the batch dimension is split
 * over `data`; heads, feed-forward columns (with them every large weight of a block, Sec. 3.2)
 * and the rows of the token table over `tensor`.
 *
 * fax_analyze() takes the GLOBAL model (blk.B = global batch, blk.H = all heads, blk.F = full
 * feed-forward width) and fills in what ONE device of the mesh holds and does per step:
 *   local            the dims of its share (B/data, H/tensor, F/tensor, V/tensor when every
 *                    rank's slice is a multiple of 128 rows, else V): the shapes every kernel
 *                    of fax_train_step would see.
 *                    Only the shapes: the reductions over the tensor axis (four [T, D] sums per
 *                    block, the loss's row statistics) are not built.
 *   params_*         parameter counts (LayerNorm tensors, the position table and the biases
 *                    added after a reduction are replicated over the tensor axis)
 *   bytes_*          device memory: fp32 master parameters, the two Adam moments, fp32
 *                    gradients, the low-precision compute copy, saved activations and the
 *                    rest of the workspace, exactly as the fax_*_layout / *_workspace_bytes
 *                    calls size them
 *   flop_*, hbm_bytes_step, launches
 *                    algorithmic work of one training step on this device
 *   ms_*             predicted time on one MI355X from the library's own launch plans: every
 *                    GEMM priced by the tile/split plan it would run with, attention per
 *                    score, bandwidth-bound kernels at a sustained HBM rate
 *   bytes_*_axis     what one device would send per step over each mesh axis
 * Errors: FAX_ERR_INVALID_ARG for NULL pointers, non-positive sizes, or a batch, head count or
 * feed-forward width that the mesh does not divide (Sec. 3.2 requires it of the heads).
 */
typedef struct FaxMesh {
  int32_t data, tensor;
} FaxMesh;

typedef struct FaxAnalysis {
  FaxModelDims local;
  double params_global, params_local;
  double bytes_master, bytes_moments, bytes_grads, bytes_lowp, bytes_saved, bytes_workspace, bytes_total;
  double flop_step, flop_step_unhalved, hbm_bytes_step;
  int32_t launches;
  double ms_gemm, ms_attention, ms_bandwidth, ms_step;
  double bytes_tensor_axis, bytes_data_axis;
} FaxAnalysis;

int fax_analyze(const FaxModelDims* global_dims, const FaxMesh* mesh, FaxAnalysis* out);

/*
 * Building blocks, exported so each kernel can be checked and timed alone: test and benchmark
 * hooks into the steps of the four entry points above.  They follow no passage of the paper of
 * their own (the steps they perform are those listed at fax_block_fwd / fax_block_bwd /
 * fax_train_step) and the conventions above; dtype is FAX_F32 or FAX_BF16.
 */

/* C[M,N] = op(A) op(B), fp32 accumulate.  ta = 0: A is [M,K] row-major (lda); ta = 1: A is
 * stored [K,M].  tb = 0: B is [K,N] row-major; tb = 1: B is stored [N,K].  c_f32 != 0
 * stores C as fp32 (and adds into it when accumulate != 0), else in dtype.
 * bias: optional [N] in dtype; residual: optional [M,N] in dtype, added after the bias.
 * path: 0 = choose, 1 = force the scalar-FMA kernel, 2 = force the MFMA kernel (bf16 only,
 * FAX_ERR_UNSUPPORTED if the shape does not tile). */
int fax_gemm(int dtype, int ta, int tb, int M, int N, int K, const void* A, int lda, const void* B,
             int ldb, void* C, int ldc, int c_f32, int accumulate, const void* bias,
             const void* residual, int ldr, int path, void* stream);

/* h = LN(x); mu, rstd: fp32 [rows]. */
int fax_layernorm_fwd(int dtype, int rows, int D, const void* x, const void* gamma, const void* beta,
                      float eps, void* h, float* mu, float* rstd, void* stream);
/* dx = (dres ? dres : 0) + LN-backward(dh); dgamma, dbeta fp32 [D] (accumulate as above).
 * ws: at least fax_layernorm_bwd_workspace_bytes(D). */
int fax_layernorm_bwd(int dtype, int rows, int D, const void* dh, const void* x, const float* mu,
                      const float* rstd, const void* gamma, const void* dres, void* dx,
                      float* dgamma, float* dbeta, int accumulate, void* ws, size_t ws_bytes,
                      void* stream);
size_t fax_layernorm_bwd_workspace_bytes(int D);

/* Causal attention over qkv [B,S,3*H*dh] -> ctx [B,S,H*dh], lse fp32 [B,H,S].
 * path: 0 = choose, 1 = scalar kernel, 2 = MFMA kernel. */
int fax_attention_fwd(int dtype, int B, int S, int H, int dh, const void* qkv, void* ctx, float* lse,
                      int path, void* stream);
/* dqkv from dctx; delta: fp32 [B,H,S] scratch. */
int fax_attention_bwd(int dtype, int B, int S, int H, int dh, const void* qkv, const void* ctx,
                      const float* lse, const void* dctx, void* dqkv, float* delta, int path,
                      void* stream);

/* Mean softmax cross-entropy over rows of logits [N,V]; dlogits may alias logits.
 * row_loss: fp32 [N] scratch; loss_out: one fp32. */
int fax_cross_entropy(int dtype, int N, int V, const void* logits, const int32_t* labels,
                      void* dlogits, float* row_loss, float* loss_out, void* stream);

/*
 * fax_cross_entropy for callers that cannot allocate device memory or may not call an allocator
 * where they stand: code under HIP graph capture, tight serving or evaluation loops, harnesses
 * that forbid hipMalloc.  Same kernels and same results as fax_cross_entropy; the per-row losses
 * (the one scratch buffer of that call) live in a device array built into the library instead of
 * a buffer of the caller's, so the call needs nothing but its inputs and outputs.  It allocates
 * and frees nothing and calls no allocating routine.
 *   Limit: N <= fax_cross_entropy_static_max_rows() = 262144 rows (1 MiB of scratch per GPU, held
 *   from the first use on that GPU until the process ends); more rows: FAX_ERR_WORKSPACE, nothing
 *   enqueued.
 *   The device that owns `stream` must be the current device.  All calls on one GPU share the one
 *   array: calls that overlap in time on the same GPU (different streams, or different threads)
 *   race on it; calls on one stream, or ordered by events, do not.  Nothing has to be cleared
 *   between calls: every entry a call reads it has written before.
 */
int fax_cross_entropy_static(int dtype, int N, int V, const void* logits, const int32_t* labels,
                             void* dlogits, float* loss_out, void* stream);
int fax_cross_entropy_static_max_rows(void);

/*
 * Measured ceilings, for benchmarks: what this GPU delivers to a kernel that does nothing but
 * matrix-core instructions, and to one that does nothing but copy.  Timed like every other kernel
 * through fax_timing_enable / fax_timing_report (rows "probe_mfma_zero", "probe_mfma_random",
 * "probe_copy").
 * fax_probe_mfma: `workgroups` x 4 waves each issue iters x 16 back-to-back 32x32x16 bf16 MFMAs on
 *   register operands (seed 0: all zero; otherwise pseudo-random finite values): 2 * 32 * 32 * 16
 *   flop each.  sink: one fp32 on the device (never written in practice).
 * fax_probe_copy: dst[0, bytes) = src[0, bytes), bytes a multiple of 16; both on the device.
 */
int fax_probe_mfma(int workgroups, int iters, unsigned seed, float* sink, void* stream);
int fax_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * Per-kernel timing with HIP events on the caller's stream: the split of a step into its
 * phases that Fig. 4 reports, at kernel granularity.  Off by default (no events recorded).
 * fax_timing_enable(1) clears earlier records and starts recording a start/stop event pair
 * around every kernel family launched by any entry point of this process; (0) stops.
 * fax_timing_report synchronises the recorded events and writes up to `capacity` rows (HOST
 * memory), one per kernel variant: launches, summed milliseconds, and summed algorithmic work
 * (unit 0: floating-point operations, 2 M N K per GEMM and 4 B H S^2 dh / 2 per causal
 * attention product set; unit 1: bytes that must cross HBM).  *count receives the rows written.
 * Process-wide state behind a mutex; meant for benchmarks, not for concurrent callers.
 */
typedef struct FaxKernelTime {
  char name[64];
  int32_t launches;
  int32_t unit;
  double ms;
  double work;
} FaxKernelTime;
int fax_timing_enable(int on);
int fax_timing_report(FaxKernelTime* out, int capacity, int* count);

#ifdef __cplusplus
}
#endif
#endif /* FAX_H */
