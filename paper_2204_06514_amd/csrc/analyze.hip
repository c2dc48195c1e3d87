// Host-side static analysis of a model on a data x tensor device mesh: what one device holds and
// does per training step, and how long this library would take for it on one MI355X.
//
// The paper observes that such figures follow from the model's description alone (Sec. 2.1:
// memory requirements, latency estimates) and places tensors on a logical device mesh by naming
// the mesh axis each tensor axis is split over (Sec. 2.2); its tensor parallelism splits heads and
// every large weight over the model axis and requires the head count to divide (Sec. 3.2).
// Nothing here touches a GPU; sizes come from the same layout functions the entry points use and
// GEMM times from the launch planner's own cost model, so the analysis cannot drift from the code.
#include <cmath>
#include <cstring>

#include "fax_internal.h"

namespace fax {

// Measured cost of the attention kernels per 1000 (query, key) pairs under the causal mask, in
// nanoseconds, by head width (forward, dQ, dK/dV kernels at S = 2048 on 128 (b, h) problems or more).
struct AttnCost {
  double fwd, dq, dkv;
};
static AttnCost attn_cost(int dh, int S, int dtype) {
  if (dtype == FAX_BF16 && S % 128 == 0 && dh == 128) return {0.59, 0.84, 1.48};
  if (dtype == FAX_BF16 && S % 128 == 0 && dh == 64) return {0.32, 0.42, 0.63};
  const double c = 0.25 * dh;  // the scalar kernels: a few TFLOP/s
  return {c, 2 * c, 2 * c};
}

static double block_params(double D, double Hd, double F) {
  return D * 3 * Hd + 3 * Hd + Hd * D + D + 4 * D + D * F + F + F * D + D;
}

}  // namespace fax

using namespace fax;

extern "C" int fax_analyze(const FaxModelDims* g, const FaxMesh* mesh, FaxAnalysis* out) {
  if (!g || !mesh || !out) {
    set_error("fax_analyze: NULL argument");
    return FAX_ERR_INVALID_ARG;
  }
  FAX_TRY(fax_block_dims_check(&g->blk));
  if (g->L <= 0 || g->V <= 0 || g->S_max < g->blk.S) {
    set_error("model dims: L=%d V=%d S_max=%d (S=%d)", g->L, g->V, g->S_max, g->blk.S);
    return FAX_ERR_INVALID_ARG;
  }
  const int dp = mesh->data, tp = mesh->tensor;
  if (dp <= 0 || tp <= 0) {
    set_error("mesh %d x %d", dp, tp);
    return FAX_ERR_INVALID_ARG;
  }
  if (g->blk.B % dp) {
    set_error("batch %d is not divisible by the data axis (%d)", g->blk.B, dp);
    return FAX_ERR_INVALID_ARG;
  }
  if (g->blk.H % tp) {
    set_error("%d attention heads are not divisible by the tensor axis (%d)", g->blk.H, tp);
    return FAX_ERR_INVALID_ARG;
  }
  if (g->blk.F % tp) {
    set_error("feed-forward width %d is not divisible by the tensor axis (%d)", g->blk.F, tp);
    return FAX_ERR_INVALID_ARG;
  }
  FaxAnalysis a;
  memset(&a, 0, sizeof(a));
  a.local = *g;
  a.local.blk.B = g->blk.B / dp;
  a.local.blk.H = g->blk.H / tp;
  a.local.blk.F = g->blk.F / tp;
  // rows of the token table: split only if every rank's slice stays on the MFMA path (a multiple of 128 rows)
  a.local.V = g->V % (tp * 128) == 0 ? g->V / tp : g->V;
  if (tp > 1) a.local.blk.flags |= FAX_FLAG_TP_PARTIAL;
  const FaxBlockDims& b = a.local.blk;
  const int L = g->L, V = a.local.V;
  const double es = b.dtype == FAX_F32 ? 4.0 : 2.0;
  const int T = b.B * b.S, D = b.D, Hd = b.H * b.dh, F = b.F;

  // parameters
  a.params_global = L * block_params(g->blk.D, (double)g->blk.H * g->blk.dh, g->blk.F) + (double)g->V * D +
                    (double)g->S_max * D + 2.0 * D;
  a.params_local = L * block_params(D, Hd, F) + (double)V * D + (double)g->S_max * D + 2.0 * D;

  // memory, as the entry points size it
  FaxSavedLayout sl;
  FAX_TRY(fax_block_saved_layout(&b, &sl));
  size_t train_ws = 0;
  FAX_TRY(fax_train_workspace_bytes(&a.local, &train_ws));
  a.bytes_master = 4.0 * a.params_local;
  a.bytes_moments = 8.0 * a.params_local;
  a.bytes_grads = 4.0 * a.params_local;
  a.bytes_lowp = b.dtype == FAX_BF16 ? 2.0 * a.params_local : 0.0;
  a.bytes_saved = (double)L * (double)sl.total;
  a.bytes_workspace = (double)train_ws - a.bytes_saved;
  a.bytes_total = a.bytes_master + a.bytes_moments + a.bytes_grads + a.bytes_lowp + (double)train_ws;

  // work: forward GEMMs [M, N, K] of a block, the head, and their two backward products each
  const int fwd[4][3] = {{T, 3 * Hd, D}, {T, D, Hd}, {T, F, D}, {T, D, F}};
  double gemm_flop_fwd = 0, us_gemm = 0;
  for (const auto& s : fwd) {
    gemm_flop_fwd += 2.0 * s[0] * s[1] * s[2];
    us_gemm += gemm_time_estimate_us(s[0], s[1], s[2], false);  // forward
    us_gemm += gemm_time_estimate_us(s[0], s[2], s[1], false);  // input gradient: contraction over N
    us_gemm += gemm_time_estimate_us(s[2], s[1], s[0], true);   // weight gradient: contraction over the tokens
  }
  gemm_flop_fwd *= L;
  us_gemm *= L;
  gemm_flop_fwd += 2.0 * T * (double)D * V;
  us_gemm += gemm_time_estimate_us(T, V, D, false) + gemm_time_estimate_us(T, D, V, false) +
             gemm_time_estimate_us(V, D, T, true);
  const double pairs = (double)b.B * b.H * b.S * b.S / 2.0;  // (query, key) pairs under the mask, per layer
  const double attn_flop_fwd = L * 4.0 * pairs * b.dh;
  a.flop_step = 3.0 * (gemm_flop_fwd + attn_flop_fwd);
  a.flop_step_unhalved = 3.0 * (gemm_flop_fwd + 2.0 * attn_flop_fwd);
  const AttnCost ac = attn_cost(b.dh, b.S, b.dtype);
  a.ms_attention = L * pairs * (ac.fwd + ac.dq + ac.dkv) * 1e-9;
  a.ms_gemm = us_gemm * 1e-3;

  // bandwidth-bound kernels: algorithmic bytes and launches
  const double act = (double)T * D * es;
  const int n_ln = 2 * L + 1;
  double bytes = n_ln * (2 * act)              // LayerNorm forward: read x, write h
                 + n_ln * (4 * act)            // backward: read dh, x, residual gradient; write dx
                 + 2.0 * T * (double)V * es    // loss: read the logits, write their gradient over them
                 + 2 * act + 2 * act           // embedding forward and backward
                 + (28.0 + (b.dtype == FAX_BF16 ? 2.0 : 0.0)) * a.params_local;  // AdamW
  a.hbm_bytes_step = bytes;
  const int n_tensors = 12 * L + 4;
  const int bw_launches = n_ln + 2 * n_ln + 1 + 3 + n_tensors;
  a.launches = L * (4 * 3 + 3) + 3 + bw_launches;
  a.ms_bandwidth = bytes / 4.5e9 + bw_launches * 0.006;  // 4.5 TB/s sustained, ~6 us per small launch
  a.ms_step = a.ms_gemm + a.ms_attention + a.ms_bandwidth;

  // exchange volume per step and device
  a.bytes_tensor_axis = tp > 1 ? L * 4.0 * act : 0.0;       // p_attn, p_mlp forward; dh1, dh2 backward
  a.bytes_data_axis = dp > 1 ? 4.0 * a.params_local : 0.0;  // one pass over the fp32 gradients
  *out = a;
  return FAX_OK;
}
