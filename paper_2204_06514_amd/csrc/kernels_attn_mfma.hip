// Causal flash attention on the matrix cores (bf16, fp32 softmax statistics).
#include "fax_internal.h"

namespace fax {

bool attn_mfma_supported(int dtype, int B, int S, int H, int dh) {
  (void)dtype; (void)B; (void)S; (void)H; (void)dh;
  return false;
}

int attn_fwd_mfma(int, int, int, int, const void*, void*, float*, hipStream_t) {
  set_error("attention MFMA kernel not available");
  return FAX_ERR_UNSUPPORTED;
}

int attn_bwd_mfma(int, int, int, int, const void*, const void*, const float*, const void*, void*, float*, hipStream_t) {
  set_error("attention MFMA kernel not available");
  return FAX_ERR_UNSUPPORTED;
}

}  // namespace fax
