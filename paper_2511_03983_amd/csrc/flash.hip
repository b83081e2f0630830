// Tiled MFMA attention kernels for bf16 models (placeholder: reports "not handled" so that the plain
// kernels run).
#include "nn.h"

twist_status twist_attention_fwd_mfma(twist_ctx *, const void *, void *, float *, int, int, int, int, bool *done) {
  *done = false;
  return TWIST_OK;
}
twist_status twist_attention_bwd_mfma(twist_ctx *, const void *, const void *, const void *, const float *, float *, void *, int, int, int,
                                      int, bool *done) {
  *done = false;
  return TWIST_OK;
}
