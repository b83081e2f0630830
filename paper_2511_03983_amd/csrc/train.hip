// Subnet training entry points (placeholder until the kernels land).
#include "twist_internal.h"

twist_status twist_train_workspace_bytes(twist_ctx *ctx, const twist_subnet *, int, int, size_t *) {
  TW_FAIL(ctx, TWIST_ESHAPE, "training kernels are not built in this library");
}
twist_status twist_train_fwd_bwd(twist_ctx *ctx, twist_subnet *, const void *, const void *, int, int, void *, size_t, float *) {
  TW_FAIL(ctx, TWIST_ESHAPE, "training kernels are not built in this library");
}
twist_status twist_train_step(twist_ctx *ctx, twist_subnet *, const twist_opt_desc *) {
  TW_FAIL(ctx, TWIST_ESHAPE, "training kernels are not built in this library");
}
