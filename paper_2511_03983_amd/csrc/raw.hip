// Kernel-level entry points for tests: one memory-bound step of the subnet pass in isolation (norms of Appendix A.1,
// rotary positions, FFN activations of Appendix A.1, the loss, the embedding), run by the same launchers
// twist_subnet_fwd_bwd uses, on the context's stream.  Argument checks only; no arithmetic lives here.
#include "nn.h"

extern "C" twist_status twist_norm_raw(twist_ctx *ctx, const float *x, const void *w, const void *b, int32_t T, void *y, float *stats,
                                       const void *dy, float *dx, void *dxb, float *dw, float *db, float *scratch, size_t scratch_floats) {
  if (!ctx || !x || !w || !y || !stats || T < 1) TW_FAIL(ctx, TWIST_EINVAL, "twist_norm_raw: null argument or empty input");
  const int bf = ctx->d.dtype == TWIST_BF16, rms = ctx->d.norm == TWIST_NORM_RMS, D = ctx->d.d_model;
  TW_TRY(twist_norm_fwd(ctx, bf, rms, x, w, b, y, stats, T, D, ctx->d.norm_eps));
  if (!dy) return TWIST_OK;
  if (!dx || !dw || !scratch) TW_FAIL(ctx, TWIST_EINVAL, "twist_norm_raw: the backward half needs dx, dw and scratch");
  if (scratch_floats < twist_norm_partial_floats(T, D))
    TW_FAIL(ctx, TWIST_ESHAPE, "twist_norm_raw: scratch of %zu floats is smaller than the %zu needed", scratch_floats, twist_norm_partial_floats(T, D));
  return twist_norm_bwd(ctx, bf, rms, dy, x, w, stats, dx, 0, dxb, dw, db, scratch, T, D);
}

extern "C" twist_status twist_rope_raw(twist_ctx *ctx, void *qkv, int32_t B, int32_t N, int32_t Hs, float sign, float *tab) {
  if (!ctx || !qkv || !tab || B < 1 || N < 1 || Hs < 1) TW_FAIL(ctx, TWIST_EINVAL, "twist_rope_raw: null argument or empty input");
  if (ctx->d.d_head % 2) TW_FAIL(ctx, TWIST_ESHAPE, "twist_rope_raw: d_head must be even");
  TW_TRY(twist_rope_table(ctx, tab, N, ctx->d.d_head, ctx->d.rope_theta));
  return twist_rope_apply(ctx, ctx->d.dtype == TWIST_BF16, qkv, tab, B, N, Hs, ctx->d.d_head, sign);
}

extern "C" twist_status twist_act_raw(twist_ctx *ctx, const void *gu, int32_t T, int32_t F, void *a, const void *da, void *dgu,
                                      const int32_t *keep, int32_t unit) {
  if (!ctx || !gu || !a || T < 1 || F < 1) TW_FAIL(ctx, TWIST_EINVAL, "twist_act_raw: null argument or empty input");
  if (keep && (unit < 1 || F % unit)) TW_FAIL(ctx, TWIST_ESHAPE, "twist_act_raw: F must be a whole number of blocks");
  const int bf = ctx->d.dtype == TWIST_BF16;
  TW_TRY(twist_act_fwd(ctx, bf, ctx->d.act, gu, a, T, F, keep, unit));
  if (!da) return TWIST_OK;
  if (!dgu) TW_FAIL(ctx, TWIST_EINVAL, "twist_act_raw: the backward half needs dgu");
  return twist_act_bwd(ctx, bf, ctx->d.act, gu, da, dgu, T, F, keep, unit);
}

extern "C" twist_status twist_ce_raw(twist_ctx *ctx, void *logits, int64_t ld, const int32_t *targets, int32_t T, float *rowloss, float *loss) {
  if (!ctx || !logits || !targets || !rowloss || !loss || T < 1) TW_FAIL(ctx, TWIST_EINVAL, "twist_ce_raw: null argument or empty input");
  if (ctx->d.vocab < 1 || ld < ctx->d.vocab) TW_FAIL(ctx, TWIST_ESHAPE, "twist_ce_raw: needs a vocabulary and a row stride that covers it");
  return twist_ce_fwd_bwd(ctx, ctx->d.dtype == TWIST_BF16, logits, ld, targets, rowloss, loss, T, ctx->d.vocab);
}

extern "C" twist_status twist_embed_raw(twist_ctx *ctx, const int32_t *tok, int32_t B, int32_t N, const void *tok_embed, const void *pos_embed,
                                        float *x, const float *dx, float *d_tok, float *d_pos) {
  if (!ctx || !tok || !tok_embed || !x || B < 1 || N < 1) TW_FAIL(ctx, TWIST_EINVAL, "twist_embed_raw: null argument or empty input");
  const int D = ctx->d.d_model;
  TW_TRY(twist_embed_fwd(ctx, ctx->d.dtype == TWIST_BF16, tok, tok_embed, pos_embed, x, B, N, D, ctx->d.vocab));
  if (!dx) return TWIST_OK;
  if (!d_tok) TW_FAIL(ctx, TWIST_EINVAL, "twist_embed_raw: the backward half needs d_tok");
  return twist_embed_bwd(ctx, tok, dx, d_tok, d_pos, B, N, D);
}

// ------------------------------------------------------------------------------------------------ no allocation
// twist_norm_raw for callers that cannot allocate (code under graph capture, tight serving loops): the per-chunk partial
// sums of the gain / bias gradients, which twist_norm_raw takes as a caller-provided scratch argument, live in a
// file-scope device array instead.  Every GPU the library runs on holds its own copy of the array at its own address
// until the process ends; the address is looked up once per device and kept.
namespace {
constexpr size_t kStaticScratchFloats = (size_t)2 << 20;  // 8 MiB: e.g. 8192 rows of 2048, or 4096 rows of 4096
constexpr int kMaxDevices = 64;
__device__ __align__(256) float scratch[kStaticScratchFloats];
float *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, null until first use there

// The array's name is only a host-side handle: the address kernels and copies must use comes from the runtime.
twist_status static_scratch(twist_ctx *ctx, float **out) {
  int dev = -1;
  TW_HIP(ctx, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) TW_FAIL(ctx, TWIST_EHIP, "twist_norm_raw_static: device ordinal %d outside [0, %d)", dev, kMaxDevices);
  if (!g_scratch_ptr[dev]) {
    float *p = nullptr;
    TW_HIP(ctx, hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch)));
    if (!p) TW_FAIL(ctx, TWIST_EHIP, "twist_norm_raw_static: the runtime returned no address for the scratch array");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return TWIST_OK;
}
}  // namespace

extern "C" twist_status twist_norm_raw_static(twist_ctx *ctx, const float *x, const void *w, const void *b, int32_t T, void *y, float *stats,
                                              const void *dy, float *dx, void *dxb, float *dw, float *db) {
  if (!ctx || !x || !w || !y || !stats || T < 1) TW_FAIL(ctx, TWIST_EINVAL, "twist_norm_raw_static: null argument or empty input");
  const int D = ctx->d.d_model;
  const size_t need = dy ? twist_norm_partial_floats(T, D) : 0;
  if (need > kStaticScratchFloats)
    TW_FAIL(ctx, TWIST_ESHAPE, "twist_norm_raw_static: %d rows of %d need %zu floats of scratch, the built-in array holds %zu (use twist_norm_raw)", T, D,
            need, kStaticScratchFloats);
  float *ptr = nullptr;
  if (dy) TW_TRY(static_scratch(ctx, &ptr));
  return twist_norm_raw(ctx, x, w, b, T, y, stats, dy, dx, dxb, dw, db, ptr, kStaticScratchFloats);
}
