// One forward + backward pass of a dense subnet, and the local optimizer step ("True TwIST" worker,
// Section 4.1): pre-norm transformer layer of Appendix A.2 at the subnet's own width, module outputs
// scaled by sqrt(N_full / N_sub) before each residual add (Section 3.4).
//
// Host orchestration only: every step is a kernel from nn.hip / gemm.hip / attention.hip enqueued on the
// context's stream.  Activations needed by the backward pass are kept in the caller's workspace.
#include <cmath>

#include "nn.h"

namespace {

// Bump allocator over the workspace; with base == nullptr it only measures.
struct Carver {
  char *base;
  size_t off = 0;
  explicit Carver(void *b) : base(static_cast<char *>(b)) {}
  template <class T = void> T *take(size_t bytes) {
    off = align_up(off, 256);
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off += bytes;
    return p;
  }
};

struct LayerBufs {
  void *h1, *qkv, *o, *h2, *gu, *a;
  float *lse, *o32;  // o32: unrounded attention output (bf16 models), feeds the backward pass's delta
};

struct Workspace {
  std::vector<float *> xs;    // residual stream before / inside / after every layer, fp32 [T,D]
  std::vector<float *> stats; // (mean, rstd) per row for each norm
  std::vector<LayerBufs> layer;
  float *dx, *rope_tab, *rowloss, *delta;
  float *splitk;        // scratch of the weight-gradient projections that are cut along the token dimension
  float *norm_partial;  // one block of per-chunk norm-gradient sums per norm layer (2 n_layers + 1), reduced in one launch at the end
  size_t norm_partial_stride;
  float *bias_partial;  // models with biases: per layer, the per-chunk column sums behind the four bias gradients
  size_t bias_partial_stride;
  void *dxb, *dxb2, *hf, *logits, *da, *dgu, *dh, *dout, *dqkv;
  int64_t ld_logits;
  size_t bytes;
};

void carve(const twist_ctx *ctx, const twist_subnet *sub, int B, int N, void *base, Workspace &w) {
  const twist_model_desc &d = ctx->d;
  const SubLayout &L = sub->plan->layout;
  const size_t es = ctx->esize();
  const size_t T = (size_t)B * N, D = d.d_model;
  const int nf = d.act == TWIST_ACT_SWIGLU ? 2 : 1;
  Carver c(base);
  w.xs.resize(2 * d.n_layers + 1);
  w.stats.resize(2 * d.n_layers + 1);
  for (auto &p : w.xs) p = c.take<float>(T * D * 4);
  for (auto &p : w.stats) p = c.take<float>(T * 2 * 4);
  w.layer.resize(d.n_layers);
  size_t hd_max = 0, f_max = 0, h_max = 0;
  for (int l = 0; l < d.n_layers; ++l) {
    const size_t HD = (size_t)L.heads_sub[l] * d.d_head, F = (size_t)L.ffn_sub[l] * d.ffn_granule;
    hd_max = std::max(hd_max, HD); f_max = std::max(f_max, F); h_max = std::max(h_max, (size_t)L.heads_sub[l]);
    LayerBufs &b = w.layer[l];
    b.h1 = c.take(T * D * es);
    b.qkv = c.take(T * 3 * HD * es);
    b.o = c.take(T * HD * es);
    b.o32 = es == 2 ? c.take<float>(T * HD * 4) : nullptr;
    b.lse = c.take<float>((size_t)B * L.heads_sub[l] * N * 4);
    b.h2 = c.take(T * D * es);
    b.gu = c.take(T * nf * F * es);
    b.a = c.take(T * F * es);
  }
  w.dx = c.take<float>(T * D * 4);
  w.dxb = c.take(T * D * es);
  w.dxb2 = c.take(T * D * es);
  w.hf = c.take(T * D * es);
  w.ld_logits = (int64_t)align_up((size_t)d.vocab, 8);
  w.logits = d.vocab ? c.take(T * w.ld_logits * es) : nullptr;
  w.rowloss = c.take<float>(std::max<size_t>(T, 1024) * 4);
  w.rope_tab = c.take<float>((size_t)N * d.d_head * 4);
  w.splitk = c.take<float>(kSplitkFloats * 4);
  w.norm_partial_stride = align_up(twist_norm_partial_floats((int)T, (int)D), 64);
  w.norm_partial = c.take<float>(w.norm_partial_stride * (2 * (size_t)d.n_layers + 1) * 4);
  w.bias_partial_stride = d.has_bias ? align_up(twist_colsum_partial_floats((int)T, (int)(2 * D + nf * f_max + 3 * hd_max)), 64) : 0;
  w.bias_partial = c.take<float>(w.bias_partial_stride * (size_t)d.n_layers * 4);
  w.delta = c.take<float>((size_t)B * h_max * N * 4);
  w.da = c.take(T * f_max * es);
  w.dgu = c.take(T * nf * f_max * es);
  w.dh = c.take(T * D * es);
  w.dout = c.take(T * hd_max * es);
  w.dqkv = c.take(T * 3 * hd_max * es);
  w.bytes = align_up(c.off, 256);
}

// The weight-gradient projections of the backward pass only write parameter gradients, nothing downstream in
// the pass reads them, and on their own most of them have too few output tiles to fill the chip.  They are
// therefore enqueued on a second stream, where they run next to the chain of input-gradient kernels.  Slot i
// (0 = FFN down, 1 = FFN up/gate, 2 = attention output, 3 = q/k/v) has a "ready" event (the main stream has
// produced the operands) and a "done" event (the side stream has consumed them; the main stream waits for it
// before it overwrites those operands one layer later).
struct SideStream {
  twist_ctx *ctx;
  bool on = false, recorded[4] = {false, false, false, false};
  twist_status init() {
    on = ctx->overlap;
    if (!on) return TWIST_OK;
    if (!ctx->side) {
      TW_HIP(ctx, hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking));
      for (int i = 0; i < 4; ++i) {
        TW_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_ready[i], hipEventDisableTiming));
        TW_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_done[i], hipEventDisableTiming));
      }
    }
    return TWIST_OK;
  }
  hipStream_t stream() const { return on ? ctx->side : nullptr; }
  twist_status fork(int i) {  // everything enqueued on the main stream so far precedes the side stream's next kernel
    if (!on) return TWIST_OK;
    TW_HIP(ctx, hipEventRecord(ctx->ev_ready[i], ctx->stream));
    TW_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->ev_ready[i], 0));
    return TWIST_OK;
  }
  twist_status done(int i) {
    if (!on) return TWIST_OK;
    TW_HIP(ctx, hipEventRecord(ctx->ev_done[i], ctx->side));
    recorded[i] = true;
    return TWIST_OK;
  }
  twist_status wait_done(int i) {  // the main stream may overwrite slot i's operands after this
    if (!on || !recorded[i]) return TWIST_OK;
    TW_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev_done[i], 0));
    return TWIST_OK;
  }
};

twist_status check_train_shape(twist_ctx *ctx, const twist_subnet *sub, int B, int N) {
  const twist_model_desc &d = ctx->d;
  if (B < 1 || N < 1) TW_FAIL(ctx, TWIST_ESHAPE, "fwd_bwd: batch %d x %d tokens is empty", B, N);
  if (N > d.max_seq) TW_FAIL(ctx, TWIST_ESHAPE, "fwd_bwd: %d tokens exceed max_seq=%d", N, d.max_seq);
  if (d.has_bias && d.act == TWIST_ACT_SWIGLU) TW_FAIL(ctx, TWIST_ESHAPE, "fwd_bwd: gated FFN with biases is not supported");
  if (d.d_head > 256) TW_FAIL(ctx, TWIST_ESHAPE, "fwd_bwd: d_head=%d above 256 is not supported", d.d_head);
  if ((int64_t)B * N * std::max(d.d_model, d.vocab) >= (1ll << 40)) TW_FAIL(ctx, TWIST_ESHAPE, "fwd_bwd: batch too large");
  (void)sub;
  return TWIST_OK;
}

}  // namespace

twist_status twist_train_workspace_bytes(twist_ctx *ctx, const twist_subnet *sub, int B, int N, size_t *bytes) {
  TW_TRY(check_train_shape(ctx, sub, B, N));
  Workspace w;
  carve(ctx, sub, B, N, nullptr, w);
  *bytes = w.bytes;
  return TWIST_OK;
}

twist_status twist_train_fwd_bwd(twist_ctx *ctx, twist_subnet *sub, const void *inputs, const void *targets, int B, int N, void *ws,
                                 size_t ws_bytes, float *loss_dev, bool forward_only, const twist_plan *mask_plan, int mask_row) {
  TW_TRY(check_train_shape(ctx, sub, B, N));
  if (!forward_only && !sub->grads) TW_FAIL(ctx, TWIST_ESHAPE, "fwd_bwd: subnet was extracted without gradient storage");
  if (reinterpret_cast<uintptr_t>(ws) % 256) TW_FAIL(ctx, TWIST_ESHAPE, "fwd_bwd: workspace must be 256-byte aligned");
  Workspace w;
  carve(ctx, sub, B, N, ws, w);
  if (ws_bytes < w.bytes) TW_FAIL(ctx, TWIST_ESHAPE, "fwd_bwd: workspace of %zu bytes is smaller than the %zu needed", ws_bytes, w.bytes);

  const twist_model_desc &d = ctx->d;
  const SubLayout &L = sub->plan->layout;
  const int bf = d.dtype == TWIST_BF16, es = ctx->esize();
  const int T = B * N, D = d.d_model, dh = d.d_head;
  const int rms = d.norm == TWIST_NORM_RMS;
  const int nf = d.act == TWIST_ACT_SWIGLU ? 2 : 1;
  const bool lm = d.vocab > 0;
  const bool um = d.out_unit_major != 0;  // output projections stored [in, out]: the three GEMM forms rotate
  // Masked variant (Section 4.1, "Masked TwIST"): `sub` is a full-width subnet and the blocks that row `mask_row` of
  // `mask_plan` does not name are zeroed where they enter the output projections (attention output columns,
  // FFN activations) and where the gradient comes back through the same places, inside the kernels that produce
  // those tensors (attention forward / backward, activation forward / backward); the module scales are those of
  // the masked widths.  Everything else is the ordinary pass, with the same number of launches.
  if (mask_plan) {
    for (int l = 0; l < d.n_layers; ++l)
      if (L.heads_sub[l] != d.n_heads || L.ffn_sub[l] != ctx->n_ffn_units())
        TW_FAIL(ctx, TWIST_ESHAPE, "masked pass: the subnet must hold every block of layer %d", l);
  }
  // per-block mask of layer l (device table: entry < 0 = block not kept), handed to the kernels that produce the attention
  // output, the FFN activation and their gradients; null in the ordinary pass
  auto keep_of = [&](int l, int kind) -> const int32_t * {
    if (!mask_plan) return nullptr;
    const PlanEntry &pe = mask_plan->at(l, kind);
    return pe.d_inv + (size_t)mask_row * pe.n_full;
  };
  auto kept = [&](int l, int kind, int full) { return mask_plan ? mask_plan->at(l, kind).n_sub : full; };
  const int scale_mode = mask_plan ? mask_plan->scale_mode : sub->plan->scale_mode;
  auto P = [&](const Slot &s) -> void * { return s.off < 0 ? nullptr : sub->params + s.off * es; };
  auto G = [&](const Slot &s) -> float * { return s.off < 0 ? nullptr : sub->grads + s.off; };
  auto gemm = [&](GemmLayout lay, int M, int Nn, int K, const void *A, int64_t lda, const void *Bm, int64_t ldb, void *out, int64_t ldc, int out_f32,
                  float alpha = 1.f, const void *bias = nullptr, const float *residual = nullptr) {
    GemmEpilogue e;
    e.alpha = alpha; e.bias = bias; e.residual = residual; e.out = out; e.out_f32 = out_f32;
    return twist_gemm(ctx, bf, lay, M, Nn, K, A, lda, Bm, ldb, ldc, e);
  };
  // Norm backward of norm layer `idx` (2l, 2l+1: the two norms of layer l; 2 n_layers: the final norm).  Its parameter
  // gradients are left as per-chunk partial sums in the layer's own block and summed for all layers by one launch at
  // the end of the pass, which takes 2 n_layers small kernels off the chain of dependent kernels.
  std::vector<ColReduce> reduce_items;
  auto norm_bwd = [&](int idx, const void *dy, const float *x, const void *nw, int accumulate, void *dxb, float *dw, float *db) {
    float *part = w.norm_partial + (size_t)idx * w.norm_partial_stride;
    reduce_items.push_back({part, dw, 2 * (int64_t)D, D, 1.f});
    if (db) reduce_items.push_back({part + D, db, 2 * (int64_t)D, D, 1.f});
    return twist_norm_bwd(ctx, bf, rms, dy, x, nw, w.stats[idx], w.dx, accumulate, dxb, dw, db, part, T, D, true);
  };

  // ------------------------------------------------------------------------------------ forward
  if (lm) {
    TW_TRY(twist_embed_fwd(ctx, bf, static_cast<const int32_t *>(inputs), P(L.global[TWIST_TOK_EMBED]), P(L.global[TWIST_POS_EMBED]), w.xs[0], B, N, D,
                           d.vocab));
  } else {
    TW_TRY(twist_cast_in(ctx, bf, inputs, w.xs[0], (int64_t)T * D));
  }
  if (d.use_rope) TW_TRY(twist_rope_table(ctx, w.rope_tab, N, dh, d.rope_theta));

  for (int l = 0; l < d.n_layers; ++l) {
    const int Hs = L.heads_sub[l], HD = Hs * dh, F = L.ffn_sub[l] * d.ffn_granule;
    const float c_a = scale_mode ? sqrtf((float)d.n_heads / (float)kept(l, TWIST_KIND_HEAD, Hs)) : 1.f;
    const float c_f = scale_mode ? sqrtf((float)ctx->n_ffn_units() / (float)kept(l, TWIST_KIND_FFN, L.ffn_sub[l])) : 1.f;
    const LayerBufs &b = w.layer[l];
    TW_TRY(twist_norm_fwd(ctx, bf, rms, w.xs[2 * l], P(L.at(l, TWIST_NORM1_W)), P(L.at(l, TWIST_NORM1_B)), b.h1, w.stats[2 * l], T, D, d.norm_eps));
    TW_TRY(gemm(GEMM_NT, T, 3 * HD, D, b.h1, D, P(L.at(l, TWIST_WQ)), D, b.qkv, 3 * HD, 0, 1.f, P(L.at(l, TWIST_BQ))));
    if (d.use_rope) TW_TRY(twist_rope_apply(ctx, bf, b.qkv, w.rope_tab, B, N, Hs, dh, 1.f));
    TW_TRY(twist_attention_fwd(ctx, bf, b.qkv, b.o, b.o32, b.lse, B, N, Hs, dh, keep_of(l, TWIST_KIND_HEAD)));
    if (um) TW_TRY(gemm(GEMM_NN, T, D, HD, b.o, HD, P(L.at(l, TWIST_WO)), D, w.xs[2 * l + 1], D, 1, c_a, P(L.at(l, TWIST_BO)), w.xs[2 * l]));
    else TW_TRY(gemm(GEMM_NT, T, D, HD, b.o, HD, P(L.at(l, TWIST_WO)), HD, w.xs[2 * l + 1], D, 1, c_a, P(L.at(l, TWIST_BO)), w.xs[2 * l]));
    TW_TRY(twist_norm_fwd(ctx, bf, rms, w.xs[2 * l + 1], P(L.at(l, TWIST_NORM2_W)), P(L.at(l, TWIST_NORM2_B)), b.h2, w.stats[2 * l + 1], T, D, d.norm_eps));
    const Slot &w1 = nf == 2 ? L.at(l, TWIST_W_GATE) : L.at(l, TWIST_W_UP);
    TW_TRY(gemm(GEMM_NT, T, nf * F, D, b.h2, D, P(w1), D, b.gu, nf * F, 0, 1.f, P(L.at(l, TWIST_B_UP))));
    TW_TRY(twist_act_fwd(ctx, bf, d.act, b.gu, b.a, T, F, keep_of(l, TWIST_KIND_FFN), d.ffn_granule));
    if (um) TW_TRY(gemm(GEMM_NN, T, D, F, b.a, F, P(L.at(l, TWIST_W_DOWN)), D, w.xs[2 * l + 2], D, 1, c_f, P(L.at(l, TWIST_B_DOWN)), w.xs[2 * l + 1]));
    else TW_TRY(gemm(GEMM_NT, T, D, F, b.a, F, P(L.at(l, TWIST_W_DOWN)), F, w.xs[2 * l + 2], D, 1, c_f, P(L.at(l, TWIST_B_DOWN)), w.xs[2 * l + 1]));
  }

  // ------------------------------------------------------------------------------------ loss and its gradient
  float *x_last = w.xs[2 * d.n_layers];
  if (lm) {
    const int V = d.vocab;
    const Slot &wout = d.tied_head ? L.global[TWIST_TOK_EMBED] : L.global[TWIST_LM_HEAD];
    TW_TRY(twist_norm_fwd(ctx, bf, rms, x_last, P(L.global[TWIST_FINAL_NORM_W]), P(L.global[TWIST_FINAL_NORM_B]), w.hf, w.stats[2 * d.n_layers], T, D,
                          d.norm_eps));
    TW_TRY(gemm(GEMM_NT, T, V, D, w.hf, D, P(wout), D, w.logits, w.ld_logits, 0));
    TW_TRY(twist_ce_fwd_bwd(ctx, bf, w.logits, w.ld_logits, static_cast<const int32_t *>(targets), w.rowloss, loss_dev, T, V));
    if (forward_only) return TWIST_OK;
    // projection weight gradient, then the gradient flowing back into the final norm
    TW_TRY(gemm(GEMM_TN, V, D, T, w.logits, w.ld_logits, w.hf, D, G(wout), D, 1));
    {
      // gradient of the final normed input: few output tiles ([T, d_model]) and a contraction as long as the vocabulary, so
      // it may be cut along the vocabulary like the weight gradients (the scratch is free here: the second stream's
      // projections of this pass have not started, those of the previous pass were joined before it returned)
      GemmEpilogue e;
      e.out = w.dh; e.out_f32 = 0;
      e.splitk_ws = w.splitk; e.splitk_floats = kSplitkFloats;
      TW_TRY(twist_gemm(ctx, bf, GEMM_NN, T, D, V, w.logits, w.ld_logits, P(wout), D, D, e));
    }
    TW_TRY(norm_bwd(2 * d.n_layers, w.dh, x_last, P(L.global[TWIST_FINAL_NORM_W]), 0, w.dxb, G(L.global[TWIST_FINAL_NORM_W]),
                    G(L.global[TWIST_FINAL_NORM_B])));
  } else {
    TW_TRY(twist_mse_fwd_bwd(ctx, bf, x_last, targets, w.dx, w.dxb, w.rowloss, loss_dev, (int64_t)T * D));
    if (forward_only) return TWIST_OK;
  }

  // ------------------------------------------------------------------------------------ backward through the layers
  SideStream side{ctx};
  TW_TRY(side.init());
  auto wgrad = [&](int M, int Nn, const void *A, int64_t lda, const void *Bm, int64_t ldb, float *out, float alpha) {
    GemmEpilogue e;
    e.alpha = alpha; e.out = out; e.out_f32 = 1;
    e.splitk_ws = w.splitk; e.splitk_floats = kSplitkFloats;  // one scratch: these projections are serialised on their stream
    return twist_gemm(ctx, bf, GEMM_TN, M, Nn, T, A, lda, Bm, ldb, Nn, e, side.stream());
  };
  void *gx = w.dxb, *gx_other = w.dxb2;  // gradient of the residual stream in activation type: current, spare
  for (int l = d.n_layers - 1; l >= 0; --l) {
    const int Hs = L.heads_sub[l], HD = Hs * dh, F = L.ffn_sub[l] * d.ffn_granule;
    const float c_a = scale_mode ? sqrtf((float)d.n_heads / (float)kept(l, TWIST_KIND_HEAD, Hs)) : 1.f;
    const float c_f = scale_mode ? sqrtf((float)ctx->n_ffn_units() / (float)kept(l, TWIST_KIND_FFN, L.ffn_sub[l])) : 1.f;
    const LayerBufs &b = w.layer[l];
    const Slot &w1 = nf == 2 ? L.at(l, TWIST_W_GATE) : L.at(l, TWIST_W_UP);
    // FFN branch: y = c_f (a W_down^T + b_down)
    // bias gradients: per-chunk column sums now (into this layer's block), reduced with everything else at the end
    float *bias_part = w.bias_partial + (size_t)l * w.bias_partial_stride;
    auto bias_grad = [&](const void *src, int64_t ld, float alpha, float *out, int n) {
      float *part = bias_part;
      bias_part += twist_colsum_partial_floats(T, n);
      reduce_items.push_back({part, out, (int64_t)n, n, alpha});
      return twist_colsum(ctx, bf, src, ld, alpha, out, part, T, n, true);
    };
    if (L.at(l, TWIST_B_DOWN).off >= 0) TW_TRY(bias_grad(gx, D, c_f, G(L.at(l, TWIST_B_DOWN)), D));
    TW_TRY(side.fork(0));
    if (um) TW_TRY(wgrad(F, D, b.a, F, gx, D, G(L.at(l, TWIST_W_DOWN)), c_f));
    else TW_TRY(wgrad(D, F, gx, D, b.a, F, G(L.at(l, TWIST_W_DOWN)), c_f));
    TW_TRY(side.done(0));
    if (um) TW_TRY(gemm(GEMM_NT, T, F, D, gx, D, P(L.at(l, TWIST_W_DOWN)), D, w.da, F, 0, c_f));
    else TW_TRY(gemm(GEMM_NN, T, F, D, gx, D, P(L.at(l, TWIST_W_DOWN)), F, w.da, F, 0, c_f));
    TW_TRY(side.wait_done(1));
    TW_TRY(twist_act_bwd(ctx, bf, d.act, b.gu, w.da, w.dgu, T, F, keep_of(l, TWIST_KIND_FFN), d.ffn_granule));
    if (L.at(l, TWIST_B_UP).off >= 0) TW_TRY(bias_grad(w.dgu, nf * F, 1.f, G(L.at(l, TWIST_B_UP)), nf * F));
    TW_TRY(side.fork(1));
    TW_TRY(wgrad(nf * F, D, w.dgu, nf * F, b.h2, D, G(w1), 1.f));
    TW_TRY(side.done(1));
    TW_TRY(gemm(GEMM_NN, T, D, nf * F, w.dgu, nf * F, P(w1), D, w.dh, D, 0));
    TW_TRY(side.wait_done(2));
    TW_TRY(norm_bwd(2 * l + 1, w.dh, w.xs[2 * l + 1], P(L.at(l, TWIST_NORM2_W)), 1, gx_other, G(L.at(l, TWIST_NORM2_W)), G(L.at(l, TWIST_NORM2_B))));
    // attention branch: y = c_a (o C_attn^T + b_o)
    if (L.at(l, TWIST_BO).off >= 0) TW_TRY(bias_grad(gx_other, D, c_a, G(L.at(l, TWIST_BO)), D));
    TW_TRY(side.fork(2));
    if (um) TW_TRY(wgrad(HD, D, b.o, HD, gx_other, D, G(L.at(l, TWIST_WO)), c_a));
    else TW_TRY(wgrad(D, HD, gx_other, D, b.o, HD, G(L.at(l, TWIST_WO)), c_a));
    TW_TRY(side.done(2));
    if (um) TW_TRY(gemm(GEMM_NT, T, HD, D, gx_other, D, P(L.at(l, TWIST_WO)), D, w.dout, HD, 0, c_a));
    else TW_TRY(gemm(GEMM_NN, T, HD, D, gx_other, D, P(L.at(l, TWIST_WO)), HD, w.dout, HD, 0, c_a));
    TW_TRY(side.wait_done(3));
    TW_TRY(twist_attention_bwd(ctx, bf, b.qkv, b.o32, w.dout, b.lse, w.delta, w.dqkv, B, N, Hs, dh, d.use_rope ? w.rope_tab : nullptr,
                               keep_of(l, TWIST_KIND_HEAD)));
    if (L.at(l, TWIST_BQ).off >= 0) TW_TRY(bias_grad(w.dqkv, 3 * HD, 1.f, G(L.at(l, TWIST_BQ)), 3 * HD));
    TW_TRY(side.fork(3));
    TW_TRY(wgrad(3 * HD, D, w.dqkv, 3 * HD, b.h1, D, G(L.at(l, TWIST_WQ)), 1.f));
    TW_TRY(side.done(3));
    TW_TRY(gemm(GEMM_NN, T, D, 3 * HD, w.dqkv, 3 * HD, P(L.at(l, TWIST_WQ)), D, w.dh, D, 0));
    TW_TRY(side.wait_done(0));
    TW_TRY(norm_bwd(2 * l, w.dh, w.xs[2 * l], P(L.at(l, TWIST_NORM1_W)), 1, gx, G(L.at(l, TWIST_NORM1_W)), G(L.at(l, TWIST_NORM1_B))));
  }
  TW_TRY(twist_col_reduce_batch(ctx, reduce_items.data(), (int)reduce_items.size(), T));
  for (int i = 0; i < 4; ++i) TW_TRY(side.wait_done(i));  // join: the caller's stream sees the whole pass
  (void)gx_other;

  if (lm) {
    // token embedding: rows used by this batch receive dx (on top of the projection gradient when tied)
    const Slot &te = L.global[TWIST_TOK_EMBED];
    if (!d.tied_head) TW_TRY(twist_zero_f32(ctx, G(te), (int64_t)te.rows * te.cols));
    TW_TRY(twist_embed_bwd(ctx, static_cast<const int32_t *>(inputs), w.dx, G(te), G(L.global[TWIST_POS_EMBED]), B, N, D));
    const Slot &pe = L.global[TWIST_POS_EMBED];
    if (pe.off >= 0 && N < pe.rows) TW_TRY(twist_zero_f32(ctx, G(pe) + (size_t)N * D, (int64_t)(pe.rows - N) * D));
  }
  return TWIST_OK;
}

twist_status twist_train_step(twist_ctx *ctx, twist_subnet *sub, const twist_opt_desc *opt) {
  if (!sub->grads) TW_FAIL(ctx, TWIST_ESHAPE, "step: subnet was extracted without gradient storage");
  const SubLayout &L = sub->plan->layout;
  const int bf = ctx->d.dtype == TWIST_BF16;
  if (opt->kind == TWIST_OPT_SGD) return twist_sgd(ctx, bf, sub->params, sub->master, sub->grads, L.n_total, opt->lr);
  if (opt->kind == TWIST_OPT_ADAMW) {
    if (!sub->adam_m) TW_FAIL(ctx, TWIST_ESHAPE, "step: AdamW needs a subnet extracted with TWIST_STORE_ADAMW");
    sub->step_count += 1;
    return twist_adamw(ctx, bf, sub->params, sub->master, sub->grads, sub->adam_m, sub->adam_v, L.n_total, L.n_matrix, opt->lr, opt->beta1, opt->beta2,
                       opt->eps, opt->weight_decay, sub->step_count);
  }
  TW_FAIL(ctx, TWIST_EINVAL, "step: unknown optimizer %d", opt->kind);
}
