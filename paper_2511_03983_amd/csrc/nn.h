// Kernel launchers of the subnet training path (internal).  `bf16` selects the activation / weight
// storage type: 0 = fp32, 1 = bf16.  Residual stream, statistics, gradients of parameters: always fp32.
#pragma once
#include "twist_internal.h"

struct GemmEpilogue {
  float alpha = 1.f;             // out = alpha * (A.B + bias) + residual
  const void *bias = nullptr;    // [N], activation type
  const float *residual = nullptr;  // [M,N] fp32
  void *out = nullptr;           // [M,N]
  int out_f32 = 0;               // 1: out is fp32, 0: out is the activation type
  // Optional scratch for products with few output tiles and a long contraction (weight gradients): when given (and no
  // bias/residual is asked for) the contraction may be cut into parts whose fp32 partial products go here and are then
  // summed in a fixed order.  At most 256 tiles of 256 x 256 floats are ever needed.
  float *splitk_ws = nullptr;
  size_t splitk_floats = 0;
};
constexpr size_t kSplitkFloats = (size_t)256 * 256 * 256;

enum GemmLayout {
  GEMM_NT = 0,  // A [M,K] row-major, B [N,K] row-major         (y = x W^T)
  GEMM_NN = 1,  // A [M,K] row-major, B [K,N] row-major         (dx = dy W)
  GEMM_TN = 2   // A stored [K,M] row-major, B stored [K,N]     (dW = dy^T x)
};

// C[M,N] = epilogue( op(A) op(B) ), fp32 accumulation.  lda/ldb are the row strides of the stored operands.
// `st`: stream to enqueue on (null: the context's stream).
twist_status twist_gemm(twist_ctx *ctx, int bf16, GemmLayout lay, int M, int N, int K, const void *A, int64_t lda, const void *B,
                        int64_t ldb, int64_t ldc, const GemmEpilogue &ep, hipStream_t st = nullptr);

// causal multi-head attention on a fused qkv buffer [T, 3*Hs*dh] (q | k | v); o [T, Hs*dh]; lse [B,Hs,N] fp32.
// o32 (may be null): the same output unrounded, [T, Hs*dh] fp32, written by the tiled bf16 kernels only; the
// tiled backward kernels need it (without it, or on shapes they do not cover, the plain kernels run).
// keep (may be null; device, one entry per head): heads with keep[h] < 0 are masked (Masked TwIST, Section 4.1): the forward
// kernels write zeros for them, the backward kernels zero gradients, and neither visits their keys.
twist_status twist_attention_fwd(twist_ctx *ctx, int bf16, const void *qkv, void *o, float *o32, float *lse, int B, int N, int Hs, int dh,
                                 const int32_t *keep = nullptr);
// dqkv [T, 3*Hs*dh] from do [T, Hs*dh]; delta [B,Hs,N] fp32 scratch (sum_j p_ij dp_ij, written by the dq pass).
// rope_tab (may be null): the table of twist_rope_table; when given, the q and k gradients are also taken back through
// the rotary embedding (inside the tiled kernels where they cover the shape, else by twist_rope_apply afterwards).
twist_status twist_attention_bwd(twist_ctx *ctx, int bf16, const void *qkv, const float *o32, const void *dout, const float *lse, float *delta,
                                 void *dqkv, int B, int N, int Hs, int dh, const float *rope_tab, const int32_t *keep = nullptr);

twist_status twist_embed_fwd(twist_ctx *ctx, int bf16, const int32_t *tok, const void *tok_embed, const void *pos_embed, float *x, int B, int N, int D, int vocab);
twist_status twist_embed_bwd(twist_ctx *ctx, const int32_t *tok, const float *dx, float *d_tok, float *d_pos, int B, int N, int D);
twist_status twist_zero_f32(twist_ctx *ctx, float *p, int64_t n);
twist_status twist_cast_in(twist_ctx *ctx, int bf16, const void *src, float *dst, int64_t n);

// y = norm(x) * w (+ b); stats[2*T] = (mean or 0, rstd) per row
twist_status twist_norm_fwd(twist_ctx *ctx, int bf16, int rms, const float *x, const void *w, const void *b, void *y, float *stats, int T, int D, float eps);
// dx (+)= norm backward of dy; dxb = activation-type copy of the resulting dx (may be null);
// dw, db (fp32, overwritten; db may be null); partial: scratch of at least norm_partial_floats(T, D).
// With defer_reduce the per-chunk partial sums are left in `partial` and dw/db are not written: the caller later sums
// many such buffers with one twist_col_reduce_batch launch (items {partial, dw, 2 D, D, 1} and {partial + D, db, 2 D, D, 1};
// same summation order, hence the same bits).
twist_status twist_norm_bwd(twist_ctx *ctx, int bf16, int rms, const void *dy, const float *x, const void *w, const float *stats, float *dx,
                            int accumulate, void *dxb, float *dw, float *db, float *partial, int T, int D, bool defer_reduce = false);
size_t twist_norm_partial_floats(int T, int D);
// One deferred column reduction: out[c] = alpha * sum over the T/16-row chunks k of partial[k * stride + c], c < n.
struct ColReduce {
  const float *partial;
  float *out;
  int64_t stride;
  int n;
  float alpha;
};
twist_status twist_col_reduce_batch(twist_ctx *ctx, const ColReduce *items, int n_items, int T);

// column sums: out[n] = alpha * sum_t src[t, n] (fp32, overwritten); partial scratch >= colsum_partial_floats.
// With defer_reduce only the per-chunk sums are written (stride Ncols); the caller reduces them later in a batch.
twist_status twist_colsum(twist_ctx *ctx, int bf16, const void *src, int64_t ld, float alpha, float *out, float *partial, int T, int Ncols,
                          bool defer_reduce = false);
size_t twist_colsum_partial_floats(int T, int Ncols);

// cos/sin table [N, dh/2, 2] (computed in fp64), then in-place rotation of the q and k heads of a fused qkv buffer
twist_status twist_rope_table(twist_ctx *ctx, float *tab, int N, int dh, float theta);
twist_status twist_rope_apply(twist_ctx *ctx, int bf16, void *qkv, const float *tab, int B, int N, int Hs, int dh, float sign);

// act: a = f(u) (gu = [T,F]) or a = silu(g) * u (gu = [T,2F], gate first).
// keep (may be null; device, one entry per FFN block of `unit` neurons): blocks with keep[b] < 0 are masked (Masked TwIST,
// Section 4.1): their activations are written as zero and, in the backward kernel, da is taken as zero there.
twist_status twist_act_fwd(twist_ctx *ctx, int bf16, int act, const void *gu, void *a, int T, int F, const int32_t *keep = nullptr, int unit = 1);
twist_status twist_act_bwd(twist_ctx *ctx, int bf16, int act, const void *gu, const void *da, void *dgu, int T, int F, const int32_t *keep = nullptr,
                           int unit = 1);

// logits [T,V] -> in place dlogits = (softmax - onehot)/T; row losses to rowloss[T]; then loss = mean
twist_status twist_ce_fwd_bwd(twist_ctx *ctx, int bf16, void *logits, int64_t ld, const int32_t *targets, float *rowloss, float *loss, int T, int V);
// dx = 2 (x - y)/n ; dxb = activation-type copy; loss = mean squared error
twist_status twist_mse_fwd_bwd(twist_ctx *ctx, int bf16, const float *x, const void *y, float *dx, void *dxb, float *partial, float *loss, int64_t n);

twist_status twist_sgd(twist_ctx *ctx, int bf16, void *params, float *master, const float *grads, int64_t n, float lr);
twist_status twist_adamw(twist_ctx *ctx, int bf16, void *params, float *master, const float *grads, float *m, float *v, int64_t n, int64_t n_decay,
                         float lr, float b1, float b2, float eps, float wd, int64_t step);
