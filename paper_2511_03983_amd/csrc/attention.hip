// Causal multi-head attention (Appendix A.1) on a fused q|k|v buffer, forward and backward.
// This file holds the plain kernels: one wave per query (or key) row, fp32 arithmetic, any d_head <= 256.
// They serve fp32 models and shapes the tiled kernels do not cover.
#include "nn.h"

namespace {

template <int BF> struct El;
template <> struct El<0> {
  static __device__ __forceinline__ float ld(const void *p, int64_t i) { return static_cast<const float *>(p)[i]; }
  static __device__ __forceinline__ void st(void *p, int64_t i, float v) { static_cast<float *>(p)[i] = v; }
};
template <> struct El<1> {
  static __device__ __forceinline__ float ld(const void *p, int64_t i) {
    return __uint_as_float((uint32_t) static_cast<const uint16_t *>(p)[i] << 16);
  }
  static __device__ __forceinline__ void st(void *p, int64_t i, float v) {
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) u = (u >> 16) | 0x40u;
    else { u += 0x7fffu + ((u >> 16) & 1u); u >>= 16; }
    static_cast<uint16_t *>(p)[i] = (uint16_t)u;
  }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

constexpr int kE = 4;  // d_head <= 64 * kE

struct RowId { int b, h, i; bool ok; };
__device__ __forceinline__ RowId row_id(int B, int N, int Hs) {
  const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  RowId r;
  r.ok = w < (int64_t)B * Hs * N;
  r.i = (int)(w % N);
  r.h = (int)((w / N) % Hs);
  r.b = (int)(w / ((int64_t)N * Hs));
  return r;
}

template <int BF>
__global__ __launch_bounds__(256) void attn_fwd_plain(const void *qkv, void *o, float *lse, int B, int N, int Hs, int dh, float scale, const int32_t *keep) {
  const RowId r = row_id(B, N, Hs);
  if (!r.ok) return;
  const int lane = threadIdx.x & 63;
  const int64_t HD = (int64_t)Hs * dh, ld = 3 * HD;
  const int64_t qoff = ((int64_t)r.b * N + r.i) * ld + (int64_t)r.h * dh;
  float q[kE], acc[kE];
#pragma unroll
  for (int t = 0; t < kE; ++t) { int e = lane + 64 * t; q[t] = e < dh ? El<BF>::ld(qkv, qoff + e) : 0.f; acc[t] = 0.f; }
  float m = -INFINITY, l = 0.f;
  const int64_t ooff = ((int64_t)r.b * N + r.i) * HD + (int64_t)r.h * dh;
  if (keep && keep[r.h] < 0) {  // masked head (Masked TwIST, Section 4.1): its output is zero
#pragma unroll
    for (int t = 0; t < kE; ++t) { int e = lane + 64 * t; if (e < dh) El<BF>::st(o, ooff + e, 0.f); }
    if (lane == 0) lse[((int64_t)r.b * Hs + r.h) * N + r.i] = 0.f;
    return;
  }
  for (int j = 0; j <= r.i; ++j) {
    const int64_t koff = ((int64_t)r.b * N + j) * ld + HD + (int64_t)r.h * dh;
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < kE; ++t) { int e = lane + 64 * t; if (e < dh) s += q[t] * El<BF>::ld(qkv, koff + e); }
    s = wave_sum(s) * scale;
    const float mn = fmaxf(m, s);
    const float c = __expf(m - mn), p = __expf(s - mn);
    l = l * c + p;
#pragma unroll
    for (int t = 0; t < kE; ++t) { int e = lane + 64 * t; if (e < dh) acc[t] = acc[t] * c + p * El<BF>::ld(qkv, koff + HD + e); }
    m = mn;
  }
#pragma unroll
  for (int t = 0; t < kE; ++t) { int e = lane + 64 * t; if (e < dh) El<BF>::st(o, ooff + e, acc[t] / l); }
  if (lane == 0) lse[((int64_t)r.b * Hs + r.h) * N + r.i] = m + logf(l);
}

// The softmax backward needs delta_i = sum_j p_ij dp_ij.  It equals do_i . o_i only for the UNROUNDED output, and
// ds = p (dp - delta) cancels almost completely when attention is close to uniform, so delta is recomputed
// here from the same p and dp the gradient uses (a first pass over the keys) instead of from the stored o.
template <int BF>
__global__ __launch_bounds__(256) void attn_bwd_dq_plain(const void *qkv, const void *dout, const float *lse, float *delta, void *dqkv, int B,
                                                         int N, int Hs, int dh, float scale, const int32_t *keep) {
  const RowId r = row_id(B, N, Hs);
  if (!r.ok) return;
  const int lane = threadIdx.x & 63;
  const int64_t HD = (int64_t)Hs * dh, ld = 3 * HD;
  const int64_t qoff = ((int64_t)r.b * N + r.i) * ld + (int64_t)r.h * dh;
  const int64_t doff = ((int64_t)r.b * N + r.i) * HD + (int64_t)r.h * dh;
  const float L = lse[((int64_t)r.b * Hs + r.h) * N + r.i];
  float q[kE], g[kE], acc[kE];
#pragma unroll
  for (int t = 0; t < kE; ++t) {
    int e = lane + 64 * t;
    q[t] = e < dh ? El<BF>::ld(qkv, qoff + e) : 0.f;
    g[t] = e < dh ? El<BF>::ld(dout, doff + e) : 0.f;
    acc[t] = 0.f;
  }
  float Dl = 0.f;
  const int n_keys = (keep && keep[r.h] < 0) ? 0 : r.i + 1;  // masked head: zero gradient, no key is visited
  for (int j = 0; j < n_keys; ++j) {
    const int64_t koff = ((int64_t)r.b * N + j) * ld + HD + (int64_t)r.h * dh;
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int t = 0; t < kE; ++t) {
      int e = lane + 64 * t;
      if (e < dh) { s += q[t] * El<BF>::ld(qkv, koff + e); dp += g[t] * El<BF>::ld(qkv, koff + HD + e); }
    }
    Dl += __expf(wave_sum(s) * scale - L) * wave_sum(dp);
  }
  if (lane == 0) delta[((int64_t)r.b * Hs + r.h) * N + r.i] = Dl;
  for (int j = 0; j < n_keys; ++j) {
    const int64_t koff = ((int64_t)r.b * N + j) * ld + HD + (int64_t)r.h * dh;
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int t = 0; t < kE; ++t) {
      int e = lane + 64 * t;
      if (e < dh) { s += q[t] * El<BF>::ld(qkv, koff + e); dp += g[t] * El<BF>::ld(qkv, koff + HD + e); }
    }
    s = wave_sum(s) * scale;
    dp = wave_sum(dp);
    const float ds = __expf(s - L) * (dp - Dl) * scale;
#pragma unroll
    for (int t = 0; t < kE; ++t) { int e = lane + 64 * t; if (e < dh) acc[t] += ds * El<BF>::ld(qkv, koff + e); }
  }
#pragma unroll
  for (int t = 0; t < kE; ++t) { int e = lane + 64 * t; if (e < dh) El<BF>::st(dqkv, qoff + e, acc[t]); }
}

template <int BF>
__global__ __launch_bounds__(256) void attn_bwd_dkv_plain(const void *qkv, const void *dout, const float *lse, const float *delta, void *dqkv, int B,
                                                          int N, int Hs, int dh, float scale, const int32_t *keep) {
  const RowId r = row_id(B, N, Hs);  // r.i is the key/value row j
  if (!r.ok) return;
  const int lane = threadIdx.x & 63;
  const int64_t HD = (int64_t)Hs * dh, ld = 3 * HD;
  const int64_t koff = ((int64_t)r.b * N + r.i) * ld + HD + (int64_t)r.h * dh;
  float k[kE], v[kE], dk[kE], dv[kE];
#pragma unroll
  for (int t = 0; t < kE; ++t) {
    int e = lane + 64 * t;
    k[t] = e < dh ? El<BF>::ld(qkv, koff + e) : 0.f;
    v[t] = e < dh ? El<BF>::ld(qkv, koff + HD + e) : 0.f;
    dk[t] = dv[t] = 0.f;
  }
  const int n_q = (keep && keep[r.h] < 0) ? 0 : N;  // masked head: zero gradients
  for (int i = r.i; i < n_q; ++i) {
    const int64_t qoff = ((int64_t)r.b * N + i) * ld + (int64_t)r.h * dh;
    const int64_t doff = ((int64_t)r.b * N + i) * HD + (int64_t)r.h * dh;
    float qv[kE], gv[kE];
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int t = 0; t < kE; ++t) {
      int e = lane + 64 * t;
      qv[t] = e < dh ? El<BF>::ld(qkv, qoff + e) : 0.f;
      gv[t] = e < dh ? El<BF>::ld(dout, doff + e) : 0.f;
      s += qv[t] * k[t];
      dp += gv[t] * v[t];
    }
    s = wave_sum(s) * scale;
    dp = wave_sum(dp);
    const int64_t si = ((int64_t)r.b * Hs + r.h) * N + i;
    const float p = __expf(s - lse[si]);
    const float ds = p * (dp - delta[si]) * scale;
#pragma unroll
    for (int t = 0; t < kE; ++t) { dk[t] += ds * qv[t]; dv[t] += p * gv[t]; }
  }
#pragma unroll
  for (int t = 0; t < kE; ++t) {
    int e = lane + 64 * t;
    if (e < dh) { El<BF>::st(dqkv, koff + e, dk[t]); El<BF>::st(dqkv, koff + HD + e, dv[t]); }
  }
}

}  // namespace

twist_status twist_attention_fwd_mfma(twist_ctx *ctx, const void *qkv, void *o, float *o32, float *lse, int B, int N, int Hs, int dh, const int32_t *keep,
                                      bool *done);
twist_status twist_attention_bwd_mfma(twist_ctx *ctx, const void *qkv, const float *o32, const void *dout, const float *lse, float *delta,
                                      void *dqkv, int B, int N, int Hs, int dh, const float *rope_tab, const int32_t *keep, bool *done, bool *rope_done);

twist_status twist_attention_fwd(twist_ctx *ctx, int bf16, const void *qkv, void *o, float *o32, float *lse, int B, int N, int Hs, int dh,
                                 const int32_t *keep) {
  if (dh > 64 * kE) TW_FAIL(ctx, TWIST_ESHAPE, "attention: d_head=%d above %d is not supported", dh, 64 * kE);
  const float scale = 1.0f / sqrtf((float)dh);
  if (bf16) {
    bool done = false;
    TW_TRY(twist_attention_fwd_mfma(ctx, qkv, o, o32, lse, B, N, Hs, dh, keep, &done));
    if (done) return TWIST_OK;
  }
  dim3 grid((unsigned)(((int64_t)B * Hs * N + 3) / 4)), block(256);
  if (bf16) hipLaunchKernelGGL(attn_fwd_plain<1>, grid, block, 0, ctx->stream, qkv, o, lse, B, N, Hs, dh, scale, keep);
  else hipLaunchKernelGGL(attn_fwd_plain<0>, grid, block, 0, ctx->stream, qkv, o, lse, B, N, Hs, dh, scale, keep);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_attention_bwd(twist_ctx *ctx, int bf16, const void *qkv, const float *o32, const void *dout, const float *lse, float *delta,
                                 void *dqkv, int B, int N, int Hs, int dh, const float *rope_tab, const int32_t *keep) {
  if (dh > 64 * kE) TW_FAIL(ctx, TWIST_ESHAPE, "attention: d_head=%d above %d is not supported", dh, 64 * kE);
  const float scale = 1.0f / sqrtf((float)dh);
  dim3 grid((unsigned)(((int64_t)B * Hs * N + 3) / 4)), block(256);
  if (bf16) {
    bool done = false, rope_done = false;
    TW_TRY(twist_attention_bwd_mfma(ctx, qkv, o32, dout, lse, delta, dqkv, B, N, Hs, dh, rope_tab, keep, &done, &rope_done));
    if (done) return (rope_tab && !rope_done) ? twist_rope_apply(ctx, bf16, dqkv, rope_tab, B, N, Hs, dh, -1.f) : TWIST_OK;
  }
  if (bf16) {
    hipLaunchKernelGGL(attn_bwd_dq_plain<1>, grid, block, 0, ctx->stream, qkv, dout, lse, delta, dqkv, B, N, Hs, dh, scale, keep);
    hipLaunchKernelGGL(attn_bwd_dkv_plain<1>, grid, block, 0, ctx->stream, qkv, dout, lse, delta, dqkv, B, N, Hs, dh, scale, keep);
  } else {
    hipLaunchKernelGGL(attn_bwd_dq_plain<0>, grid, block, 0, ctx->stream, qkv, dout, lse, delta, dqkv, B, N, Hs, dh, scale, keep);
    hipLaunchKernelGGL(attn_bwd_dkv_plain<0>, grid, block, 0, ctx->stream, qkv, dout, lse, delta, dqkv, B, N, Hs, dh, scale, keep);
  }
  TW_HIP(ctx, hipGetLastError());
  return rope_tab ? twist_rope_apply(ctx, bf16, dqkv, rope_tab, B, N, Hs, dh, -1.f) : TWIST_OK;
}

extern "C" twist_status twist_attention_raw(twist_ctx *ctx, const void *qkv, const void *dout, int32_t B, int32_t N, int32_t Hs, void *o, float *o32,
                                            float *lse, float *delta, void *dqkv, const int32_t *keep, float *rope_tab) {
  if (!ctx || !qkv || !o || !o32 || !lse) TW_FAIL(ctx, TWIST_EINVAL, "twist_attention_raw: null argument");
  if (B < 1 || N < 1 || Hs < 1) TW_FAIL(ctx, TWIST_ESHAPE, "twist_attention_raw: empty shape");
  const int bf = ctx->d.dtype == TWIST_BF16;
  TW_TRY(twist_attention_fwd(ctx, bf, qkv, o, o32, lse, B, N, Hs, ctx->d.d_head, keep));
  if (dout) {
    if (!delta || !dqkv) TW_FAIL(ctx, TWIST_EINVAL, "twist_attention_raw: backward needs delta and dqkv");
    if (rope_tab) {
      if (ctx->d.d_head % 2) TW_FAIL(ctx, TWIST_ESHAPE, "twist_attention_raw: rotary positions need an even d_head");
      TW_TRY(twist_rope_table(ctx, rope_tab, N, ctx->d.d_head, ctx->d.rope_theta));
    }
    TW_TRY(twist_attention_bwd(ctx, bf, qkv, o32, dout, lse, delta, dqkv, B, N, Hs, ctx->d.d_head, rope_tab, keep));
  }
  return TWIST_OK;
}
