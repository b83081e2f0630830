// Memory-bound kernels of the subnet training path: embedding, norms (Appendix A.1), rotary positions,
// activations, losses, reductions for bias / gain gradients, and the local optimizer steps.
// Activations and weights are fp32 or bf16 (template flag BF); all arithmetic is fp32.
#include "nn.h"

namespace {

constexpr int kT = 256;

template <int BF> struct El;
template <> struct El<0> {
  using T = float;
  static __device__ __forceinline__ float ld(const void *p, int64_t i) { return static_cast<const float *>(p)[i]; }
  static __device__ __forceinline__ void st(void *p, int64_t i, float v) { static_cast<float *>(p)[i] = v; }
};
template <> struct El<1> {
  using T = uint16_t;
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
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// block-wide sum for kT threads; result valid in every thread
__device__ __forceinline__ float block_sum(float v, float *sh) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}
__device__ __forceinline__ float block_max(float v, float *sh) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}

// ------------------------------------------------------------------------------------------- embedding
template <int BF>
__global__ __launch_bounds__(kT) void embed_fwd_kernel(const int32_t *tok, const void *E, const void *P, float *x, int N, int D, int64_t total) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  int64_t t = i / D;
  int c = (int)(i - t * D);
  float v = El<BF>::ld(E, (int64_t)tok[t] * D + c);
  if (P) v += El<BF>::ld(P, (int64_t)(t % N) * D + c);
  x[i] = v;
}

__global__ __launch_bounds__(kT) void embed_bwd_tok_kernel(const int32_t *tok, const float *dx, float *dE, int D, int64_t total) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  int64_t t = i / D;
  int c = (int)(i - t * D);
  atomicAdd(&dE[(int64_t)tok[t] * D + c], dx[i]);
}

__global__ __launch_bounds__(kT) void embed_bwd_pos_kernel(const float *dx, float *dP, int B, int N, int D) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;  // over N*D
  if (i >= (int64_t)N * D) return;
  float s = 0.f;
  for (int b = 0; b < B; ++b) s += dx[(int64_t)b * N * D + i];
  dP[i] = s;
}

template <int BF>
__global__ __launch_bounds__(kT) void cast_in_kernel(const void *src, float *dst, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i < n) dst[i] = El<BF>::ld(src, i);
}

// ------------------------------------------------------------------------------------------- norms
// one wave per row
template <int BF, int RMS>
__global__ __launch_bounds__(kT) void norm_fwd_kernel(const float *x, const void *w, const void *b, void *y, float *stats, int T, int D, float eps) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= T) return;
  const float *xr = x + (int64_t)row * D;
  float mean = 0.f;
  if (!RMS) {
    float s = 0.f;
    for (int c = lane; c < D; c += 64) s += xr[c];
    mean = wave_sum(s) / D;
  }
  float s2 = 0.f;
  for (int c = lane; c < D; c += 64) { float d = xr[c] - mean; s2 += d * d; }
  const float rstd = 1.0f / sqrtf(wave_sum(s2) / D + eps);
  for (int c = lane; c < D; c += 64) {
    float v = (xr[c] - mean) * rstd * El<BF>::ld(w, c);
    if (b) v += El<BF>::ld(b, c);
    El<BF>::st(y, (int64_t)row * D + c, v);
  }
  if (lane == 0) { stats[2 * row] = mean; stats[2 * row + 1] = rstd; }
}

template <int BF, int RMS>
__global__ __launch_bounds__(kT) void norm_bwd_dx_kernel(const void *dy, const float *x, const void *w, const float *stats, float *dx, int accumulate,
                                                          void *dxb, int T, int D) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= T) return;
  const float mean = stats[2 * row], rstd = stats[2 * row + 1];
  const float *xr = x + (int64_t)row * D;
  float c1 = 0.f, c2 = 0.f;
  for (int c = lane; c < D; c += 64) {
    float dz = El<BF>::ld(dy, (int64_t)row * D + c) * El<BF>::ld(w, c);
    float z = (xr[c] - mean) * rstd;
    c1 += dz;
    c2 += dz * z;
  }
  c1 = RMS ? 0.f : wave_sum(c1) / D;
  c2 = wave_sum(c2) / D;
  for (int c = lane; c < D; c += 64) {
    float dz = El<BF>::ld(dy, (int64_t)row * D + c) * El<BF>::ld(w, c);
    float z = (xr[c] - mean) * rstd;
    float g = rstd * (dz - c1 - z * c2);
    const int64_t i = (int64_t)row * D + c;
    if (accumulate) g += dx[i];
    dx[i] = g;
    if (dxb) El<BF>::st(dxb, i, g);
  }
}

constexpr int kChunkRows = 16;

// partial[chunk][0][c] = sum over the chunk's rows of dy*z ; partial[chunk][1][c] = sum of dy
template <int BF>
__global__ __launch_bounds__(64) void norm_bwd_dw_kernel(const void *dy, const float *x, const float *stats, float *partial, int T, int D) {
  const int c = blockIdx.x * 64 + threadIdx.x;
  const int chunk = blockIdx.y;
  if (c >= D) return;
  const int r0 = chunk * kChunkRows, r1 = min(r0 + kChunkRows, T);
  float sw = 0.f, sb = 0.f;
  for (int r = r0; r < r1; ++r) {
    float g = El<BF>::ld(dy, (int64_t)r * D + c);
    float z = (x[(int64_t)r * D + c] - stats[2 * r]) * stats[2 * r + 1];
    sw += g * z;
    sb += g;
  }
  partial[((int64_t)chunk * 2) * D + c] = sw;
  partial[((int64_t)chunk * 2 + 1) * D + c] = sb;
}

// Fused norm backward for rows of NV * 256 elements: one pass over dy and x yields dx (+= when accumulating), its
// activation-type copy, and this chunk's partial sums for the gain / bias gradients.  A wave owns a row at a time and
// a lane the same 4 NV columns of every row (vector v = lane + 64 k holds columns 4v .. 4v+3), so the parameter sums
// stay in registers across the chunk's rows; the four waves' sums are combined through LDS.
template <int BF, int RMS, int NV>
__global__ __launch_bounds__(kT) void norm_bwd_fused_kernel(const void *dy, const float *x, const void *w, const float *stats, float *dx, int accumulate,
                                                             void *dxb, float *partial, int T) {
  constexpr int D = NV * 256;
  typedef float f4 __attribute__((ext_vector_type(4)));
  typedef uint32_t u2 __attribute__((ext_vector_type(2)));
  __shared__ float red[(RMS ? 1 : 2) * 4 * D];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r0 = blockIdx.x * kChunkRows, r1 = min(r0 + kChunkRows, T);
  auto load4 = [](const void *p, int64_t vec) -> f4 {
    if (BF) {
      const u2 u = static_cast<const u2 *>(p)[vec];
      return f4{__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u)};
    }
    return static_cast<const f4 *>(p)[vec];
  };
  f4 wv[NV], aw[NV], ab[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    wv[k] = load4(w, lane + 64 * k);
    aw[k] = f4{0.f, 0.f, 0.f, 0.f};
    ab[k] = f4{0.f, 0.f, 0.f, 0.f};
  }
  for (int r = r0 + wave; r < r1; r += 4) {
    const float mean = stats[2 * r], rstd = stats[2 * r + 1];
    const int64_t rv = (int64_t)r * (D / 4);
    f4 g[NV], z[NV];
    float c1 = 0.f, c2 = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      g[k] = load4(dy, rv + lane + 64 * k);
      z[k] = (reinterpret_cast<const f4 *>(x)[rv + lane + 64 * k] - mean) * rstd;
    }
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      aw[k] += g[k] * z[k];
      if (!RMS) ab[k] += g[k];
      g[k] *= wv[k];  // dz
#pragma unroll
      for (int e = 0; e < 4; ++e) { c1 += g[k][e]; c2 += g[k][e] * z[k][e]; }
    }
    c1 = RMS ? 0.f : wave_sum(c1) / D;
    c2 = wave_sum(c2) / D;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      f4 o = rstd * (g[k] - c1 - z[k] * c2);
      f4 *dp = reinterpret_cast<f4 *>(dx) + rv + lane + 64 * k;
      if (accumulate) o += *dp;
      *dp = o;
      if (dxb) {
        if (BF) {
          typedef __bf16 b2 __attribute__((ext_vector_type(2)));
          typedef float f2 __attribute__((ext_vector_type(2)));
          const f2 lo = {o[0], o[1]}, hi = {o[2], o[3]};
          const u2 pk = {__builtin_bit_cast(uint32_t, __builtin_convertvector(lo, b2)), __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, b2))};
          static_cast<u2 *>(dxb)[rv + lane + 64 * k] = pk;
        } else {
          static_cast<f4 *>(dxb)[rv + lane + 64 * k] = o;
        }
      }
    }
  }
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    *reinterpret_cast<f4 *>(&red[wave * D + 4 * (lane + 64 * k)]) = aw[k];
    if (!RMS) *reinterpret_cast<f4 *>(&red[(4 + wave) * D + 4 * (lane + 64 * k)]) = ab[k];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < D; c += kT) {
    partial[((int64_t)blockIdx.x * 2) * D + c] = red[c] + red[D + c] + red[2 * D + c] + red[3 * D + c];
    if (!RMS) partial[((int64_t)blockIdx.x * 2 + 1) * D + c] = red[4 * D + c] + red[5 * D + c] + red[6 * D + c] + red[7 * D + c];
  }
}

// out[c] = alpha * sum_k partial[k*stride + c].  A workgroup owns 16 columns; its 256 threads are 16 chunk slices x
// 16 columns, each summing every sixteenth chunk in ascending order; the slices are then added in order.
__global__ __launch_bounds__(kT) void reduce_partial_kernel(const float *partial, int64_t stride, int n_chunks, float alpha, float *out, int n) {
  __shared__ float sh[16][16];
  const int col = threadIdx.x & 15, slice = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + col;
  float s = 0.f;
  if (c < n)
    for (int k = slice; k < n_chunks; k += 16) s += partial[(int64_t)k * stride + c];
  sh[slice][col] = s;
  __syncthreads();
  if (slice == 0 && c < n) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += sh[i][col];
    out[c] = alpha * t;
  }
}

// the same reduction for a batch of buffers in one launch: blockIdx.y = item
constexpr int kReduceBatch = 64;
struct ColReduceArgs {
  ColReduce item[kReduceBatch];
};
__global__ __launch_bounds__(kT) void reduce_partial_batch_kernel(const ColReduceArgs a, int n_chunks) {
  __shared__ float sh[16][16];
  const ColReduce it = a.item[blockIdx.y];
  const int col = threadIdx.x & 15, slice = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + col;
  if (blockIdx.x * 16 >= it.n) return;  // uniform over the workgroup
  float s = 0.f;
  if (c < it.n)
    for (int k = slice; k < n_chunks; k += 16) s += it.partial[(int64_t)k * it.stride + c];
  sh[slice][col] = s;
  __syncthreads();
  if (slice == 0 && c < it.n) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += sh[i][col];
    it.out[c] = it.alpha * t;
  }
}

template <int BF>
__global__ __launch_bounds__(64) void colsum_kernel(const void *src, int64_t ld, float *partial, int T, int n) {
  const int c = blockIdx.x * 64 + threadIdx.x;
  const int chunk = blockIdx.y;
  if (c >= n) return;
  const int r0 = chunk * kChunkRows, r1 = min(r0 + kChunkRows, T);
  float s = 0.f;
  for (int r = r0; r < r1; ++r) s += El<BF>::ld(src, (int64_t)r * ld + c);
  partial[(int64_t)chunk * n + c] = s;
}

// ------------------------------------------------------------------------------------------- rotary
__global__ __launch_bounds__(kT) void rope_table_kernel(float *tab, int N, int half, int dh, float theta) {
  int i = blockIdx.x * kT + threadIdx.x;
  if (i >= N * half) return;
  int pos = i / half, f = i - pos * half;
  double ang = (double)pos * pow((double)theta, -2.0 * (double)f / (double)dh);
  tab[2 * i] = (float)cos(ang);
  tab[2 * i + 1] = (float)sin(ang);
}

// q and k heads of a fused [T, 3*Hs*dh] buffer, in place; pair (i, i + dh/2)
template <int BF>
__global__ __launch_bounds__(kT) void rope_kernel(void *qkv, const float *tab, int N, int Hs, int dh, float sign, int64_t total) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;  // over T * 2Hs * half
  if (i >= total) return;
  const int half = dh / 2;
  int f = (int)(i % half);
  int64_t r = i / half;
  int head = (int)(r % (2 * Hs));
  int64_t t = r / (2 * Hs);
  int pos = (int)(t % N);
  const float c = tab[2 * (pos * half + f)], s = sign * tab[2 * (pos * half + f) + 1];
  const int64_t base = t * (3 * (int64_t)Hs * dh) + (int64_t)head * dh + f;
  float a = El<BF>::ld(qkv, base), b = El<BF>::ld(qkv, base + half);
  El<BF>::st(qkv, base, a * c - b * s);
  El<BF>::st(qkv, base + half, b * c + a * s);
}

// ------------------------------------------------------------------------------------------- activations
__device__ __forceinline__ float gelu_tanh(float u) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  return 0.5f * u * (1.f + tanhf(k0 * (u + k1 * u * u * u)));
}
__device__ __forceinline__ float gelu_tanh_grad(float u) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  float t = tanhf(k0 * (u + k1 * u * u * u));
  return 0.5f * (1.f + t) + 0.5f * u * (1.f - t * t) * k0 * (1.f + 3.f * k1 * u * u);
}
__device__ __forceinline__ float sigmoidf(float x) { return 1.f / (1.f + __expf(-x)); }

// `keep` (may be null): the Masked-TwIST neuron mask of Section 4.1, y = M * f(x).  keep[b] < 0 marks FFN block b (of
// `unit` neurons) as masked: its activations, and in the backward kernels its pre-activation gradients, are zero.
template <int BF>
__global__ __launch_bounds__(kT) void act_fwd_kernel(int act, const void *gu, void *a, int F, int64_t total, const int32_t *keep, int unit) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  const int64_t t = i / F;
  const int c = (int)(i - t * F);
  float o;
  if (act == TWIST_ACT_SWIGLU) {
    float g = El<BF>::ld(gu, t * 2 * F + c), u = El<BF>::ld(gu, t * 2 * F + F + c);
    o = g * sigmoidf(g) * u;
  } else {
    float u = El<BF>::ld(gu, i);
    o = act == TWIST_ACT_RELU ? fmaxf(u, 0.f) : gelu_tanh(u);
  }
  if (keep && keep[c / unit] < 0) o = 0.f;
  El<BF>::st(a, i, o);
}

template <int BF>
__global__ __launch_bounds__(kT) void act_bwd_kernel(int act, const void *gu, const void *da, void *dgu, int F, int64_t total, const int32_t *keep, int unit) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  const int64_t t = i / F;
  const int c = (int)(i - t * F);
  const float d = (keep && keep[c / unit] < 0) ? 0.f : El<BF>::ld(da, i);
  if (act == TWIST_ACT_SWIGLU) {
    float g = El<BF>::ld(gu, t * 2 * F + c), u = El<BF>::ld(gu, t * 2 * F + F + c);
    float sg = sigmoidf(g);
    El<BF>::st(dgu, t * 2 * F + F + c, d * g * sg);
    El<BF>::st(dgu, t * 2 * F + c, d * u * (sg + g * sg * (1.f - sg)));
  } else {
    float u = El<BF>::ld(gu, i);
    El<BF>::st(dgu, i, d * (act == TWIST_ACT_RELU ? (u > 0.f ? 1.f : 0.f) : gelu_tanh_grad(u)));
  }
}

// ------------------------------------------------------------------------------------------- losses
// one workgroup per row: logsumexp, row loss, then dlogits in place
template <int BF>
__global__ __launch_bounds__(kT) void ce_kernel(void *logits, int64_t ld, const int32_t *targets, float *rowloss, int V, float inv_T) {
  __shared__ float sh[4];
  const int64_t base = (int64_t)blockIdx.x * ld;
  float m = -INFINITY;
  for (int c = threadIdx.x; c < V; c += kT) m = fmaxf(m, El<BF>::ld(logits, base + c));
  m = block_max(m, sh);
  float s = 0.f;
  for (int c = threadIdx.x; c < V; c += kT) s += __expf(El<BF>::ld(logits, base + c) - m);
  s = block_sum(s, sh);
  const float lse = m + logf(s);
  const int tgt = targets[blockIdx.x];
  if (threadIdx.x == 0) rowloss[blockIdx.x] = lse - El<BF>::ld(logits, base + tgt);
  __syncthreads();
  for (int c = threadIdx.x; c < V; c += kT) {
    float p = __expf(El<BF>::ld(logits, base + c) - lse);
    El<BF>::st(logits, base + c, (p - (c == tgt ? 1.f : 0.f)) * inv_T);
  }
  // columns between V and the padded row stride are read (times zero weights) by the next projection
  for (int c = V + threadIdx.x; c < ld; c += kT) El<BF>::st(logits, base + c, 0.f);
}

__global__ __launch_bounds__(kT) void mean_kernel(const float *v, int64_t n, float scale, float *out) {
  __shared__ float sh[4];
  float s = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += kT) s += v[i];
  s = block_sum(s, sh);
  if (threadIdx.x == 0) *out = s * scale;
}

template <int BF>
__global__ __launch_bounds__(kT) void mse_kernel(const float *x, const void *y, float *dx, void *dxb, float *partial, int64_t n, float two_over_n) {
  __shared__ float sh[4];
  float s = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += (int64_t)gridDim.x * kT) {
    float d = x[i] - El<BF>::ld(y, i);
    s += d * d;
    float g = d * two_over_n;
    dx[i] = g;
    El<BF>::st(dxb, i, g);
  }
  s = block_sum(s, sh);
  if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

// ------------------------------------------------------------------------------------------- optimizers
template <int BF>
__global__ __launch_bounds__(kT) void sgd_kernel(void *params, float *master, const float *grads, int64_t n, float lr) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= n) return;
  if (BF) {
    float w = master[i] - lr * grads[i];
    master[i] = w;
    El<BF>::st(params, i, w);
  } else {
    static_cast<float *>(params)[i] -= lr * grads[i];
  }
}

// `first`: the moments count as zero and are not read (a subnet's first step after extraction).
template <int BF>
__global__ __launch_bounds__(kT) void adamw_kernel(void *params, float *master, const float *grads, float *m, float *v, int64_t n, int64_t n_decay,
                                                    float lr, float b1, float b2, float eps, float wd, float inv_bc1, float inv_bc2, int first) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= n) return;
  const float g = grads[i];
  const float m0 = first ? 0.f : m[i], v0 = first ? 0.f : v[i];
  const float mi = b1 * m0 + (1.f - b1) * g;
  const float vi = b2 * v0 + (1.f - b2) * g * g;
  m[i] = mi;
  v[i] = vi;
  float w = BF ? master[i] : static_cast<float *>(params)[i];
  const float decay = i < n_decay ? wd : 0.f;
  w -= lr * ((mi * inv_bc1) / (sqrtf(vi * inv_bc2) + eps) + decay * w);
  if (BF) { master[i] = w; El<BF>::st(params, i, w); }
  else static_cast<float *>(params)[i] = w;
}

__global__ __launch_bounds__(kT) void zero_f32_kernel(float *p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

// ------------------------------------------------------------------------------------------- 16-byte paths (bf16)
// Eight bf16 values per thread and access, used when rows are multiples of 8 elements and bases 16-byte aligned.
typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
typedef float f32x4v __attribute__((ext_vector_type(4)));
struct F8 { float v[8]; };
__device__ __forceinline__ F8 unpack8(const u32x4v &u) {
  F8 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) { r.v[2 * i] = __uint_as_float(u[i] << 16); r.v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u); }
  return r;
}
__device__ __forceinline__ u32x4v pack8(const F8 &f) {
  typedef __bf16 b2 __attribute__((ext_vector_type(2)));
  typedef float f2 __attribute__((ext_vector_type(2)));
  u32x4v u;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f2 p = {f.v[2 * i], f.v[2 * i + 1]};
    u[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, b2));  // round to nearest even
  }
  return u;
}

// Cross-entropy of a bf16 row of at most NV * 2048 logits held in registers: one read of the row, one write of its
// gradient (the general kernel above walks the row three times with 2-byte accesses).  ld8 = row stride / 8; columns
// between V and the stride are padding and get zeros.
template <int NV>
__global__ __launch_bounds__(kT) void ce_vec_kernel(u32x4v *logits, int64_t ld8, const int32_t *targets, float *rowloss, int V, float inv_T) {
  __shared__ float sh[4];
  u32x4v *row = logits + (int64_t)blockIdx.x * ld8;
  F8 x[NV];
  float m = -INFINITY;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int idx = k * kT + threadIdx.x;
    if (idx < ld8) {
      x[k] = unpack8(row[idx]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (idx * 8 + e >= V) x[k].v[e] = -INFINITY;
        m = fmaxf(m, x[k].v[e]);
      }
    }
  }
  m = block_max(m, sh);
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < NV; ++k)
    if (k * kT + (int)threadIdx.x < ld8) {
#pragma unroll
      for (int e = 0; e < 8; ++e) s += __expf(x[k].v[e] - m);
    }
  s = block_sum(s, sh);
  const float lse = m + logf(s);
  const int tgt = targets[blockIdx.x];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int idx = k * kT + threadIdx.x;
    if (idx < ld8) {
      F8 g;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int c = idx * 8 + e;
        if (c == tgt) rowloss[blockIdx.x] = lse - x[k].v[e];
        g.v[e] = c < V ? (__expf(x[k].v[e] - lse) - (c == tgt ? 1.f : 0.f)) * inv_T : 0.f;
      }
      row[idx] = pack8(g);
    }
  }
}

// The same for rows of any length (row stride a multiple of 8): one vectorised pass keeps a running maximum and a
// sum of exponentials relative to it, a second pass re-reads the row (it is still in the L2) and writes the gradient.
__global__ __launch_bounds__(kT) void ce_vec_long_kernel(u32x4v *logits, int64_t ld8, const int32_t *targets, float *rowloss, int V, float inv_T) {
  __shared__ float sh[4];
  u32x4v *row = logits + (int64_t)blockIdx.x * ld8;
  float m = -INFINITY, s = 0.f;
  for (int idx = threadIdx.x; idx < ld8; idx += kT) {
    const F8 x = unpack8(row[idx]);
    float mx = m;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (idx * 8 + e < V) mx = fmaxf(mx, x.v[e]);
    if (mx == -INFINITY) continue;  // nothing but padding so far
    float t = s * __expf(m - mx);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (idx * 8 + e < V) t += __expf(x.v[e] - mx);
    m = mx;
    s = t;
  }
  const float M = block_max(m, sh);
  s = block_sum(m == -INFINITY ? 0.f : s * __expf(m - M), sh);
  const float lse = M + logf(s);
  const int tgt = targets[blockIdx.x];
  for (int idx = threadIdx.x; idx < ld8; idx += kT) {
    const F8 x = unpack8(row[idx]);
    F8 g;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = idx * 8 + e;
      if (c == tgt) rowloss[blockIdx.x] = lse - x.v[e];
      g.v[e] = c < V ? (__expf(x.v[e] - lse) - (c == tgt ? 1.f : 0.f)) * inv_T : 0.f;
    }
    row[idx] = pack8(g);
  }
}

// a = silu(g) * u on [T, 2F] (gate | up) -> [T, F]; i8 runs over T * F/8
// multiplies the 8 values of columns col0 .. col0 + 7 by the block mask (see act_fwd_kernel)
__device__ __forceinline__ void mask8(F8 &x, const int32_t *keep, int unit, int col0) {
#pragma unroll
  for (int e = 0; e < 8; ++e)
    if (keep[(col0 + e) / unit] < 0) x.v[e] = 0.f;
}

__global__ __launch_bounds__(kT) void swiglu_fwd_vec_kernel(const u32x4v *gu, u32x4v *a, int F8n, int64_t total, const int32_t *keep, int unit) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  const int64_t t = i / F8n;
  const int c = (int)(i - t * F8n);
  const F8 g = unpack8(gu[t * 2 * F8n + c]), u = unpack8(gu[t * 2 * F8n + F8n + c]);
  F8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o.v[e] = g.v[e] * sigmoidf(g.v[e]) * u.v[e];
  if (keep) mask8(o, keep, unit, 8 * c);
  a[i] = pack8(o);
}

// ungated activations (GELU, ReLU), eight values per thread
// F8n = F / 8 (a row's 8-column groups) where a mask is given, so that a thread knows its columns
__global__ __launch_bounds__(kT) void act_fwd_vec_kernel(int act, const u32x4v *u, u32x4v *a, int64_t total, const int32_t *keep, int unit, int F8n) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  const F8 x = unpack8(u[i]);
  F8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o.v[e] = act == TWIST_ACT_RELU ? fmaxf(x.v[e], 0.f) : gelu_tanh(x.v[e]);
  if (keep) mask8(o, keep, unit, 8 * (int)(i % F8n));
  a[i] = pack8(o);
}

__global__ __launch_bounds__(kT) void act_bwd_vec_kernel(int act, const u32x4v *u, const u32x4v *da, u32x4v *du, int64_t total, const int32_t *keep, int unit,
                                                          int F8n) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  const F8 x = unpack8(u[i]);
  F8 d = unpack8(da[i]);
  if (keep) mask8(d, keep, unit, 8 * (int)(i % F8n));
  F8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o.v[e] = d.v[e] * (act == TWIST_ACT_RELU ? (x.v[e] > 0.f ? 1.f : 0.f) : gelu_tanh_grad(x.v[e]));
  du[i] = pack8(o);
}

__global__ __launch_bounds__(kT) void swiglu_bwd_vec_kernel(const u32x4v *gu, const u32x4v *da, u32x4v *dgu, int F8n, int64_t total, const int32_t *keep,
                                                             int unit) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  const int64_t t = i / F8n;
  const int c = (int)(i - t * F8n);
  const F8 g = unpack8(gu[t * 2 * F8n + c]), u = unpack8(gu[t * 2 * F8n + F8n + c]);
  F8 d = unpack8(da[i]);
  if (keep) mask8(d, keep, unit, 8 * c);
  F8 dg, du;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float sg = sigmoidf(g.v[e]);
    du.v[e] = d.v[e] * g.v[e] * sg;
    dg.v[e] = d.v[e] * u.v[e] * (sg + g.v[e] * sg * (1.f - sg));
  }
  dgu[t * 2 * F8n + c] = pack8(dg);
  dgu[t * 2 * F8n + F8n + c] = pack8(du);
}

// rotation of the q and k heads of a fused [T, 3 Hs dh] buffer; i runs over T * 2Hs * (dh/16): 8 pairs per thread
__global__ __launch_bounds__(kT) void rope_vec_kernel(u32x4v *qkv, const float *tab, int N, int Hs, int dh, float sign, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  const int half = dh / 2, h8 = half / 8;
  const int f8 = (int)(i % h8);
  const int64_t r = i / h8;
  const int head = (int)(r % (2 * Hs));
  const int64_t t = r / (2 * Hs);
  const int pos = (int)(t % N);
  const int64_t base = (t * (3 * (int64_t)Hs * dh) + (int64_t)head * dh) / 8 + f8;
  const F8 a = unpack8(qkv[base]), b = unpack8(qkv[base + h8]);
  const f32x4v *cs = reinterpret_cast<const f32x4v *>(tab + 2 * ((int64_t)pos * half + 8 * f8));  // (cos, sin) pairs
  F8 oa, ob;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const f32x4v w = cs[e];
    oa.v[2 * e] = a.v[2 * e] * w[0] - b.v[2 * e] * (sign * w[1]);
    ob.v[2 * e] = b.v[2 * e] * w[0] + a.v[2 * e] * (sign * w[1]);
    oa.v[2 * e + 1] = a.v[2 * e + 1] * w[2] - b.v[2 * e + 1] * (sign * w[3]);
    ob.v[2 * e + 1] = b.v[2 * e + 1] * w[2] + a.v[2 * e + 1] * (sign * w[3]);
  }
  qkv[base] = pack8(oa);
  qkv[base + h8] = pack8(ob);
}

// norm forward for bf16 outputs and rows of NV * 256 elements: a wave per row, the row held in registers
template <int RMS, int NV>
__global__ __launch_bounds__(kT) void norm_fwd_vec_kernel(const float *x, const void *w, const void *b, void *y, float *stats, int T, float eps) {
  constexpr int D = NV * 256;
  typedef uint32_t u2 __attribute__((ext_vector_type(2)));
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= T) return;
  const int64_t rv = (int64_t)row * (D / 4);
  auto load4b = [](const void *p, int64_t vec) -> f32x4v {
    const u2 u = static_cast<const u2 *>(p)[vec];
    return f32x4v{__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u)};
  };
  f32x4v xv[NV];
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    xv[k] = reinterpret_cast<const f32x4v *>(x)[rv + lane + 64 * k];
    s += xv[k][0] + xv[k][1] + xv[k][2] + xv[k][3];
  }
  const float mean = RMS ? 0.f : wave_sum(s) / D;
  float s2 = 0.f;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    xv[k] -= mean;
    s2 += xv[k][0] * xv[k][0] + xv[k][1] * xv[k][1] + xv[k][2] * xv[k][2] + xv[k][3] * xv[k][3];
  }
  const float rstd = 1.0f / sqrtf(wave_sum(s2) / D + eps);
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    f32x4v o = xv[k] * rstd * load4b(w, lane + 64 * k);
    if (b) o += load4b(b, lane + 64 * k);
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    const f2 lo = {o[0], o[1]}, hi = {o[2], o[3]};
    const u2 pk = {__builtin_bit_cast(uint32_t, __builtin_convertvector(lo, b2)), __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, b2))};
    static_cast<u2 *>(y)[rv + lane + 64 * k] = pk;
  }
  if (lane == 0) { stats[2 * row] = mean; stats[2 * row + 1] = rstd; }
}

inline dim3 grid1(int64_t n) { return dim3((unsigned)((n + kT - 1) / kT)); }

}  // namespace

#define LAUNCH_BF(kern, bf, grid, block, ...)                                             \
  do {                                                                                    \
    if (bf) hipLaunchKernelGGL((kern<1>), grid, block, 0, ctx->stream, __VA_ARGS__);      \
    else hipLaunchKernelGGL((kern<0>), grid, block, 0, ctx->stream, __VA_ARGS__);         \
    TW_HIP(ctx, hipGetLastError());                                                       \
  } while (0)

#define LAUNCH_BF2(kern, bf, flag, grid, block, ...)                                                  \
  do {                                                                                                \
    if (bf && flag) hipLaunchKernelGGL((kern<1, 1>), grid, block, 0, ctx->stream, __VA_ARGS__);       \
    else if (bf) hipLaunchKernelGGL((kern<1, 0>), grid, block, 0, ctx->stream, __VA_ARGS__);          \
    else if (flag) hipLaunchKernelGGL((kern<0, 1>), grid, block, 0, ctx->stream, __VA_ARGS__);        \
    else hipLaunchKernelGGL((kern<0, 0>), grid, block, 0, ctx->stream, __VA_ARGS__);                  \
    TW_HIP(ctx, hipGetLastError());                                                                   \
  } while (0)

twist_status twist_zero_f32(twist_ctx *ctx, float *p, int64_t n) {
  if (n <= 0) return TWIST_OK;
  hipLaunchKernelGGL(zero_f32_kernel, grid1(n), dim3(kT), 0, ctx->stream, p, n);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_embed_fwd(twist_ctx *ctx, int bf16, const int32_t *tok, const void *E, const void *P, float *x, int B, int N, int D, int) {
  const int64_t total = (int64_t)B * N * D;
  LAUNCH_BF(embed_fwd_kernel, bf16, grid1(total), dim3(kT), tok, E, P, x, N, D, total);
  return TWIST_OK;
}

twist_status twist_embed_bwd(twist_ctx *ctx, const int32_t *tok, const float *dx, float *d_tok, float *d_pos, int B, int N, int D) {
  const int64_t total = (int64_t)B * N * D;
  hipLaunchKernelGGL(embed_bwd_tok_kernel, grid1(total), dim3(kT), 0, ctx->stream, tok, dx, d_tok, D, total);
  TW_HIP(ctx, hipGetLastError());
  if (d_pos) {
    hipLaunchKernelGGL(embed_bwd_pos_kernel, grid1((int64_t)N * D), dim3(kT), 0, ctx->stream, dx, d_pos, B, N, D);
    TW_HIP(ctx, hipGetLastError());
  }
  return TWIST_OK;
}

twist_status twist_cast_in(twist_ctx *ctx, int bf16, const void *src, float *dst, int64_t n) {
  LAUNCH_BF(cast_in_kernel, bf16, grid1(n), dim3(kT), src, dst, n);
  return TWIST_OK;
}

static bool al16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

twist_status twist_norm_fwd(twist_ctx *ctx, int bf16, int rms, const float *x, const void *w, const void *b, void *y, float *stats, int T, int D, float eps) {
  const int nv = D % 256 == 0 ? D / 256 : 0;
  if (bf16 && al16(x) && al16(w) && al16(y) && (!b || al16(b)) && (nv == 1 || nv == 2 || nv == 3 || nv == 4 || nv == 8 || nv == 16)) {
#define TW_NORM_FWD(NV)                                                                                                                          \
  do {                                                                                                                                           \
    if (rms) hipLaunchKernelGGL((norm_fwd_vec_kernel<1, NV>), dim3((T + 3) / 4), dim3(kT), 0, ctx->stream, x, w, b, y, stats, T, eps);           \
    else hipLaunchKernelGGL((norm_fwd_vec_kernel<0, NV>), dim3((T + 3) / 4), dim3(kT), 0, ctx->stream, x, w, b, y, stats, T, eps);              \
  } while (0)
    switch (nv) {
      case 1: TW_NORM_FWD(1); break;
      case 2: TW_NORM_FWD(2); break;
      case 3: TW_NORM_FWD(3); break;
      case 4: TW_NORM_FWD(4); break;
      case 8: TW_NORM_FWD(8); break;
      default: TW_NORM_FWD(16); break;
    }
#undef TW_NORM_FWD
    TW_HIP(ctx, hipGetLastError());
    return TWIST_OK;
  }
  LAUNCH_BF2(norm_fwd_kernel, bf16, rms, dim3((T + 3) / 4), dim3(kT), x, w, b, y, stats, T, D, eps);
  return TWIST_OK;
}

static int n_chunks(int T) { return (T + kChunkRows - 1) / kChunkRows; }
size_t twist_norm_partial_floats(int T, int D) { return (size_t)n_chunks(T) * 2 * D; }
size_t twist_colsum_partial_floats(int T, int n) { return (size_t)n_chunks(T) * n; }

twist_status twist_norm_bwd(twist_ctx *ctx, int bf16, int rms, const void *dy, const float *x, const void *w, const float *stats, float *dx,
                            int accumulate, void *dxb, float *dw, float *db, float *partial, int T, int D, bool defer_reduce) {
  const int nc = n_chunks(T);
  const int nv = D % 256 == 0 ? D / 256 : 0;
  const bool fused_ok = al16(dy) && al16(x) && al16(w) && al16(dx) && (!dxb || al16(dxb)) && (nv == 1 || nv == 2 || nv == 3 || nv == 4 || nv == 8 || (nv == 16 && rms && bf16));
  if (fused_ok) {
#define TW_NORM_FUSED(NV)                                                                                                                              \
  do {                                                                                                                                                 \
    if (bf16 && rms) hipLaunchKernelGGL((norm_bwd_fused_kernel<1, 1, NV>), dim3(nc), dim3(kT), 0, ctx->stream, dy, x, w, stats, dx, accumulate, dxb, partial, T);      \
    else if (bf16) hipLaunchKernelGGL((norm_bwd_fused_kernel<1, 0, NV>), dim3(nc), dim3(kT), 0, ctx->stream, dy, x, w, stats, dx, accumulate, dxb, partial, T);       \
    else if (rms) hipLaunchKernelGGL((norm_bwd_fused_kernel<0, 1, NV>), dim3(nc), dim3(kT), 0, ctx->stream, dy, x, w, stats, dx, accumulate, dxb, partial, T);        \
    else hipLaunchKernelGGL((norm_bwd_fused_kernel<0, 0, NV>), dim3(nc), dim3(kT), 0, ctx->stream, dy, x, w, stats, dx, accumulate, dxb, partial, T);                 \
  } while (0)
    switch (nv) {
      case 1: TW_NORM_FUSED(1); break;
      case 2: TW_NORM_FUSED(2); break;
      case 3: TW_NORM_FUSED(3); break;
      case 4: TW_NORM_FUSED(4); break;
      case 8: TW_NORM_FUSED(8); break;
      default:
        hipLaunchKernelGGL((norm_bwd_fused_kernel<1, 1, 16>), dim3(nc), dim3(kT), 0, ctx->stream, dy, x, w, stats, dx, accumulate, dxb, partial, T);
        break;
    }
#undef TW_NORM_FUSED
    TW_HIP(ctx, hipGetLastError());
    if (defer_reduce) return TWIST_OK;
    hipLaunchKernelGGL(reduce_partial_kernel, dim3((D + 15) / 16), dim3(kT), 0, ctx->stream, partial, (int64_t)2 * D, nc, 1.f, dw, D);
    if (db) hipLaunchKernelGGL(reduce_partial_kernel, dim3((D + 15) / 16), dim3(kT), 0, ctx->stream, partial + D, (int64_t)2 * D, nc, 1.f, db, D);
    TW_HIP(ctx, hipGetLastError());
    return TWIST_OK;
  }
  // general shapes: parameter gradients first (they read dy and x, which the dx pass leaves untouched)
  LAUNCH_BF(norm_bwd_dw_kernel, bf16, dim3((D + 63) / 64, nc), dim3(64), dy, x, stats, partial, T, D);
  if (!defer_reduce) hipLaunchKernelGGL(reduce_partial_kernel, dim3((D + 15) / 16), dim3(kT), 0, ctx->stream, partial, (int64_t)2 * D, nc, 1.f, dw, D);
  TW_HIP(ctx, hipGetLastError());
  if (db && !defer_reduce) {
    hipLaunchKernelGGL(reduce_partial_kernel, dim3((D + 15) / 16), dim3(kT), 0, ctx->stream, partial + D, (int64_t)2 * D, nc, 1.f, db, D);
    TW_HIP(ctx, hipGetLastError());
  }
  LAUNCH_BF2(norm_bwd_dx_kernel, bf16, rms, dim3((T + 3) / 4), dim3(kT), dy, x, w, stats, dx, accumulate, dxb, T, D);
  return TWIST_OK;
}

twist_status twist_col_reduce_batch(twist_ctx *ctx, const ColReduce *items, int n_items, int T) {
  const int nc = n_chunks(T);
  for (int i0 = 0; i0 < n_items; i0 += kReduceBatch) {
    ColReduceArgs a;
    const int m = std::min(kReduceBatch, n_items - i0);
    int widest = 1;
    for (int i = 0; i < m; ++i) { a.item[i] = items[i0 + i]; widest = std::max(widest, items[i0 + i].n); }
    hipLaunchKernelGGL(reduce_partial_batch_kernel, dim3((widest + 15) / 16, m), dim3(kT), 0, ctx->stream, a, nc);
    TW_HIP(ctx, hipGetLastError());
  }
  return TWIST_OK;
}

twist_status twist_colsum(twist_ctx *ctx, int bf16, const void *src, int64_t ld, float alpha, float *out, float *partial, int T, int n,
                          bool defer_reduce) {
  const int nc = n_chunks(T);
  LAUNCH_BF(colsum_kernel, bf16, dim3((n + 63) / 64, nc), dim3(64), src, ld, partial, T, n);
  if (defer_reduce) return TWIST_OK;
  hipLaunchKernelGGL(reduce_partial_kernel, dim3((n + 15) / 16), dim3(kT), 0, ctx->stream, partial, (int64_t)n, nc, alpha, out, n);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

// rotary table lives at the start of `qkv`-independent scratch handed in by the caller through twist_rope_table
twist_status twist_rope_table(twist_ctx *ctx, float *tab, int N, int dh, float theta) {
  const int half = dh / 2;
  hipLaunchKernelGGL(rope_table_kernel, grid1((int64_t)N * half), dim3(kT), 0, ctx->stream, tab, N, half, dh, theta);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_rope_apply(twist_ctx *ctx, int bf16, void *qkv, const float *tab, int B, int N, int Hs, int dh, float sign) {
  if (bf16 && dh % 16 == 0 && al16(qkv) && al16(tab)) {
    const int64_t total8 = (int64_t)B * N * 2 * Hs * (dh / 16);
    hipLaunchKernelGGL(rope_vec_kernel, grid1(total8), dim3(kT), 0, ctx->stream, static_cast<u32x4v *>(qkv), tab, N, Hs, dh, sign, total8);
    TW_HIP(ctx, hipGetLastError());
    return TWIST_OK;
  }
  const int64_t total = (int64_t)B * N * 2 * Hs * (dh / 2);
  LAUNCH_BF(rope_kernel, bf16, grid1(total), dim3(kT), qkv, tab, N, Hs, dh, sign, total);
  return TWIST_OK;
}

twist_status twist_act_fwd(twist_ctx *ctx, int bf16, int act, const void *gu, void *a, int T, int F, const int32_t *keep, int unit) {
  const int64_t total = (int64_t)T * F;
  if (bf16 && act == TWIST_ACT_SWIGLU && F % 8 == 0 && al16(gu) && al16(a)) {
    hipLaunchKernelGGL(swiglu_fwd_vec_kernel, grid1(total / 8), dim3(kT), 0, ctx->stream, static_cast<const u32x4v *>(gu), static_cast<u32x4v *>(a), F / 8, total / 8,
                       keep, unit);
    TW_HIP(ctx, hipGetLastError());
    return TWIST_OK;
  }
  if (bf16 && act != TWIST_ACT_SWIGLU && (keep ? F % 8 == 0 : total % 8 == 0) && al16(gu) && al16(a)) {
    hipLaunchKernelGGL(act_fwd_vec_kernel, grid1(total / 8), dim3(kT), 0, ctx->stream, act, static_cast<const u32x4v *>(gu), static_cast<u32x4v *>(a), total / 8,
                       keep, unit, F / 8);
    TW_HIP(ctx, hipGetLastError());
    return TWIST_OK;
  }
  LAUNCH_BF(act_fwd_kernel, bf16, grid1(total), dim3(kT), act, gu, a, F, total, keep, unit);
  return TWIST_OK;
}

twist_status twist_act_bwd(twist_ctx *ctx, int bf16, int act, const void *gu, const void *da, void *dgu, int T, int F, const int32_t *keep, int unit) {
  const int64_t total = (int64_t)T * F;
  if (bf16 && act == TWIST_ACT_SWIGLU && F % 8 == 0 && al16(gu) && al16(da) && al16(dgu)) {
    hipLaunchKernelGGL(swiglu_bwd_vec_kernel, grid1(total / 8), dim3(kT), 0, ctx->stream, static_cast<const u32x4v *>(gu), static_cast<const u32x4v *>(da),
                       static_cast<u32x4v *>(dgu), F / 8, total / 8, keep, unit);
    TW_HIP(ctx, hipGetLastError());
    return TWIST_OK;
  }
  if (bf16 && act != TWIST_ACT_SWIGLU && (keep ? F % 8 == 0 : total % 8 == 0) && al16(gu) && al16(da) && al16(dgu)) {
    hipLaunchKernelGGL(act_bwd_vec_kernel, grid1(total / 8), dim3(kT), 0, ctx->stream, act, static_cast<const u32x4v *>(gu), static_cast<const u32x4v *>(da),
                       static_cast<u32x4v *>(dgu), total / 8, keep, unit, F / 8);
    TW_HIP(ctx, hipGetLastError());
    return TWIST_OK;
  }
  LAUNCH_BF(act_bwd_kernel, bf16, grid1(total), dim3(kT), act, gu, da, dgu, F, total, keep, unit);
  return TWIST_OK;
}

twist_status twist_ce_fwd_bwd(twist_ctx *ctx, int bf16, void *logits, int64_t ld, const int32_t *targets, float *rowloss, float *loss, int T, int V) {
  if (bf16 && ld % 8 == 0 && al16(logits)) {
    u32x4v *lv = static_cast<u32x4v *>(logits);
    if (ld <= 4 * 2048) hipLaunchKernelGGL(ce_vec_kernel<4>, dim3(T), dim3(kT), 0, ctx->stream, lv, ld / 8, targets, rowloss, V, 1.f / (float)T);
    else if (ld <= 16 * 2048) hipLaunchKernelGGL(ce_vec_kernel<16>, dim3(T), dim3(kT), 0, ctx->stream, lv, ld / 8, targets, rowloss, V, 1.f / (float)T);
    else hipLaunchKernelGGL(ce_vec_long_kernel, dim3(T), dim3(kT), 0, ctx->stream, lv, ld / 8, targets, rowloss, V, 1.f / (float)T);
  } else
    LAUNCH_BF(ce_kernel, bf16, dim3(T), dim3(kT), logits, ld, targets, rowloss, V, 1.f / (float)T);
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(kT), 0, ctx->stream, rowloss, (int64_t)T, 1.f / (float)T, loss);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_mse_fwd_bwd(twist_ctx *ctx, int bf16, const float *x, const void *y, float *dx, void *dxb, float *partial, float *loss, int64_t n) {
  const int blocks = (int)std::min<int64_t>((n + kT - 1) / kT, 1024);
  LAUNCH_BF(mse_kernel, bf16, dim3(blocks), dim3(kT), x, y, dx, dxb, partial, n, 2.f / (float)n);
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(kT), 0, ctx->stream, partial, (int64_t)blocks, 1.f / (float)n, loss);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_sgd(twist_ctx *ctx, int bf16, void *params, float *master, const float *grads, int64_t n, float lr) {
  LAUNCH_BF(sgd_kernel, bf16, grid1(n), dim3(kT), params, master, grads, n, lr);
  return TWIST_OK;
}

twist_status twist_adamw(twist_ctx *ctx, int bf16, void *params, float *master, const float *grads, float *m, float *v, int64_t n, int64_t n_decay,
                         float lr, float b1, float b2, float eps, float wd, int64_t step) {
  const double bc1 = 1.0 - pow((double)b1, (double)step), bc2 = 1.0 - pow((double)b2, (double)step);
  LAUNCH_BF(adamw_kernel, bf16, grid1(n), dim3(kT), params, master, grads, m, v, n, n_decay, lr, b1, b2, eps, wd, (float)(1.0 / bc1), (float)(1.0 / bc2), step == 1 ? 1 : 0);
  return TWIST_OK;
}
