// Tiled causal attention for bf16 models on the matrix cores (v_mfma_f32_32x32x16_bf16), forward and backward.
//
// All kernels work on the fused [T, 3*Hs*dh] q|k|v buffer, d_head 64 or 128, N a multiple of 128.
// Layout facts used throughout (32x32x16 MFMA, wave of 64 lanes, g = lane/32, c = lane%32):
//   A operand (M x K): lane supplies row c, k = 8g .. 8g+7          B operand (K x N): lane supplies column c, same k
//   D (32 x 32):       lane holds column c, register r holds row 8*(r/4) + 4g + r%4
// Scores are formed TRANSPOSED, S^T = K Q^T, so that a lane owns one query column: the softmax statistics of a
// query live in one lane (plus its partner lane^32), and the probability tile can be fed straight back as the
// B operand of the next product by renaming the contraction index: MFMA k-slot (g, i) of step t stands for row
// 16t + 8*(i/4) + 4g + i%4 of the tile, which is exactly where register 8t+i of the D layout sits.
// Operands whose contraction index is the slow axis in memory (V in P.V, K in dS.K, Q and dO in the dK/dV
// products) stay row-major in LDS and are read with the transposing LDS load ds_read_tr16_b64, which hands
// each lane 4 consecutive contraction rows of one column.
//
// delta_i = sum_j p_ij dp_ij equals dO_i . O_i.  The forward kernel therefore also writes its output unrounded
// (fp32) and normalises by the sum of the probabilities AS ROUNDED for the matrix cores, so that O is an exact
// convex combination of the value rows; the dQ kernel forms delta from that fp32 output in its prologue.  With
// both in place a component common to all value rows (a large value bias) cancels exactly in p (dp - delta),
// which it does not when delta is taken from the bf16-rounded output.
//
// MASKED HEADS (Masked TwIST, Section 4.1: the full-width model with y = M * f(x)): every kernel takes an optional table
// `keep` with one entry per head; a head with keep[h] < 0 is masked, its output and its input gradients are written
// as zeros and none of its keys are visited, so the masked pass needs no extra kernels.
#include <type_traits>

#include "nn.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

// 2^x as the bare hardware instruction: results below the smallest normal number flush to zero, which is what a
// probability that small is worth; the library routine's extra range handling costs five more instructions per value
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// two floats to a packed pair of bf16, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ bf16x8 pack8(const f32x16 &v, int r0) {
  u32x4 u = {pack2(v[r0], v[r0 + 1]), pack2(v[r0 + 2], v[r0 + 3]), pack2(v[r0 + 4], v[r0 + 5]), pack2(v[r0 + 6], v[r0 + 7])};
  return __builtin_bit_cast(bf16x8, u);
}

__device__ __forceinline__ bf16x8 lds_frag(const uint16_t *p) { return *reinterpret_cast<const bf16x8 *>(p); }

// 8 contraction rows (two groups of 4) of one column, from a row-major LDS tile: rows row0..row0+3 and row0+8..row0+11
__device__ __forceinline__ bf16x8 lds_frag_tr(const uint16_t *tile, int ld, int row0, int col0) {
  const int s = threadIdx.x & 15;
  const uint16_t *p = tile + (row0 + (s >> 2)) * ld + col0 + 4 * (s & 3);
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 8 * ld));
  s16x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// cooperative copy of a [ROWS][DH] tile (row stride ldg in memory) into LDS with row stride ldl; 256 threads
template <int ROWS, int DH>
__device__ __forceinline__ void load_tile(uint16_t *lds, int ldl, const uint16_t *g, int64_t ldg) {
  constexpr int CPR = DH / 8, TOTAL = ROWS * CPR;
#pragma unroll
  for (int i = 0; i < TOTAL / 256; ++i) {
    const int c = threadIdx.x + 256 * i;
    const int r = c / CPR, k = (c % CPR) * 8;
    *reinterpret_cast<u32x4 *>(lds + r * ldl + k) = *reinterpret_cast<const u32x4 *>(g + (int64_t)r * ldg + k);
  }
}

// Causal work per query (or key) block grows linearly with its index, and all workgroups of a launch are
// usually resident at once, two per CU (workgroup b and b + half land on the same CU).  Blocks are therefore
// handed out in "snake" order: the first half of the grid takes the items from the most expensive down, the
// second half from the cheapest up, so that the two workgroups sharing a CU add up to the same work.
// Returns the rank of this workgroup's item in the list sorted by decreasing work.
__device__ __forceinline__ int snake_rank(int b, int nwg) {
  const int half = nwg >> 1;
  return b < half ? b : nwg - 1 - (b - half);
}

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

// ------------------------------------------------------------------------------------------- forward
// grid: (N/128) * B * Hs workgroups of 4 waves; wave w owns query rows [qb*128 + 32w, +32)
template <int DH>
__global__ __launch_bounds__(256) void flash_fwd_kernel(const uint16_t *qkv, uint16_t *o, float *o32, float *lse, int N, int Hs, float scale, const int32_t *keep) {
  constexpr int KS = DH / 16, MT = DH / 32, LDK = DH + 8, LDV = DH + 16;
  __shared__ __attribute__((aligned(16))) uint16_t Ks[64 * LDK];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[64 * LDV];
  const int nqb = N / 128, nbh = gridDim.x / nqb;
  const int rank = snake_rank(blockIdx.x, gridDim.x);
  const int qb = nqb - 1 - rank / nbh;  // late query blocks see the most keys
  const int bh = rank % nbh, b = bh / Hs, h = bh % Hs;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, c = lane & 31, g = lane >> 5;
  const int64_t HD = (int64_t)Hs * DH, ld = 3 * HD;
  const uint16_t *qp = qkv + (int64_t)b * N * ld + (int64_t)h * DH;
  const uint16_t *kp = qp + HD, *vp = qp + 2 * HD;
  const int q0 = qb * 128 + wave * 32, q = q0 + c;
  const float sc = scale * kLog2e;

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + (int64_t)q * ld + ks * 16 + g * 8);
  f32x16 oacc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const bool masked = keep && keep[h] < 0;  // a masked head (see MASKED HEADS above): no key is visited, zeros are written
  const int n_tiles = masked ? 0 : (qb + 1) * 2;
  for (int kt = 0; kt < n_tiles; ++kt) {
    __syncthreads();
    load_tile<64, DH>(Ks, LDK, kp + (int64_t)kt * 64 * ld, ld);
    load_tile<64, DH>(Vs, LDV, vp + (int64_t)kt * 64 * ld, ld);
    __syncthreads();
    if (kt * 64 > q0 + 31) continue;  // whole tile is in this wave's future
    f32x16 s[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[mt][r] = 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) s[mt] = MFMA(lds_frag(Ks + (mt * 32 + c) * LDK + ks * 16 + g * 8), qf[ks], s[mt]);
    const bool diag = kt * 64 + 63 > q0;
    float mx = -INFINITY;
    if (diag) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kt * 64 + mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (kv > q) s[mt][r] = -INFINITY;
        }
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mt][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The running maximum only has to keep 2^(s - m) in range, so it is raised (and the accumulators rescaled) only
    // when some query of the wave would otherwise exceed 2^8; on most tiles nothing is rescaled.  The first tile
    // always raises it: key 0 is visible to every query, so the new maximum is finite.
    const float mcand = fmaxf(m, mx * sc);
    const bool raise = __any(mcand > m + 8.f);
    const float mn = raise ? mcand : m;
    // probabilities, rounded to bf16 in pairs; the row sum is taken over the rounded values
    uint32_t pk[2][8];
    float sum = 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const uint32_t u = pack2(fast_exp2(fmaf(s[mt][r], sc, -mn)), fast_exp2(fmaf(s[mt][r + 1], sc, -mn)));
        pk[mt][r >> 1] = u;
        sum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, u), __builtin_bit_cast(bf16x2, 0x3f803f80u), sum, false);  // + both halves
      }
    if (raise) {
      const float alpha = fast_exp2(m - mn);
      l *= alpha;
      m = mn;
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
    }
    l += sum;
    // O^T[dh][q] += V^T[dh][kv] P^T[kv][q]
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const u32x4 pu = {pk[mt][4 * t], pk[mt][4 * t + 1], pk[mt][4 * t + 2], pk[mt][4 * t + 3]};
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pu);
#pragma unroll
        for (int i = 0; i < MT; ++i)
          oacc[i] = MFMA(lds_frag_tr(Vs, LDV, mt * 32 + 16 * t + 4 * g, i * 32 + 16 * ((lane >> 4) & 1)), pf, oacc[i]);
      }
  }
  l += __shfl_xor(l, 32, 64);
  const float inv = masked ? 0.f : 1.f / l;
  uint16_t *op = o + ((int64_t)b * N + q) * HD + (int64_t)h * DH;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      u32x2 w = {pack2(oacc[i][4 * j] * inv, oacc[i][4 * j + 1] * inv), pack2(oacc[i][4 * j + 2] * inv, oacc[i][4 * j + 3] * inv)};
      *reinterpret_cast<u32x2 *>(op + i * 32 + 8 * j + 4 * g) = w;
      if (o32) {
        const f32x4 w4 = {oacc[i][4 * j] * inv, oacc[i][4 * j + 1] * inv, oacc[i][4 * j + 2] * inv, oacc[i][4 * j + 3] * inv};
        *reinterpret_cast<f32x4 *>(o32 + ((int64_t)b * N + q) * HD + (int64_t)h * DH + i * 32 + 8 * j + 4 * g) = w4;
      }
    }
  if (g == 0) lse[((int64_t)b * Hs + h) * N + q] = masked ? 0.f : (m + log2f(l)) * kLn2;
}

// ------------------------------------------------------------------------------------------- backward: dQ (and delta)
// Same decomposition as the forward kernel.  delta_q = dO_q . O_q from the unrounded forward output, then
// dS^T = p (dp - delta) scale and dQ^T[dh][q] += K^T[dh][kv] dS^T[kv][q].
template <int DH>
__global__ __launch_bounds__(256) void flash_bwd_dq_kernel(const uint16_t *qkv, const uint16_t *dout, const float *o32, const float *lse, float *delta,
                                                           uint16_t *dqkv, int N, int Hs, float scale, const int32_t *keep) {
  constexpr int KS = DH / 16, MT = DH / 32, LD = DH + 16;
  __shared__ __attribute__((aligned(16))) uint16_t Ks[64 * LD];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[64 * LD];
  const int nqb = N / 128, nbh = gridDim.x / nqb;
  const int rank = snake_rank(blockIdx.x, gridDim.x);
  const int qb = nqb - 1 - rank / nbh;  // late query blocks see the most keys
  const int bh = rank % nbh, b = bh / Hs, h = bh % Hs;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, c = lane & 31, g = lane >> 5;
  const int64_t HD = (int64_t)Hs * DH, ld = 3 * HD;
  const uint16_t *qp = qkv + (int64_t)b * N * ld + (int64_t)h * DH;
  const uint16_t *kp = qp + HD, *vp = qp + 2 * HD;
  const int q0 = qb * 128 + wave * 32, q = q0 + c;
  const float sc = scale * kLog2e;
  const float L2 = lse[((int64_t)b * Hs + h) * N + q] * kLog2e;

  bf16x8 qf[KS], gf[KS];
  const uint16_t *gp = dout + ((int64_t)b * N + q) * HD + (int64_t)h * DH;
  const float *op32 = o32 + ((int64_t)b * N + q) * HD + (int64_t)h * DH;
  float dl = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + (int64_t)q * ld + ks * 16 + g * 8);
    gf[ks] = *reinterpret_cast<const bf16x8 *>(gp + ks * 16 + g * 8);
    const f32x4 oa = *reinterpret_cast<const f32x4 *>(op32 + ks * 16 + g * 8), ob = *reinterpret_cast<const f32x4 *>(op32 + ks * 16 + g * 8 + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) dl += (float)gf[ks][e] * oa[e] + (float)gf[ks][e + 4] * ob[e];
  }
  dl += __shfl_xor(dl, 32, 64);
  if (g == 0) delta[((int64_t)b * Hs + h) * N + q] = dl;
  f32x16 acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  const int n_tiles = (keep && keep[h] < 0) ? 0 : (qb + 1) * 2;  // masked head: the gradient is zero
  for (int kt = 0; kt < n_tiles; ++kt) {
    __syncthreads();
    load_tile<64, DH>(Ks, LD, kp + (int64_t)kt * 64 * ld, ld);
    load_tile<64, DH>(Vs, LD, vp + (int64_t)kt * 64 * ld, ld);
    __syncthreads();
    if (kt * 64 > q0 + 31) continue;
    f32x16 s[2], dp[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[mt][r] = 0.f; dp[mt][r] = 0.f; }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s[mt] = MFMA(lds_frag(Ks + (mt * 32 + c) * LD + ks * 16 + g * 8), qf[ks], s[mt]);
        dp[mt] = MFMA(lds_frag(Vs + (mt * 32 + c) * LD + ks * 16 + g * 8), gf[ks], dp[mt]);
      }
    const bool diag = kt * 64 + 63 > q0;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kv = kt * 64 + mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        float p = fast_exp2(fmaf(s[mt][r], sc, -L2));
        if (diag && kv > q) p = 0.f;
        s[mt][r] = p * (dp[mt][r] - dl) * scale;
      }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 df = pack8(s[mt], 8 * t);
#pragma unroll
        for (int i = 0; i < MT; ++i)
          acc[i] = MFMA(lds_frag_tr(Ks, LD, mt * 32 + 16 * t + 4 * g, i * 32 + 16 * ((lane >> 4) & 1)), df, acc[i]);
      }
  }
  uint16_t *op = dqkv + ((int64_t)b * N + q) * ld + (int64_t)h * DH;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      u32x2 w = {pack2(acc[i][4 * j], acc[i][4 * j + 1]), pack2(acc[i][4 * j + 2], acc[i][4 * j + 3])};
      *reinterpret_cast<u32x2 *>(op + i * 32 + 8 * j + 4 * g) = w;
    }
}

// ------------------------------------------------------------------------------------------- backward: dK, dV
// grid: (N/128) * B * Hs; wave w owns key/value rows [kb*128 + 32w, +32) and walks the query tiles at or below the
// diagonal.  S[q][kv] = Q K^T and dP = dO V^T put a key column in each lane; P and dS then are the B operands of
// dV^T[dh][kv] += dO^T[dh][q] P[q][kv]  and  dK^T[dh][kv] += Q^T[dh][q] dS[q][kv].
template <int DH>
__global__ __launch_bounds__(256) void flash_bwd_dkv_kernel(const uint16_t *qkv, const uint16_t *dout, const float *lse, const float *delta,
                                                            uint16_t *dqkv, int N, int Hs, float scale, const int32_t *keep) {
  constexpr int KS = DH / 16, MT = DH / 32, LD = DH + 16;
  __shared__ __attribute__((aligned(16))) uint16_t Qs[64 * LD];
  __shared__ __attribute__((aligned(16))) uint16_t Gs[64 * LD];
  __shared__ __attribute__((aligned(16))) float Ls[64], Ds[64];
  const int nkb = N / 128, nbh = gridDim.x / nkb;
  const int rank = snake_rank(blockIdx.x, gridDim.x);
  const int kb = rank / nbh;  // early key blocks see the most queries
  const int bh = rank % nbh, b = bh / Hs, h = bh % Hs;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, c = lane & 31, g = lane >> 5;
  const int64_t HD = (int64_t)Hs * DH, ld = 3 * HD;
  const uint16_t *qp = qkv + (int64_t)b * N * ld + (int64_t)h * DH;
  const uint16_t *gp = dout + (int64_t)b * N * HD + (int64_t)h * DH;
  const int k0 = kb * 128 + wave * 32, kv = k0 + c;
  const float sc = scale * kLog2e;
  const float *lse_b = lse + ((int64_t)b * Hs + h) * N, *del_b = delta + ((int64_t)b * Hs + h) * N;

  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = *reinterpret_cast<const bf16x8 *>(qp + HD + (int64_t)kv * ld + ks * 16 + g * 8);
    vf[ks] = *reinterpret_cast<const bf16x8 *>(qp + 2 * HD + (int64_t)kv * ld + ks * 16 + g * 8);
  }
  f32x16 dk[MT], dv[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[i][r] = 0.f; dv[i][r] = 0.f; }

  const int n_q = (keep && keep[h] < 0) ? 0 : N / 64;  // masked head: the gradients are zero
  for (int qt = kb * 2; qt < n_q; ++qt) {
    __syncthreads();
    load_tile<64, DH>(Qs, LD, qp + (int64_t)qt * 64 * ld, ld);
    load_tile<64, DH>(Gs, LD, gp + (int64_t)qt * 64 * HD, HD);
    if (threadIdx.x < 64) Ls[threadIdx.x] = lse_b[qt * 64 + threadIdx.x] * kLog2e;
    else if (threadIdx.x < 128) Ds[threadIdx.x - 64] = del_b[qt * 64 + threadIdx.x - 64];
    __syncthreads();
    if (qt * 64 + 63 < k0) continue;  // every query of the tile precedes this wave's keys
    f32x16 s[2], dp[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[mt][r] = 0.f; dp[mt][r] = 0.f; }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s[mt] = MFMA(lds_frag(Qs + (mt * 32 + c) * LD + ks * 16 + g * 8), kf[ks], s[mt]);
        dp[mt] = MFMA(lds_frag(Gs + (mt * 32 + c) * LD + ks * 16 + g * 8), vf[ks], dp[mt]);
      }
    const bool diag = qt * 64 < k0 + 31;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ql = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);  // query row inside the tile
        float p = fast_exp2(fmaf(s[mt][r], sc, -Ls[ql]));
        if (diag && qt * 64 + ql < kv) p = 0.f;
        dp[mt][r] = p * (dp[mt][r] - Ds[ql]) * scale;  // dS
        s[mt][r] = p;
      }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pf = pack8(s[mt], 8 * t), df = pack8(dp[mt], 8 * t);
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          dv[i] = MFMA(lds_frag_tr(Gs, LD, mt * 32 + 16 * t + 4 * g, i * 32 + 16 * ((lane >> 4) & 1)), pf, dv[i]);
          dk[i] = MFMA(lds_frag_tr(Qs, LD, mt * 32 + 16 * t + 4 * g, i * 32 + 16 * ((lane >> 4) & 1)), df, dk[i]);
        }
      }
  }
  uint16_t *op = dqkv + ((int64_t)b * N + kv) * ld + (int64_t)h * DH;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      u32x2 wk = {pack2(dk[i][4 * j], dk[i][4 * j + 1]), pack2(dk[i][4 * j + 2], dk[i][4 * j + 3])};
      u32x2 wv = {pack2(dv[i][4 * j], dv[i][4 * j + 1]), pack2(dv[i][4 * j + 2], dv[i][4 * j + 3])};
      *reinterpret_cast<u32x2 *>(op + HD + i * 32 + 8 * j + 4 * g) = wk;
      *reinterpret_cast<u32x2 *>(op + 2 * HD + i * 32 + 8 * j + 4 * g) = wv;
    }
}

// =========================================================================================== d_head = 128, pipelined
// Same decomposition, but the 64 x 128 key / value (or query / dO) tiles of step t+1 travel from global memory
// straight into LDS (buffer_load_dwordx4 ... lds, lane l of a wave writes 16 bytes at base + 16 l) while step t is
// computed: two stages of two 16 KB tiles, one barrier per step.  The fixed write pattern leaves no room for row
// padding; bank conflicts are avoided by storing chunk c (16 bytes) of row r at position c ^ swz(r),
// swz(r) = 4 (r & 3) + ((r >> 2) & 3), which serves both read patterns: 16 consecutive rows of one chunk column
// (plain 16-byte fragment reads) and 4 consecutive rows of two adjacent chunks (transposing reads).
namespace dl {

constexpr int DH = 128, KS = 8, MT = 4;
constexpr int TILE_B = 64 * DH * 2;    // one staged tile
constexpr int STAGE_B = 2 * TILE_B;    // K and V (or Q and dO)
typedef __attribute__((address_space(3))) void *lds_void;

__device__ __forceinline__ int swz(int r) { return 4 * (r & 3) + ((r >> 2) & 3); }
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}

// Per-lane byte offsets (within a tile) of the two kinds of fragment reads.
struct ReadOffsets {
  uint32_t fo[KS];          // plain fragment of k-step ks for tile row (lane & 31); add 8192 per 32 rows
  uint32_t ta[MT], tb[MT];  // transposing reads of head-dim block i: contraction rows +0..3 and +8..11; add 256 per row
  __device__ __forceinline__ void init(int lane) {
    const int c = lane & 31, g = lane >> 5, s16 = lane & 15, rho = (s16 >> 2) & 3, dlt = (s16 & 3) >> 1, hi = (lane >> 4) & 1;
    const int x = swz(c);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fo[ks] = (uint32_t)(c * 256 + (((2 * ks + g) ^ x) << 4));
    const int within = (s16 & 1) * 8;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      ta[i] = (uint32_t)((4 * g + rho) * 256 + within + (((2 * hi + dlt) ^ g) << 4) + ((i ^ rho) << 6));
      tb[i] = (uint32_t)((4 * g + rho + 8) * 256 + within + (((2 * hi + dlt) ^ (g + 2)) << 4) + ((i ^ rho) << 6));
    }
  }
};

__device__ __forceinline__ bf16x8 frag(const char *tile, uint32_t off) { return *reinterpret_cast<const bf16x8 *>(tile + off); }
__device__ __forceinline__ bf16x8 frag_tr(const char *rows, uint32_t a, uint32_t b) {
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  s16x4 x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(rows + a));
  s16x4 y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(rows + b));
  s16x8 v = {x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// Loads from global memory straight into LDS (lane l writes its 16 or 4 bytes at lds + bytes * l; lanes whose offset
// is outside the descriptor's range write zeros).  Written as assembly on purpose: for the builtin form the compiler
// cannot tell which LDS bytes a load fills and makes every later transposing LDS read wait for ALL such loads in
// flight, which turns the prefetch of the next tile into a stall.  Completion is awaited explicitly (DL_WAIT_VM0
// followed by a barrier) before any wave reads the bytes.  M0 (the LDS base of the instruction) is saved and restored.
typedef uint32_t desc_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ desc_t make_desc(const void *p, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(p);
  desc_t d;
  d.x = __builtin_amdgcn_readfirstlane((uint32_t)a);
  d.y = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
  d.z = __builtin_amdgcn_readfirstlane(bytes);
  d.w = 0x00020000u;
  return d;
}
template <int BYTES>
__device__ __forceinline__ void dma(desc_t desc, const char *lds, uint32_t voff) {
  const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void)(lds));
  uint32_t keep;
  if (BYTES == 16)
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep) : "s"(l), "v"(voff), "s"(desc) : "memory");
  else
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dword %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep) : "s"(l), "v"(voff), "s"(desc) : "memory");
}

// Each of the 4 waves brings in 4 of the 16 one-KB pieces (4 rows each) of a tile.
struct TileLoader {
  uint32_t off[4];  // byte offset of this lane's chunk within tile 0, from the buffer base
  __device__ __forceinline__ void init(int64_t ld_elems, uint32_t col_byte0, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 4 * (wave + 4 * i) + (lane >> 4), chunk = (lane & 15) ^ swz(row);
      off[i] = (uint32_t)(row * ld_elems * 2) + col_byte0 + chunk * 16;
    }
  }
  __device__ __forceinline__ void issue(desc_t rsrc, char *dst, uint32_t tile_byte0, int wave) const {
#pragma unroll
    for (int i = 0; i < 4; ++i) dma<16>(rsrc, dst + (wave + 4 * i) * 1024, off[i] + tile_byte0);
  }
};

#define DL_WAIT_VM0 __builtin_amdgcn_s_waitcnt(0x0f70)

// two waves per SIMD (two workgroups per CU) is what lets one workgroup's softmax overlap the other's matrix work
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void flash_fwd_dl_kernel(const uint16_t *qkv, uint16_t *o, float *o32, float *lse, int N, int Hs, float scale, const int32_t *keep) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE_B];
  const int nqb = N / 128, nbh = gridDim.x / nqb;
  const int rank = snake_rank(blockIdx.x, gridDim.x);
  const int qb = nqb - 1 - rank / nbh;
  const int bh = rank % nbh, b = bh / Hs, h = bh % Hs;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, c = lane & 31, g = lane >> 5;
  const int64_t HD = (int64_t)Hs * DH, ld = 3 * HD;
  const uint16_t *batch = qkv + (int64_t)b * N * ld;
  const uint16_t *qp = batch + (int64_t)h * DH;
  const int q0 = qb * 128 + wave * 32, q = q0 + c;
  const float sc = scale * kLog2e;
  const desc_t rs = make_desc(batch, (uint32_t)(N * ld * 2));
  const uint32_t tstep = (uint32_t)(64 * ld * 2);
  TileLoader lk, lv;
  lk.init(ld, (uint32_t)((HD + h * DH) * 2), wave, lane);
  lv.init(ld, (uint32_t)((2 * HD + h * DH) * 2), wave, lane);
  ReadOffsets ro;
  ro.init(lane);

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + (int64_t)q * ld + ks * 16 + g * 8);
  f32x16 oacc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const bool masked = keep && keep[h] < 0;  // a masked head: no key is visited (and nothing is loaded), zeros are written
  const int n_tiles = masked ? 0 : (qb + 1) * 2;
  if (!masked) {
    lk.issue(rs, smem, 0, wave);
    lv.issue(rs, smem + TILE_B, 0, wave);
  }
  auto step = [&](int kt, auto stage_c) {
    constexpr int ST = decltype(stage_c)::value;
    DL_WAIT_VM0;                    // this wave's pieces of tile kt have landed
    __builtin_amdgcn_s_barrier();   // everybody's have, and everybody is done with the other stage
    if (kt + 1 < n_tiles) {
      lk.issue(rs, smem + (ST ^ 1) * STAGE_B, (uint32_t)(kt + 1) * tstep, wave);
      lv.issue(rs, smem + (ST ^ 1) * STAGE_B + TILE_B, (uint32_t)(kt + 1) * tstep, wave);
    }
    if (kt * 64 > q0 + 31) return;  // whole tile is in this wave's future
    const char *Kt = smem + ST * STAGE_B, *Vt = Kt + TILE_B;
    f32x16 s[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[mt][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) s[mt] = MFMA(frag(Kt + mt * 8192, ro.fo[ks]), qf[ks], s[mt]);
    }
    if (kt * 64 + 63 > q0) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kt * 64 + mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (kv > q) s[mt][r] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mt][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The running maximum only has to keep 2^(s - m) in range, so it is raised (and the accumulators rescaled) only
    // when some query of the wave would otherwise exceed 2^8; on most tiles nothing is rescaled.  The first tile
    // always raises it: key 0 is visible to every query, so the new maximum is finite.
    const float mcand = fmaxf(m, mx * sc);
    const bool raise = __any(mcand > m + 8.f);
    const float mn = raise ? mcand : m;
    uint32_t pk[2][8];
    float sum = 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const uint32_t u = pack2(fast_exp2(fmaf(s[mt][r], sc, -mn)), fast_exp2(fmaf(s[mt][r + 1], sc, -mn)));
        pk[mt][r >> 1] = u;
        sum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, u), __builtin_bit_cast(bf16x2, 0x3f803f80u), sum, false);  // + both halves
      }
    if (raise) {
      const float alpha = fast_exp2(m - mn);
      l *= alpha;
      m = mn;
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
    }
    l += sum;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const u32x4 pu = {pk[mt][4 * t], pk[mt][4 * t + 1], pk[mt][4 * t + 2], pk[mt][4 * t + 3]};
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pu);
#pragma unroll
        for (int i = 0; i < MT; ++i) oacc[i] = MFMA(frag_tr(Vt + (mt * 32 + 16 * t) * 256, ro.ta[i], ro.tb[i]), pf, oacc[i]);
      }
  };
  for (int kt = 0; kt < n_tiles; kt += 2) {
    step(kt, std::integral_constant<int, 0>());
    step(kt + 1, std::integral_constant<int, 1>());  // n_tiles is even
  }
  l += __shfl_xor(l, 32, 64);
  const float inv = masked ? 0.f : 1.f / l;
  uint16_t *op = o + ((int64_t)b * N + q) * HD + (int64_t)h * DH;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      u32x2 w = {pack2(oacc[i][4 * j] * inv, oacc[i][4 * j + 1] * inv), pack2(oacc[i][4 * j + 2] * inv, oacc[i][4 * j + 3] * inv)};
      *reinterpret_cast<u32x2 *>(op + i * 32 + 8 * j + 4 * g) = w;
      if (o32) {
        const f32x4 w4 = {oacc[i][4 * j] * inv, oacc[i][4 * j + 1] * inv, oacc[i][4 * j + 2] * inv, oacc[i][4 * j + 3] * inv};
        *reinterpret_cast<f32x4 *>(o32 + ((int64_t)b * N + q) * HD + (int64_t)h * DH + i * 32 + 8 * j + 4 * g) = w4;
      }
    }
  if (g == 0) lse[((int64_t)b * Hs + h) * N + q] = masked ? 0.f : (m + log2f(l)) * kLn2;
}

// Backward of the rotary embedding on a lane's 64 gradient values of one row (acc[i][4 j + e] is head-dim column
// 32 i + 8 j + 4 g + e): columns f and f + 64 form a pair rotated by the angle of (position, f); the backward pass turns
// the gradient by the opposite angle.  tab holds (cos, sin) for f = 0..63 of every position, 128 floats per position.
__device__ __forceinline__ void rope_grad(f32x16 (&acc)[MT], const float *tab, int pos, int g) {
  const f32x4 *row = reinterpret_cast<const f32x4 *>(tab + (int64_t)pos * DH);
#pragma unroll
  for (int i = 0; i < MT / 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int f = 32 * i + 8 * j + 4 * g;  // first of the lane's four consecutive pair indices
      const f32x4 w0 = row[f / 2], w1 = row[f / 2 + 1];
      const float cs[4] = {w0[0], w0[2], w1[0], w1[2]}, sn[4] = {w0[1], w0[3], w1[1], w1[3]};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float a = acc[i][4 * j + e], b = acc[i + MT / 2][4 * j + e];
        acc[i][4 * j + e] = a * cs[e] + b * sn[e];
        acc[i + MT / 2][4 * j + e] = b * cs[e] - a * sn[e];
      }
    }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void flash_bwd_dq_dl_kernel(const uint16_t *qkv, const uint16_t *dout, const float *o32, const float *lse, float *delta,
                                                              uint16_t *dqkv, int N, int Hs, float scale, const float *rope, const int32_t *keep) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE_B];
  const int nqb = N / 128, nbh = gridDim.x / nqb;
  const int rank = snake_rank(blockIdx.x, gridDim.x);
  const int qb = nqb - 1 - rank / nbh;
  const int bh = rank % nbh, b = bh / Hs, h = bh % Hs;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, c = lane & 31, g = lane >> 5;
  const int64_t HD = (int64_t)Hs * DH, ld = 3 * HD;
  const uint16_t *batch = qkv + (int64_t)b * N * ld;
  const uint16_t *qp = batch + (int64_t)h * DH;
  const int q0 = qb * 128 + wave * 32, q = q0 + c;
  const float sc = scale * kLog2e;
  const float L2 = lse[((int64_t)b * Hs + h) * N + q] * kLog2e;
  const desc_t rs = make_desc(batch, (uint32_t)(N * ld * 2));
  const uint32_t tstep = (uint32_t)(64 * ld * 2);
  TileLoader lk, lv;
  lk.init(ld, (uint32_t)((HD + h * DH) * 2), wave, lane);
  lv.init(ld, (uint32_t)((2 * HD + h * DH) * 2), wave, lane);
  ReadOffsets ro;
  ro.init(lane);
  const bool masked = keep && keep[h] < 0;  // masked head: the gradient is zero, nothing is loaded
  const int n_tiles = masked ? 0 : (qb + 1) * 2;
  if (!masked) {
    lk.issue(rs, smem, 0, wave);
    lv.issue(rs, smem + TILE_B, 0, wave);
  }

  bf16x8 qf[KS], gf[KS];
  const uint16_t *gp = dout + ((int64_t)b * N + q) * HD + (int64_t)h * DH;
  const float *op32 = o32 + ((int64_t)b * N + q) * HD + (int64_t)h * DH;
  float dl = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + (int64_t)q * ld + ks * 16 + g * 8);
    gf[ks] = *reinterpret_cast<const bf16x8 *>(gp + ks * 16 + g * 8);
    const f32x4 oa = *reinterpret_cast<const f32x4 *>(op32 + ks * 16 + g * 8), ob = *reinterpret_cast<const f32x4 *>(op32 + ks * 16 + g * 8 + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) dl += (float)gf[ks][e] * oa[e] + (float)gf[ks][e + 4] * ob[e];
  }
  dl += __shfl_xor(dl, 32, 64);
  if (g == 0) delta[((int64_t)b * Hs + h) * N + q] = dl;
  const float dls = dl * scale;
  f32x16 acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  auto step = [&](int kt, auto stage_c) {
    constexpr int ST = decltype(stage_c)::value;
    DL_WAIT_VM0;
    __builtin_amdgcn_s_barrier();
    if (kt + 1 < n_tiles) {
      lk.issue(rs, smem + (ST ^ 1) * STAGE_B, (uint32_t)(kt + 1) * tstep, wave);
      lv.issue(rs, smem + (ST ^ 1) * STAGE_B + TILE_B, (uint32_t)(kt + 1) * tstep, wave);
    }
    if (kt * 64 > q0 + 31) return;
    const char *Kt = smem + ST * STAGE_B, *Vt = Kt + TILE_B;
    const bool diag = kt * 64 + 63 > q0;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s = MFMA(frag(Kt + mt * 8192, ro.fo[ks]), qf[ks], s);
        dp = MFMA(frag(Vt + mt * 8192, ro.fo[ks]), gf[ks], dp);
      }
      if (diag) {  // tiles that straddle the diagonal: keys after the query get no weight
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kt * 64 + mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (kv > q) s[r] = -INFINITY;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = fast_exp2(fmaf(s[r], sc, -L2)) * fmaf(dp[r], scale, -dls);  // p (dp - delta) scale
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 df = pack8(s, 8 * t);
#pragma unroll
        for (int i = 0; i < MT; ++i) acc[i] = MFMA(frag_tr(Kt + (mt * 32 + 16 * t) * 256, ro.ta[i], ro.tb[i]), df, acc[i]);
      }
    }
  };
  for (int kt = 0; kt < n_tiles; kt += 2) {
    step(kt, std::integral_constant<int, 0>());
    step(kt + 1, std::integral_constant<int, 1>());
  }
  if (rope) rope_grad(acc, rope, q, g);
  uint16_t *op = dqkv + ((int64_t)b * N + q) * ld + (int64_t)h * DH;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      u32x2 w = {pack2(acc[i][4 * j], acc[i][4 * j + 1]), pack2(acc[i][4 * j + 2], acc[i][4 * j + 3])};
      *reinterpret_cast<u32x2 *>(op + i * 32 + 8 * j + 4 * g) = w;
    }
}

// dK / dV with 8 waves per workgroup, one workgroup per CU.  The waves w and w + 4 of a SIMD own the SAME 32 keys and
// split the work of a query tile between them instead of each doing all of it with one wave per SIMD:
//   producer (w < 4): S = Q K^T and dP = dO V^T for 32 queries x its 32 keys (K and V fragments stay in registers),
//                     then P = 2^(S sc - lse) and dS = P (dP - delta) scale, handed over through LDS in exactly the
//                     register layout the next products take them in (lane to same lane, 64 bytes per lane);
//   consumer (w >= 4): dV^T += dO^T P and dK^T += Q^T dS for the 32 queries the producer finished one phase earlier
//                     (all 128 accumulator registers are here, the producer has none).
// Both issue 16 matrix instructions per phase of 32 queries; the producer's exponentials run under the consumer's
// products on the same SIMD.  One workgroup barrier per phase.  The 64-query Q / dO tiles live in three LDS stages (the
// tile being loaded, the producer's, and the consumer's, which is half a tile behind), the hand-over area in two.
// A workgroup handles the key blocks p and nkb-1-p one after the other, so that all workgroups carry the same work.
constexpr int DKV_LD_OFF = 3 * STAGE_B;             // per stage: 64 log-sum-exps, 64 deltas
constexpr int DKV_XCH_OFF = DKV_LD_OFF + 3 * 512;   // [2 phases][4 key blocks][P lo, P hi, dS lo, dS hi][64 lanes] x 16 bytes
constexpr int DKV_SMEM = DKV_XCH_OFF + 2 * 4 * 4096;
#define DL_WAIT_LGKM0 __builtin_amdgcn_s_waitcnt(0xc07f)

__global__ __launch_bounds__(512) void flash_bwd_dkv_dl_kernel(const uint16_t *qkv, const uint16_t *dout, const float *lse, const float *delta,
                                                               uint16_t *dqkv, int N, int Hs, float scale, const float *rope, const int32_t *keep) {
  __shared__ __attribute__((aligned(1024))) char smem[DKV_SMEM];
  const int nkb = N / 128, npair = (nkb + 1) / 2, nbh = gridDim.x / npair;
  const int pr = (int)blockIdx.x / nbh;
  const int bh = blockIdx.x % nbh, b = bh / Hs, h = bh % Hs;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, c = lane & 31, g = lane >> 5;
  const int wk = wave & 3;
  const bool producer = wave < 4;
  const int64_t HD = (int64_t)Hs * DH, ld = 3 * HD;
  const uint16_t *batch = qkv + (int64_t)b * N * ld;
  const uint16_t *qp = batch + (int64_t)h * DH;
  const uint16_t *gbatch = dout + (int64_t)b * N * HD;
  const float sc = scale * kLog2e;
  const float *lse_b = lse + ((int64_t)b * Hs + h) * N, *del_b = delta + ((int64_t)b * Hs + h) * N;
  const desc_t rq = make_desc(batch, (uint32_t)(N * ld * 2)), rg = make_desc(gbatch, (uint32_t)(N * HD * 2));
  const desc_t rl = make_desc(lse_b, (uint32_t)(N * 4)), rd = make_desc(del_b, (uint32_t)(N * 4));
  const uint32_t qstep = (uint32_t)(64 * ld * 2), gstep = (uint32_t)(64 * HD * 2);
  TileLoader lt;  // the producers bring in the query tile and the log-sum-exps, the consumers the dO tile and the deltas
  if (producer) lt.init(ld, (uint32_t)(h * DH * 2), wk, lane);
  else lt.init(HD, (uint32_t)(h * DH * 2), wk, lane);
  ReadOffsets ro;
  ro.init(lane);
  const bool masked = keep && keep[h] < 0;  // masked head: the gradients are zero, nothing is loaded
  auto issue = [&](int qt, int st) {
    if (producer) {
      lt.issue(rq, smem + st * STAGE_B, (uint32_t)qt * qstep, wk);
      if (wk == 0) dma<4>(rl, smem + DKV_LD_OFF + st * 512, (uint32_t)((qt * 64 + lane) * 4));
    } else {
      lt.issue(rg, smem + st * STAGE_B + TILE_B, (uint32_t)qt * gstep, wk);
      if (wk == 0) dma<4>(rd, smem + DKV_LD_OFF + st * 512 + 256, (uint32_t)((qt * 64 + lane) * 4));
    }
  };

  for (int item = 0; item < 2; ++item) {
    const int kb = item ? nkb - 1 - pr : pr;
    if (item && 2 * pr == nkb - 1) break;  // an odd number of key blocks: the middle one has no partner
    const int k0 = kb * 128 + wk * 32, kv = k0 + c;
    const int qt0 = kb * 2;                          // first query tile at or below the diagonal
    const int n_steps = masked ? 0 : N / 64 - qt0;   // query tiles qt0 .. N/64 - 1
    const int n_ph = 2 * n_steps;                    // phases of 32 queries; the consumer runs one phase behind
    if (n_steps) issue(qt0, 0);
    // phase ph covers queries [q_lo, q_lo + 32) of tile ph / 2 (stage (ph / 2) % 3); it is skipped when all of them
    // precede this wave's keys
    auto q_lo_of = [&](int ph) { return (qt0 + (ph >> 1)) * 64 + (ph & 1) * 32; };
    if (producer) {
      bf16x8 kf[KS], vf[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        kf[ks] = *reinterpret_cast<const bf16x8 *>(qp + HD + (int64_t)kv * ld + ks * 16 + g * 8);
        vf[ks] = *reinterpret_cast<const bf16x8 *>(qp + 2 * HD + (int64_t)kv * ld + ks * 16 + g * 8);
      }
      DL_WAIT_VM0;  // the first tile, and the key / value fragments
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(kf[ks]), "+v"(vf[ks]));  // (used here: the compiler may not sink the loads, and its waits for them, into the loop)
      __builtin_amdgcn_s_barrier();
      for (int ph = 0; ph <= n_ph; ++ph) {
        const int t = ph >> 1, mt = ph & 1;
        if (mt == 0 && t + 1 < n_steps) issue(qt0 + t + 1, (t + 1) % 3);
        const int q_lo = q_lo_of(ph);
        if (ph < n_ph && q_lo + 31 >= k0) {
          const int st = t % 3;
          const char *Qt = smem + st * STAGE_B + mt * 8192, *Gt = Qt + TILE_B;
          const float *Ls = reinterpret_cast<const float *>(smem + DKV_LD_OFF + st * 512) + mt * 32, *Ds = Ls + 64;
          f32x16 sv, dp;
#pragma unroll
          for (int r = 0; r < 16; ++r) { sv[r] = 0.f; dp[r] = 0.f; }
          // all 16 fragments are requested before the first product (the producer has the registers for it): one LDS
          // round trip per phase instead of one per pair of products
          bf16x8 qf[KS], gf[KS];
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) { qf[ks] = frag(Qt, ro.fo[ks]); gf[ks] = frag(Gt, ro.fo[ks]); }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            sv = MFMA(qf[ks], kf[ks], sv);
            dp = MFMA(gf[ks], vf[ks], dp);
          }
          const bool diag = q_lo < k0 + 31;  // some query of the phase precedes some key of the wave
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const int qrow = 8 * r4 + 4 * g;  // first of 4 consecutive query rows inside the phase
            const f32x4 L4 = *reinterpret_cast<const f32x4 *>(Ls + qrow), D4 = *reinterpret_cast<const f32x4 *>(Ds + qrow);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int r = 4 * r4 + e;
              float x = fmaf(sv[r], sc, -L4[e] * kLog2e);
              if (diag && q_lo + qrow + e < kv) x = -INFINITY;
              const float pv = fast_exp2(x);
              dp[r] = pv * fmaf(dp[r], scale, -D4[e] * scale);  // dS
              sv[r] = pv;
            }
          }
          u32x4 *X = reinterpret_cast<u32x4 *>(smem + DKV_XCH_OFF + ((ph & 1) * 4 + wk) * 4096);
          X[lane] = __builtin_bit_cast(u32x4, pack8(sv, 0));
          X[64 + lane] = __builtin_bit_cast(u32x4, pack8(sv, 8));
          X[128 + lane] = __builtin_bit_cast(u32x4, pack8(dp, 0));
          X[192 + lane] = __builtin_bit_cast(u32x4, pack8(dp, 8));
        }
        if (mt) DL_WAIT_VM0;  // end of a tile: this wave's pieces of the next one have landed
        DL_WAIT_LGKM0;        // the hand-over is written
        __builtin_amdgcn_s_barrier();
      }
    } else {
      f32x16 dk[MT], dv[MT];
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk[i][r] = 0.f; dv[i][r] = 0.f; }
      DL_WAIT_VM0;
      __builtin_amdgcn_s_barrier();
      for (int ph = 0; ph <= n_ph; ++ph) {
        const int t = ph >> 1, mt = ph & 1;
        if (mt == 0 && t + 1 < n_steps) issue(qt0 + t + 1, (t + 1) % 3);
        const int pp = ph - 1;  // the phase the producer finished before the last barrier
        if (pp >= 0 && q_lo_of(pp) + 31 >= k0) {
          const int st = (pp >> 1) % 3, mp = pp & 1;
          const char *Qt = smem + st * STAGE_B + mp * 8192, *Gt = Qt + TILE_B;
          const u32x4 *X = reinterpret_cast<const u32x4 *>(smem + DKV_XCH_OFF + ((pp & 1) * 4 + wk) * 4096);
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2) {
            const bf16x8 pf = __builtin_bit_cast(bf16x8, X[t2 * 64 + lane]), df = __builtin_bit_cast(bf16x8, X[128 + t2 * 64 + lane]);
#pragma unroll
            for (int i = 0; i < MT; ++i) {
              dv[i] = MFMA(frag_tr(Gt + 16 * t2 * 256, ro.ta[i], ro.tb[i]), pf, dv[i]);
              dk[i] = MFMA(frag_tr(Qt + 16 * t2 * 256, ro.ta[i], ro.tb[i]), df, dk[i]);
            }
          }
        }
        if (mt) DL_WAIT_VM0;
        DL_WAIT_LGKM0;  // every LDS read of the phase has returned before the stage and the hand-over area are released
        __builtin_amdgcn_s_barrier();
      }
      if (rope) rope_grad(dk, rope, kv, g);
      uint16_t *op = dqkv + ((int64_t)b * N + kv) * ld + (int64_t)h * DH;
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          u32x2 wkk = {pack2(dk[i][4 * j], dk[i][4 * j + 1]), pack2(dk[i][4 * j + 2], dk[i][4 * j + 3])};
          u32x2 wv = {pack2(dv[i][4 * j], dv[i][4 * j + 1]), pack2(dv[i][4 * j + 2], dv[i][4 * j + 3])};
          *reinterpret_cast<u32x2 *>(op + HD + i * 32 + 8 * j + 4 * g) = wkk;
          *reinterpret_cast<u32x2 *>(op + 2 * HD + i * 32 + 8 * j + 4 * g) = wv;
        }
    }
    __builtin_amdgcn_s_barrier();  // the next item's first loads overwrite stage 0
  }
}

}  // namespace dl

// the pipelined kernels address a whole batch element through one 32-bit buffer range
bool dl_ok(const twist_ctx *ctx, int N, int Hs, int dh) {
  return !ctx->staged_attention && (int64_t)N * 3 * Hs * dh * 2 < (1ll << 31);
}

bool shape_ok(const void *a, const void *b, int N, int Hs, int dh) {
  (void)Hs;
  return (dh == 64 || dh == 128) && N % 128 == 0 && (reinterpret_cast<uintptr_t>(a) % 16) == 0 && (reinterpret_cast<uintptr_t>(b) % 16) == 0;
}

}  // namespace

twist_status twist_attention_fwd_mfma(twist_ctx *ctx, const void *qkv, void *o, float *o32, float *lse, int B, int N, int Hs, int dh, const int32_t *keep,
                                      bool *done) {
  const bool off = ctx->plain_only;
  *done = false;
  if (off || !shape_ok(qkv, o, N, Hs, dh)) return TWIST_OK;
  const float scale = 1.0f / sqrtf((float)dh);
  dim3 grid((unsigned)((int64_t)(N / 128) * B * Hs)), block(256);
  const uint16_t *x = static_cast<const uint16_t *>(qkv);
  if (dh == 128 && dl_ok(ctx, N, Hs, dh)) hipLaunchKernelGGL(dl::flash_fwd_dl_kernel, grid, block, 0, ctx->stream, x, static_cast<uint16_t *>(o), o32, lse, N, Hs, scale, keep);
  else if (dh == 128) hipLaunchKernelGGL(flash_fwd_kernel<128>, grid, block, 0, ctx->stream, x, static_cast<uint16_t *>(o), o32, lse, N, Hs, scale, keep);
  else hipLaunchKernelGGL(flash_fwd_kernel<64>, grid, block, 0, ctx->stream, x, static_cast<uint16_t *>(o), o32, lse, N, Hs, scale, keep);
  TW_HIP(ctx, hipGetLastError());
  *done = true;
  return TWIST_OK;
}

twist_status twist_attention_bwd_mfma(twist_ctx *ctx, const void *qkv, const float *o32, const void *dout, const float *lse, float *delta, void *dqkv,
                                      int B, int N, int Hs, int dh, const float *rope_tab, const int32_t *keep, bool *done, bool *rope_done) {
  const bool off = ctx->plain_only;
  *done = false;
  *rope_done = false;
  if (off || !o32 || !shape_ok(qkv, dout, N, Hs, dh) || (reinterpret_cast<uintptr_t>(dqkv) % 16) || (reinterpret_cast<uintptr_t>(o32) % 16)) return TWIST_OK;
  const float scale = 1.0f / sqrtf((float)dh);
  dim3 grid((unsigned)((int64_t)(N / 128) * B * Hs)), block(256);
  const uint16_t *x = static_cast<const uint16_t *>(qkv), *gout = static_cast<const uint16_t *>(dout);
  uint16_t *dx = static_cast<uint16_t *>(dqkv);
  if (dh == 128 && dl_ok(ctx, N, Hs, dh)) {
    const float *rt = rope_tab && (reinterpret_cast<uintptr_t>(rope_tab) % 16) == 0 ? rope_tab : nullptr;
    hipLaunchKernelGGL(dl::flash_bwd_dq_dl_kernel, grid, block, 0, ctx->stream, x, gout, o32, lse, delta, dx, N, Hs, scale, rt, keep);
    hipLaunchKernelGGL(dl::flash_bwd_dkv_dl_kernel, dim3((unsigned)((int64_t)((N / 128 + 1) / 2) * B * Hs)), dim3(512), 0, ctx->stream, x, gout, lse, delta, dx, N, Hs, scale, rt,
                       keep);
    *rope_done = rt != nullptr;
  } else if (dh == 128) {
    hipLaunchKernelGGL(flash_bwd_dq_kernel<128>, grid, block, 0, ctx->stream, x, gout, o32, lse, delta, dx, N, Hs, scale, keep);
    hipLaunchKernelGGL(flash_bwd_dkv_kernel<128>, grid, block, 0, ctx->stream, x, gout, lse, delta, dx, N, Hs, scale, keep);
  } else {
    hipLaunchKernelGGL(flash_bwd_dq_kernel<64>, grid, block, 0, ctx->stream, x, gout, o32, lse, delta, dx, N, Hs, scale, keep);
    hipLaunchKernelGGL(flash_bwd_dkv_kernel<64>, grid, block, 0, ctx->stream, x, gout, lse, delta, dx, N, Hs, scale, keep);
  }
  TW_HIP(ctx, hipGetLastError());
  *done = true;
  return TWIST_OK;
}
