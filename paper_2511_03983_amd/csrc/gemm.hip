// Dense projections of the subnet: C = epilogue(op(A) op(B)) with fp32 accumulation.
//  - bf16 operands: MFMA kernel (v_mfma_f32_32x32x16_bf16), 128x128x32 workgroup tile, 4 waves of 64x64,
//    operands staged through LDS as [row][k] so that each lane reads its 8 consecutive k values in one
//    16-byte LDS load; operands whose memory layout has k as the slow axis are transposed while staging.
//  - anything else (fp32 models, unaligned shapes): a plain tiled FMA kernel with arbitrary strides.
#include "nn.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf2f(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

struct Ep {
  float alpha;
  const void *bias;
  const float *residual;
  void *out;
  int out_f32;
  int64_t ldc;
};

template <int BF>
__device__ __forceinline__ void store_out(const Ep &ep, int m, int n, float acc) {
  float v = acc;
  if (ep.bias) v += BF ? bf2f(static_cast<const uint16_t *>(ep.bias)[n]) : static_cast<const float *>(ep.bias)[n];
  v *= ep.alpha;
  const int64_t i = (int64_t)m * ep.ldc + n;
  if (ep.residual) v += ep.residual[i];
  if (ep.out_f32) static_cast<float *>(ep.out)[i] = v;
  else if (BF) static_cast<uint16_t *>(ep.out)[i] = f2bf(v);
  else static_cast<float *>(ep.out)[i] = v;
}

// ------------------------------------------------------------------------------------------- plain kernel
template <int BF>
__global__ __launch_bounds__(256) void gemm_plain_kernel(int M, int N, int K, const void *A, int64_t sam, int64_t sak, const void *B, int64_t sbk,
                                                         int64_t sbn, Ep ep) {
  __shared__ float As[16][65], Bs[16][65];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  auto ld = [](const void *p, int64_t i) -> float {
    return BF ? bf2f(static_cast<const uint16_t *>(p)[i]) : static_cast<const float *>(p)[i];
  };
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 1024; i += 256) {
      int r = i >> 4, k = i & 15;
      As[k][r] = (m0 + r < M && k0 + k < K) ? ld(A, (int64_t)(m0 + r) * sam + (int64_t)(k0 + k) * sak) : 0.f;
      Bs[k][r] = (n0 + r < N && k0 + k < K) ? ld(B, (int64_t)(k0 + k) * sbk + (int64_t)(n0 + r) * sbn) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) store_out<BF>(ep, m, n, acc[i][j]);
    }
}

// ------------------------------------------------------------------------------------------- MFMA kernel
constexpr int BM = 128, BN = 128, BK = 32, LDS_LD = BK + 8;  // padded row: 80 bytes, conflict-free 16-byte reads
constexpr int kChunks = BM * BK / 8 / 256;                  // 16-byte chunks each thread stages per tile
constexpr int kKC = BK / 8;                                 // chunks along k per row

// Stage a [128 rows][64 k] operand tile into LDS (row-major, k contiguous).
//  KMAJOR = 1: memory is [row][k]  (k contiguous): 16-byte copies.
//  KMAJOR = 0: memory is [k][row]  (row contiguous): 16-byte loads, transposed 2-byte LDS writes.
template <int KMAJOR>
struct TileLoader {
  u32x4 reg[kChunks];
  __device__ __forceinline__ void load(const uint16_t *src, int64_t ld, int row0, int k0, int rows, int K) {
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int c = threadIdx.x + 256 * i;
      reg[i] = u32x4{0, 0, 0, 0};
      if (KMAJOR) {
        const int r = c / kKC, kc = (c % kKC) * 8;
        if (row0 + r < rows && k0 + kc < K) reg[i] = *reinterpret_cast<const u32x4 *>(src + (int64_t)(row0 + r) * ld + k0 + kc);
      } else {
        const int k = c >> 4, rc = (c & 15) * 8;
        if (k0 + k < K && row0 + rc < rows) {
          const uint16_t *p = src + (int64_t)(k0 + k) * ld + row0 + rc;
          if (row0 + rc + 8 <= rows) reg[i] = *reinterpret_cast<const u32x4 *>(p);
          else {  // ragged edge: element-wise
            uint16_t t[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int j = 0; j < 8; ++j)
              if (row0 + rc + j < rows) t[j] = p[j];
            reg[i] = u32x4{(uint32_t)t[0] | ((uint32_t)t[1] << 16), (uint32_t)t[2] | ((uint32_t)t[3] << 16),
                           (uint32_t)t[4] | ((uint32_t)t[5] << 16), (uint32_t)t[6] | ((uint32_t)t[7] << 16)};
          }
        }
      }
    }
  }
  __device__ __forceinline__ void store(uint16_t *lds) const {
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int c = threadIdx.x + 256 * i;
      if (KMAJOR) {
        const int r = c / kKC, kc = (c % kKC) * 8;
        *reinterpret_cast<u32x4 *>(lds + r * LDS_LD + kc) = reg[i];
      } else {
        const int k = c >> 4, rc = (c & 15) * 8;
        const uint32_t w[4] = {reg[i].x, reg[i].y, reg[i].z, reg[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          lds[(rc + 2 * j) * LDS_LD + k] = (uint16_t)(w[j] & 0xffff);
          lds[(rc + 2 * j + 1) * LDS_LD + k] = (uint16_t)(w[j] >> 16);
        }
      }
    }
  }
};

// A operand: rows = M index; B operand: rows = N index.  AK / BK_ say whether k is contiguous in memory.
template <int AK, int BK_>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(int M, int N, int K, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, Ep ep,
                                                        int tiles_n) {
  __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * LDS_LD];
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const int lr = lane & 31, lk = (lane >> 5) * 8;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  TileLoader<AK> la;
  TileLoader<BK_> lb;
  la.load(A, lda, m0, 0, M, K);
  lb.load(B, ldb, n0, 0, N, K);
  la.store(As[0]);
  lb.store(Bs[0]);
  __syncthreads();
  const int nk = (K + BK - 1) / BK;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      la.load(A, lda, m0, (kt + 1) * BK, M, K);
      lb.load(B, ldb, n0, (kt + 1) * BK, N, K);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[2], bfr[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = *reinterpret_cast<const bf16x8 *>(As[cur] + (wm + i * 32 + lr) * LDS_LD + ks * 16 + lk);
        bfr[i] = *reinterpret_cast<const bf16x8 *>(Bs[cur] + (wn + i * 32 + lr) * LDS_LD + ks * 16 + lk);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      la.store(As[cur ^ 1]);
      lb.store(Bs[cur ^ 1]);
    }
    __syncthreads();
  }
  // accumulator layout of a 32x32 tile: column = lane % 32, row = 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn + j * 32 + lr;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < M && n < N) store_out<1>(ep, m, n, acc[i][j][r]);
      }
    }
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

twist_status twist_gemm(twist_ctx *ctx, int bf16, GemmLayout lay, int M, int N, int K, const void *A, int64_t lda, const void *B, int64_t ldb,
                        int64_t ldc, const GemmEpilogue &e) {
  if (M <= 0 || N <= 0 || K <= 0) return TWIST_OK;
  hipEvent_t ev_stop = nullptr;
  if (ctx->prof_gemm) {
    hipEvent_t ev_start;
    TW_HIP(ctx, hipEventCreate(&ev_start));
    TW_HIP(ctx, hipEventCreate(&ev_stop));
    ctx->prof_events.push_back(ev_start);
    ctx->prof_events.push_back(ev_stop);
    ctx->prof_flops += 2.0 * M * N * K;
    TW_HIP(ctx, hipEventRecord(ev_start, ctx->stream));
  }
  struct StopRecorder {  // records the closing event on every return path
    twist_ctx *c; hipEvent_t e;
    ~StopRecorder() { if (e) (void)hipEventRecord(e, c->stream); }
  } stop_recorder{ctx, ev_stop};
  Ep ep{e.alpha, e.bias, e.residual, e.out, e.out_f32, ldc};
  static const bool no_mfma = getenv("TWIST_NO_MFMA") != nullptr;
  // 16-byte chunks along k must not straddle the end of an operand row.  For y = x W with a ragged K the
  // caller pads x's rows (lda >= K rounded up to 8) with zeros; W's rows beyond K are never touched.
  const bool k_ok = lay == GEMM_TN || K % 8 == 0 || (lay == GEMM_NN && lda >= (K + 7) / 8 * 8);
  const bool vec_ok = bf16 && !no_mfma && aligned16(A) && aligned16(B) && lda % 8 == 0 && ldb % 8 == 0 && k_ok;
  if (vec_ok) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const size_t smem = 0;
    const uint16_t *a = static_cast<const uint16_t *>(A), *b = static_cast<const uint16_t *>(B);
    dim3 grid(tiles_m * tiles_n), block(256);
    switch (lay) {
      case GEMM_NT: hipLaunchKernelGGL((gemm_mfma_kernel<1, 1>), grid, block, smem, ctx->stream, M, N, K, a, lda, b, ldb, ep, tiles_n); break;
      case GEMM_NN: hipLaunchKernelGGL((gemm_mfma_kernel<1, 0>), grid, block, smem, ctx->stream, M, N, K, a, lda, b, ldb, ep, tiles_n); break;
      case GEMM_TN: hipLaunchKernelGGL((gemm_mfma_kernel<0, 0>), grid, block, smem, ctx->stream, M, N, K, a, lda, b, ldb, ep, tiles_n); break;
    }
    TW_HIP(ctx, hipGetLastError());
    return TWIST_OK;
  }
  int64_t sam, sak, sbk, sbn;
  switch (lay) {
    case GEMM_NT: sam = lda; sak = 1; sbk = 1; sbn = ldb; break;
    case GEMM_NN: sam = lda; sak = 1; sbk = ldb; sbn = 1; break;
    default: sam = 1; sak = lda; sbk = ldb; sbn = 1; break;
  }
  dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
  if (bf16) hipLaunchKernelGGL(gemm_plain_kernel<1>, grid, block, 0, ctx->stream, M, N, K, A, sam, sak, B, sbk, sbn, ep);
  else hipLaunchKernelGGL(gemm_plain_kernel<0>, grid, block, 0, ctx->stream, M, N, K, A, sam, sak, B, sbk, sbn, ep);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

extern "C" twist_status twist_profile_gemm(twist_ctx *ctx, int32_t enable) {
  if (!ctx) TW_FAIL(nullptr, TWIST_EINVAL, "twist_profile_gemm: null ctx");
  TW_HIP(ctx, hipStreamSynchronize(ctx->stream));
  for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
  ctx->prof_events.clear();
  ctx->prof_flops = 0.0;
  ctx->prof_gemm = enable != 0;
  return TWIST_OK;
}

extern "C" twist_status twist_profile_gemm_read(twist_ctx *ctx, int64_t *launches, double *ms, double *flops) {
  if (!ctx || !launches || !ms || !flops) TW_FAIL(ctx, TWIST_EINVAL, "twist_profile_gemm_read: null argument");
  TW_HIP(ctx, hipStreamSynchronize(ctx->stream));
  double total = 0.0;
  for (size_t i = 0; i + 1 < ctx->prof_events.size(); i += 2) {
    float t = 0.f;
    TW_HIP(ctx, hipEventElapsedTime(&t, ctx->prof_events[i], ctx->prof_events[i + 1]));
    total += t;
  }
  *launches = (int64_t)(ctx->prof_events.size() / 2);
  *ms = total;
  *flops = ctx->prof_flops;
  for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
  ctx->prof_events.clear();
  ctx->prof_flops = 0.0;
  return TWIST_OK;
}
