// Dense projections of the subnet: C = epilogue(op(A) op(B)) with fp32 accumulation.
//  - bf16 operands: MFMA kernels (v_mfma_f32_32x32x16_bf16): a 256x256 ping-pong kernel fed by direct-to-LDS
//    loads for all but the smallest products, and a 128x128 register-staged kernel; operands stay in LDS in their
//    memory orientation, and those whose contraction index is the slow axis in memory are read back with the
//    transposing LDS load.
//  - anything else (fp32 models, unaligned shapes): a plain tiled FMA kernel with arbitrary strides.
#include <algorithm>

#include "nn.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf2f(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
// two floats to a packed pair of bf16, round to nearest even, in one instruction (v_cvt_pk_bf16_f32): the same bits as f2bf for
// every finite value and infinity (the software form costs about eight instructions and a branch per value, which showed in
// the epilogue: 40.6 -> 39.9 ms per forward+backward pass)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
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
  int vec_ok;  // out (and residual) rows allow 4-element vector accesses: ldc % 4 == 0, 16-byte aligned bases
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
// Workgroup tile BM x BN x 32, WM x WN waves, each wave (BM/WM) x (BN/WN) in 32x32 MFMA tiles.
// An operand tile lives in LDS in the orientation of its memory:
//   k contiguous in memory ("KMAJOR"):  LDS [rows][32 + 8]; a lane's 8 k values are one 16-byte LDS read;
//   rows contiguous in memory:          LDS [32][rows + 16]; a lane's 8 k values are two transposing reads
//                                       (ds_read_tr16_b64: 4 consecutive k rows of one column each).
// Both paddings make the reads bank-conflict free.  Tiles are double-buffered: the next tile's global loads
// are issued before the MFMAs of the current one and written to the other buffer after them, one barrier per
// k-iteration.  Workgroups are renumbered so that each of the 8 XCDs (own L2) works on a contiguous range
// of tiles.
constexpr int BK = 64;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr uint32_t kOob = 0x80000000u;  // byte offset beyond every buffer: loads return 0, stores are dropped

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}

// Global accesses go through buffer instructions whose hardware range check returns zeros (loads) or drops the
// access (stores) beyond the end, so tile edges need no branches: an out-of-range row or k chunk just gets an
// offset outside the buffer.
template <int ROWS, int KMAJOR, int NT>
struct TileLoader {
  static constexpr int LD = KMAJOR ? BK + 8 : ROWS + 16;
  static constexpr int ELEMS = KMAJOR ? ROWS * LD : BK * LD;
  static constexpr int CHUNKS = ROWS * BK / 8 / NT;       // 16-byte chunks per thread
  static constexpr int CPR = KMAJOR ? BK / 8 : ROWS / 8;  // chunks per stored row
  u32x4 reg[CHUNKS];
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t off[CHUNKS];  // byte offset of each chunk at k0 = 0 (kOob if its row is outside the operand)
  int kk[CHUNKS];        // k of the chunk inside a tile
  uint32_t kstep;        // bytes to advance per k-tile
  // base = first row of this workgroup's panel (KMAJOR) or first column (otherwise)
  __device__ __forceinline__ void init(const uint16_t *base, int64_t ld, int rows_left, int K) {
    const int64_t span = KMAJOR ? ((int64_t)(min(rows_left, ROWS) - 1) * ld + K) : ((int64_t)(K - 1) * ld + min(rows_left, (int)ld));
    rsrc = make_rsrc(base, (uint32_t)(span * 2));
    kstep = KMAJOR ? BK * 2 : (uint32_t)(BK * ld * 2);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int c = threadIdx.x + NT * i;
      if (KMAJOR) {
        const int r = c / CPR, kc = (c % CPR) * 8;
        kk[i] = kc;
        off[i] = r < rows_left ? (uint32_t)((r * ld + kc) * 2) : kOob;
      } else {
        const int k = c / CPR, rc = (c % CPR) * 8;
        kk[i] = k;
        off[i] = rc < rows_left ? (uint32_t)((k * ld + rc) * 2) : kOob;
      }
    }
  }
  __device__ __forceinline__ void load(int kt, int K) {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const uint32_t o = (kt * BK + kk[i] < K) ? off[i] + kt * kstep : kOob;
      reg[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, o, 0, 0);
    }
  }
  __device__ __forceinline__ void store(uint16_t *lds) const {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int c = threadIdx.x + NT * i;
      const int r = c / CPR, kc = (c % CPR) * 8;  // (row, k chunk) or (k row, row chunk): same arithmetic
      *reinterpret_cast<u32x4 *>(lds + r * LD + kc) = reg[i];
    }
  }
  // fragment for the 32 rows starting at row0 of the tile, k-step ks (16 wide)
  static __device__ __forceinline__ bf16x8 frag(const uint16_t *lds, int row0, int ks) {
    const int lane = threadIdx.x & 63;
    if (KMAJOR) return *reinterpret_cast<const bf16x8 *>(lds + (row0 + (lane & 31)) * LD + ks * 16 + (lane >> 5) * 8);
    const int s = lane & 15;
    const uint16_t *p = lds + (ks * 16 + (lane >> 5) * 8 + (s >> 2)) * LD + row0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * LD));
    s16x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
};

// A operand: rows = M index; B operand: rows = N index.  AKM / BKM say whether k is contiguous in memory.
template <int AKM, int BKM, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64) void gemm_mfma_kernel(int M, int N, int K, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                                                                Ep ep, int tiles_m, int tiles_n) {
  constexpr int NT = WM * WN * 64, TM = BM / WM / 32, TN = BN / WN / 32, KS = BK / 16;
  using LA = TileLoader<BM, AKM, NT>;
  using LB = TileLoader<BN, BKM, NT>;
  __shared__ __attribute__((aligned(16))) uint16_t As[2][LA::ELEMS];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][LB::ELEMS];
  // XCD-aware renumbering: hardware deals workgroup ids round-robin over 8 XCDs
  const int nb = tiles_m * tiles_n;
  int bid = blockIdx.x;
  if (nb % 8 == 0) bid = (bid % 8) * (nb / 8) + bid / 8;
  // walk the tiles in column-panels of 8 tile rows so that concurrently running workgroups share operands
  constexpr int GROUP = 8;
  const int per_group = GROUP * tiles_n;
  const int grp = bid / per_group, first_m = grp * GROUP;
  const int gsize = min(GROUP, tiles_m - first_m);
  const int tile_m = first_m + (bid % per_group) % gsize, tile_n = (bid % per_group) / gsize;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = (wave / WN) * (BM / WM), wn = (wave % WN) * (BN / WN);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  LA la;
  LB lb;
  la.init(AKM ? A + (int64_t)m0 * lda : A + m0, lda, M - m0, K);
  lb.init(BKM ? B + (int64_t)n0 * ldb : B + n0, ldb, N - n0, K);
  // Pipeline: tile kt+2 travels from global memory to registers and tile kt+1 from registers to LDS while
  // tile kt is multiplied; one barrier per k-iteration.
  la.load(0, K);
  lb.load(0, K);
  la.store(As[0]);
  lb.store(Bs[0]);
  const int nk = (K + BK - 1) / BK;
  if (nk > 1) {
    la.load(1, K);
    lb.load(1, K);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      la.store(As[cur ^ 1]);
      lb.store(Bs[cur ^ 1]);
    }
    if (kt + 2 < nk) {
      la.load(kt + 2, K);
      lb.load(kt + 2, K);
    }
    // fragments of k-step ks+1 are fetched while the MFMAs of k-step ks run
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = LA::frag(As[cur], wm + i * 32, 0);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = LB::frag(Bs[cur], wn + j * 32, 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) {
#pragma unroll
        for (int i = 0; i < TM; ++i) af[(ks + 1) & 1][i] = LA::frag(As[cur], wm + i * 32, ks + 1);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[(ks + 1) & 1][j] = LB::frag(Bs[cur], wn + j * 32, ks + 1);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // Epilogue.  A 32x32 accumulator tile holds column lane % 32 and rows 8*(r/4) + 4*(lane/32) + r%4, which would store
  // 2-byte pieces; each wave instead turns its results through LDS (the operand stages are free now), 32 rows at a time,
  // so that a lane owns 4 consecutive columns and a store instruction writes four rows of 64 columns.
  static_assert(TN == 2 && sizeof(As) >= WM * WN * 32 * 72 * 4, "staging of 32 x 64 results per wave fits the A stages");
  constexpr int LDE = 72;  // floats per staged row: rows 4 apart (the two half-waves of a write) are 32 banks apart
  float *stage = reinterpret_cast<float *>(&As[0][0]) + wave * (32 * LDE);
  const int c = lane & 31, g = lane >> 5, c16 = lane & 15, rs = lane >> 4;
  const int rows_left = M - m0;
  const int ncol = n0 + wn + 4 * c16;  // first of this lane's 4 columns
  float bias[4] = {0.f, 0.f, 0.f, 0.f};
  if (ep.bias) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (ncol + e < N) bias[e] = bf2f(static_cast<const uint16_t *>(ep.bias)[ncol + e]);
  }
  const bool vec = ep.vec_ok && ncol + 3 < N;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[(8 * (r >> 2) + 4 * g + (r & 3)) * LDE + 32 * j + c] = acc[i][j][r];
#pragma unroll 4
    for (int p = 0; p < 8; ++p) {
      const int row = 4 * p + rs, ml = wm + 32 * i + row;
      const f32x4 v4 = *reinterpret_cast<const f32x4 *>(stage + row * LDE + 4 * c16);
      if (ml >= rows_left || ncol >= N) continue;
      const int64_t o = (int64_t)(m0 + ml) * ep.ldc + ncol;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (v4[e] + bias[e]) * ep.alpha;
      if (vec) {
        if (ep.residual) {
          const f32x4 rr = *reinterpret_cast<const f32x4 *>(ep.residual + o);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += rr[e];
        }
        if (ep.out_f32) {
          const f32x4 w = {v[0], v[1], v[2], v[3]};
          *reinterpret_cast<f32x4 *>(static_cast<float *>(ep.out) + o) = w;
        } else {
          const u32x2 w = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
          *reinterpret_cast<u32x2 *>(static_cast<uint16_t *>(ep.out) + o) = w;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (ncol + e >= N) break;
          float x = v[e];
          if (ep.residual) x += ep.residual[o + e];
          if (ep.out_f32) static_cast<float *>(ep.out)[o + e] = x;
          else static_cast<uint16_t *>(ep.out)[o + e] = f2bf(x);
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------- ping-pong MFMA kernel
// 256x256 workgroup tile, 8 waves of 64x128, k walked in sub-tiles of 32.  The eight waves form two groups of
// four (one wave of each group per SIMD) that run the same loop one phase apart: while one group issues the
// 16 MFMAs of a sub-tile, the other reads its fragments of the next sub-tile from LDS and starts the global
// loads three sub-tiles ahead, so the matrix pipe of every SIMD always has a wave feeding it.
// Global loads go straight to LDS (buffer_load_dwordx4 ... lds: lane l of a wave writes 16 bytes at
// base + 16 l), four stages of 32 KB.  Because that write pattern is fixed, bank conflicts are avoided by
// permuting which 16-byte chunk of a row each lane fetches (an XOR swizzle) instead of by padding:
//   k contiguous in memory:    LDS [256 rows][4 chunks];  chunk c of row r sits at position c ^ ((r >> 2) & 3)
//   rows contiguous in memory: LDS [32 k][32 chunks];     chunk c of k-row k sits at position c ^ (4 (k & 3))
namespace pp {

constexpr int SK = 32;             // k extent of a sub-tile
constexpr int OPB = 256 * SK * 2;  // bytes of one operand's sub-tile
constexpr int STG = 2 * OPB;       // one stage: A sub-tile, then B sub-tile
constexpr int NST = 4;
typedef __attribute__((address_space(3))) void *lds_void;

#define PP_WAIT_VM8_LGKM0 __builtin_amdgcn_s_waitcnt(0x0078)  // vmcnt(8) lgkmcnt(0)
#define PP_WAIT_VM0 __builtin_amdgcn_s_waitcnt(0x0f70)        // vmcnt(0)

template <int KM>
struct Loader {
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t off[2];  // byte offset of the lane's chunk in sub-tile 0 (kOob: outside the operand)
  int kk[2];        // k of that chunk inside a sub-tile
  uint32_t kstep;   // bytes from one sub-tile to the next
  __device__ __forceinline__ void init(const uint16_t *base, int64_t ld, int rows_left, int K, int wave, int lane) {
    const int64_t span = KM ? ((int64_t)(min(rows_left, 256) - 1) * ld + K) : ((int64_t)(K - 1) * ld + min(rows_left, (int)ld));
    rsrc = make_rsrc(base, (uint32_t)(span * 2));
    kstep = KM ? SK * 2 : (uint32_t)(SK * ld * 2);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int j = wave + 8 * i;  // which of the 16 one-KB pieces of the sub-tile
      if (KM) {
        const int r = 16 * j + (lane >> 2), c = (lane & 3) ^ ((r >> 2) & 3);
        kk[i] = c * 8;
        off[i] = r < rows_left ? (uint32_t)((r * ld + c * 8) * 2) : kOob;
      } else {
        const int k = 2 * j + (lane >> 5), c = (lane & 31) ^ (4 * (k & 3));
        kk[i] = k;
        off[i] = c * 8 < rows_left ? (uint32_t)((k * ld + c * 8) * 2) : kOob;
      }
    }
  }
  // start the loads of sub-tile u into the operand's 16 KB at dst (wave-uniform)
  __device__ __forceinline__ void issue(int u, int K, char *dst, int wave) const {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t o = (u * SK + kk[i] < K) ? off[i] + u * kstep : kOob;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void)(dst + (wave + 8 * i) * 1024), 16, o, 0, 0, 0);
    }
  }
};

// Per-lane LDS byte offsets (inside an operand's sub-tile) of the fragment reads of a wave whose rows start at wb.
template <int KM, int NTILE>
struct Frags {
  uint32_t a[KM ? 2 : NTILE];
  __device__ __forceinline__ void init(int wb, int lane) {
    const int c = lane & 31, g = lane >> 5, s = lane & 15, hi = (lane >> 4) & 1;
    if (KM) {
      a[0] = (uint32_t)((wb + c) * 64 + ((g ^ ((c >> 2) & 3)) * 16));
      a[1] = a[0] ^ 32u;
    } else {
#pragma unroll
      for (int i = 0; i < NTILE; ++i) {
        const int chunk = (wb >> 3) + 4 * i + 2 * hi + ((s >> 1) & 1);
        a[i] = (uint32_t)((g * 8 + (s >> 2)) * 512 + ((chunk ^ (4 * ((s >> 2) & 3))) * 16) + (s & 1) * 8);
      }
    }
  }
  // fragment of tile i (32 rows), k-step ks (16 wide) from the operand sub-tile at p
  __device__ __forceinline__ bf16x8 get(const char *p, int i, int ks) const {
    if (KM) return *reinterpret_cast<const bf16x8 *>(p + a[ks] + i * 2048);
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const char *q = p + a[i] + ks * 8192;
    s16x4 x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(q));
    s16x4 y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(q + 2048));
    s16x8 v = {x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
    return __builtin_bit_cast(bf16x8, v);
  }
};

// SPLIT: the k range is cut into `ksplit` parts of `kchunk` (a multiple of 32) and a work item is (part, tile); part p
// writes its unscaled fp32 partial product to ep.out + p * M * ldc and splitk_reduce_kernel adds the parts.  Used for
// products with few output tiles and a long k (weight gradients), which would otherwise occupy a fraction of the CUs.
template <int AKM, int BKM, bool SPLIT>
__global__ __launch_bounds__(512) void gemm_pp_kernel(int M, int N, int K, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, Ep ep,
                                                      int tiles_m, int tiles_n, int ksplit, int kchunk) {
  constexpr int TM = 2, TN = 4;
  constexpr int EPI_LD = 136;                    // floats per staged output row: 4 rows apart = 32 banks apart
  constexpr int EPI_WAVE = 32 * EPI_LD * 4;      // one wave's 32 x 128 block of fp32 results
  constexpr int SMEM = NST * STG > 8 * EPI_WAVE ? NST * STG : 8 * EPI_WAVE;
  __shared__ __attribute__((aligned(1024))) char smem[SMEM];
  const int nb = tiles_m * tiles_n;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wpos = wave & 3, half = wave >> 2;  // waves w and w+4 share a SIMD and sit in different groups
  const int wm = (wpos >> 1) * 128 + half * 64, wn = (wpos & 1) * 128;
  Frags<AKM, TM> fa;
  Frags<BKM, TN> fb;
  fa.init(wm, lane);
  fb.init(wn, lane);
  // Persistent workgroups: each walks the tiles vid, vid + gridDim.x, ...; the stores of one tile drain while the
  // next tile's loads are already under way.  Tile numbers are dealt so that each of the 8 XCDs (own L2; workgroup
  // b runs on XCD b % 8) works on a contiguous range of tiles.
  const int n_items = SPLIT ? nb * ksplit : nb;
  for (int vid = blockIdx.x; vid < n_items; vid += gridDim.x) {
  const int part = SPLIT ? vid / nb : 0;
  int bid = SPLIT ? vid - part * nb : vid;
  if (nb % 8 == 0) bid = (bid % 8) * (nb / 8) + bid / 8;
  const int kbeg = SPLIT ? part * kchunk : 0;
  const int Kl = SPLIT ? min(kchunk, K - kbeg) : K;  // this item's k extent
  constexpr int GROUP = 8;
  const int per_group = GROUP * tiles_n;
  const int grp = bid / per_group, first_m = grp * GROUP;
  const int gsize = min(GROUP, tiles_m - first_m);
  const int tile_m = first_m + (bid % per_group) % gsize, tile_n = (bid % per_group) / gsize;
  const int m0 = tile_m * 256, n0 = tile_n * 256;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  Loader<AKM> la;
  Loader<BKM> lb;
  la.init(AKM ? A + (int64_t)m0 * lda + kbeg : A + (int64_t)kbeg * lda + m0, lda, M - m0, Kl, wave, lane);
  lb.init(BKM ? B + (int64_t)n0 * ldb + kbeg : B + (int64_t)kbeg * ldb + n0, ldb, N - n0, Kl, wave, lane);

  const int nsub = (Kl + SK - 1) / SK;
#pragma unroll
  for (int u = 0; u < NST - 1; ++u) {
    la.issue(u, Kl, smem + u * STG, wave);
    lb.issue(u, Kl, smem + u * STG + OPB, wave);
  }
  PP_WAIT_VM8_LGKM0;  // sub-tile 0 has landed (4 loads per sub-tile and wave)
  __builtin_amdgcn_s_barrier();
  if (half) __builtin_amdgcn_s_barrier();  // the second group runs one phase late
  for (int u = 0; u < nsub; ++u) {
    const char *sa = smem + (u & (NST - 1)) * STG, *sb = sa + OPB;
    char *dn = smem + ((u + NST - 1) & (NST - 1)) * STG;
    __builtin_amdgcn_sched_barrier(0);
    // memory phase: fragments of sub-tile u; global loads of sub-tile u + 3 into the stage both groups left last
    // phase (beyond the last sub-tile the loads are out of range and just zero-fill)
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i) af[ks][i] = fa.get(sa, i, ks);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[ks][j] = fb.get(sb, j, ks);
    }
    la.issue(u + NST - 1, Kl, dn, wave);
    lb.issue(u + NST - 1, Kl, dn + OPB, wave);
    PP_WAIT_VM8_LGKM0;  // own fragments are in registers; own loads of sub-tile u + 1 have landed
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // compute phase
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks][i], bfr[ks][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
  }
  if (!half) __builtin_amdgcn_s_barrier();
  PP_WAIT_VM0;                   // own zero-filling loads beyond the last sub-tile
  __builtin_amdgcn_s_barrier();  // ... and everybody else's: LDS is reused below

  // Epilogue.  A 32x32 accumulator tile holds column lane % 32 and rows 8*(r/4) + 4*(lane/32) + r%4, which
  // would store 2-byte pieces; each wave instead turns its results through LDS, 32 rows at a time, so that a
  // lane owns 4 consecutive columns and a store instruction writes two full rows of 128 columns.
  float *stage = reinterpret_cast<float *>(smem + wave * EPI_WAVE);
  const int c = lane & 31, g = lane >> 5;
  const int rows_left = M - m0;
  void *const outp = SPLIT ? static_cast<void *>(static_cast<float *>(ep.out) + (int64_t)part * M * ep.ldc) : ep.out;
  const int ncol = n0 + wn + 4 * c;  // first of this lane's 4 columns
  float bias[4] = {0.f, 0.f, 0.f, 0.f};
  if (ep.bias) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (ncol + e < N) bias[e] = bf2f(static_cast<const uint16_t *>(ep.bias)[ncol + e]);
  }
  const bool vec = ep.vec_ok && ncol + 3 < N;
  // a tile that lies inside the output and needs nothing but the conversion (most projections): no edge tests, no arithmetic
  const bool bare = ep.vec_ok && !ep.bias && !ep.residual && ep.alpha == 1.f && m0 + 256 <= M && n0 + 256 <= N;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[(8 * (r >> 2) + 4 * g + (r & 3)) * EPI_LD + 32 * j + c] = acc[i][j][r];
    if (bare) {
      const int64_t o0 = (int64_t)(m0 + wm + 32 * i + g) * ep.ldc + ncol;
#pragma unroll
      for (int p = 0; p < 16; ++p) {
        const f32x4 v4 = *reinterpret_cast<const f32x4 *>(stage + (2 * p + g) * EPI_LD + 4 * c);
        const int64_t o = o0 + 2 * p * ep.ldc;
        if (ep.out_f32) {
          __builtin_nontemporal_store(v4, reinterpret_cast<f32x4 *>(static_cast<float *>(outp) + o));
        } else {
          const u32x2 w = {pack_bf16(v4[0], v4[1]), pack_bf16(v4[2], v4[3])};
          __builtin_nontemporal_store(w, reinterpret_cast<u32x2 *>(static_cast<uint16_t *>(outp) + o));
        }
      }
      continue;
    }
#pragma unroll 4
    for (int p = 0; p < 16; ++p) {
      const int row = 2 * p + g, ml = wm + 32 * i + row;
      const f32x4 v4 = *reinterpret_cast<const f32x4 *>(stage + row * EPI_LD + 4 * c);
      if (ml >= rows_left || ncol >= N) continue;
      const int64_t o = (int64_t)(m0 + ml) * ep.ldc + ncol;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (v4[e] + bias[e]) * ep.alpha;
      if (vec) {
        if (ep.residual) {
          const f32x4 rr = *reinterpret_cast<const f32x4 *>(ep.residual + o);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += rr[e];
        }
        if (ep.out_f32) {
          const f32x4 w = {v[0], v[1], v[2], v[3]};
          __builtin_nontemporal_store(w, reinterpret_cast<f32x4 *>(static_cast<float *>(outp) + o));
        } else {
          const u32x2 w = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
          __builtin_nontemporal_store(w, reinterpret_cast<u32x2 *>(static_cast<uint16_t *>(outp) + o));
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (ncol + e >= N) break;
          float x = v[e];
          if (ep.residual) x += ep.residual[o + e];
          if (ep.out_f32) static_cast<float *>(outp)[o + e] = x;
          else static_cast<uint16_t *>(outp)[o + e] = f2bf(x);
        }
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's staged results are in registers
  __builtin_amdgcn_s_barrier();        // everybody's are: the next tile's loads may overwrite the staging area
  }
}

}  // namespace pp

// out = alpha * sum over parts of the fp32 partial products [parts][M][N] (parts added in ascending order)
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *ws, int parts, int M, int N, void *out, int64_t ldc, int out_f32, float alpha) {
  const int64_t total = (int64_t)M * N, i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= total) return;
  const bool vec = N % 4 == 0 && ldc % 4 == 0;  // then a group of 4 lies in one row and is 16-byte aligned
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  for (int p = 0; p < parts; ++p) {
    const float *src = ws + (int64_t)p * total + i;
    if (vec) {
      const f32x4 t = *reinterpret_cast<const f32x4 *>(src);
      v[0] += t[0]; v[1] += t[1]; v[2] += t[2]; v[3] += t[3];
    } else {
      for (int e = 0; e < 4 && i + e < total; ++e) v[e] += src[e];
    }
  }
  for (int e = 0; e < 4 && i + e < total; ++e) {
    const int64_t m = (i + e) / N, n = (i + e) - m * N, o = m * ldc + n;
    if (out_f32) static_cast<float *>(out)[o] = alpha * v[e];
    else static_cast<uint16_t *>(out)[o] = f2bf(alpha * v[e]);
  }
}

// Measurement aid: nothing but the projection kernels' matrix instruction, four independent accumulator tiles per wave
// (enough to issue back to back), operands in registers, no loads; the result is stored so that the loop stays.
// random_operands = 0: small constants (few bits toggle between instructions); 1: four different operand pairs of
// pseudo-random bf16 values of magnitude ~1 in rotation, which is what the multipliers see in a real projection and
// what the chip's power limit responds to.
__global__ __launch_bounds__(256) void mfma_only_kernel(int iters, float *sink, int random_operands) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      uint32_t h = (threadIdx.x * 8u + i + 977u * j + 131071u * blockIdx.x) * 2654435761u;
      h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
      // sign and 7 mantissa bits at random, exponent in {2^-2 .. 2^1}: a spread like that of normalised activations
      const uint16_t ra = (uint16_t)(((h & 0x8000u)) | ((125u + ((h >> 7) & 3u)) << 7) | (h & 0x7fu));
      const uint16_t rb = (uint16_t)((((h >> 16) & 0x8000u)) | ((125u + ((h >> 23) & 3u)) << 7) | ((h >> 16) & 0x7fu));
      const uint16_t ca = (uint16_t)(0x3a80u + ((threadIdx.x + i) & 7)), cb = (uint16_t)(0x3b00u + ((threadIdx.x * 3 + i) & 7));
      a[j][i] = __builtin_bit_cast(__bf16, random_operands ? ra : ca);
      b[j][i] = __builtin_bit_cast(__bf16, random_operands ? rb : cb);
    }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; it += 4) {  // four iterations per trip so that the operand rotation is static
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + r) & 3], acc[j], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) t += acc[j][r];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
}

// number of k parts for a product with few 256x256 output tiles and a long k (1 = do not split)
int choose_ksplit(int M, int N, int K, int *kchunk) {
  const int tiles = ((M + 255) / 256) * ((N + 255) / 256);
  *kchunk = K;
  if (tiles >= 128 || K < 1024) return 1;
  int ks = std::min({16, 256 / tiles, K / 512});
  if (ks < 2) return 1;
  *kchunk = ((K + ks - 1) / ks + 31) / 32 * 32;
  return (K + *kchunk - 1) / *kchunk;
}

template <int AKM, int BKM>
void launch_mfma(hipStream_t st, int force_tile, int M, int N, int K, const uint16_t *a, int64_t lda, const uint16_t *b, int64_t ldb, const Ep &ep) {
  // the 256x256 ping-pong kernel (one persistent workgroup per CU) from 128 tiles up (half the chip), else 128x128 tiles
  // (4 waves of 64x64), four times as many, which fill the chip where the big tiles would occupy a third of it (the
  // projections of narrow subnets: 96 big tiles at GPT-2-small quarter width, 5 to 10 % faster this way)
  const int big = ((M + 255) / 256) * ((N + 255) / 256);
  const bool use_big = force_tile ? force_tile == 256 : big >= 128;
  if (use_big) {
    const int tm = (M + 255) / 256, tn = (N + 255) / 256;
    hipLaunchKernelGGL((pp::gemm_pp_kernel<AKM, BKM, false>), dim3(std::min(tm * tn, 256)), dim3(512), 0, st, M, N, K, a, lda, b, ldb, ep, tm, tn, 1, K);
  } else {
    const int tm = (M + 127) / 128, tn = (N + 127) / 128;
    hipLaunchKernelGGL((gemm_mfma_kernel<AKM, BKM, 128, 128, 2, 2>), dim3(tm * tn), dim3(256), 0, st, M, N, K, a, lda, b, ldb, ep, tm, tn);
  }
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

twist_status twist_gemm(twist_ctx *ctx, int bf16, GemmLayout lay, int M, int N, int K, const void *A, int64_t lda, const void *B, int64_t ldb,
                        int64_t ldc, const GemmEpilogue &e, hipStream_t st) {
  if (M <= 0 || N <= 0 || K <= 0) return TWIST_OK;
  const hipStream_t stream = st ? st : ctx->stream;
  hipEvent_t ev_stop = nullptr;
  if (ctx->prof_gemm) {
    hipEvent_t ev_start;
    TW_HIP(ctx, hipEventCreate(&ev_start));
    TW_HIP(ctx, hipEventCreate(&ev_stop));
    ctx->prof_events.push_back(ev_start);
    ctx->prof_events.push_back(ev_stop);
    ctx->prof_flops += 2.0 * M * N * K;
    TW_HIP(ctx, hipEventRecord(ev_start, stream));
  }
  struct StopRecorder {  // records the closing event on every return path
    hipStream_t s; hipEvent_t e;
    ~StopRecorder() { if (e) (void)hipEventRecord(e, s); }
  } stop_recorder{stream, ev_stop};
  Ep ep{e.alpha, e.bias, e.residual, e.out, e.out_f32, ldc, 0};
  ep.vec_ok = ldc % 4 == 0 && aligned16(e.out) && (!e.residual || aligned16(e.residual));
  const bool no_mfma = ctx->plain_only;
  // 16-byte chunks along k must not straddle the end of an operand row.  For y = x W with a ragged K the
  // caller pads x's rows (lda >= K rounded up to 8) with zeros; W's rows beyond K are never touched.
  const bool k_ok = lay == GEMM_TN || K % 8 == 0 || (lay == GEMM_NN && lda >= (K + 7) / 8 * 8);
  // buffer offsets are 32-bit: a row panel (256 rows) or a k-panel (K rows) of each operand and of C must stay below 2 GiB
  const int64_t a_span = (lay == GEMM_TN ? (int64_t)K : 256) * lda * 2, b_span = (lay == GEMM_NT ? 256 : (int64_t)K) * ldb * 2;
  const bool span_ok = a_span < (1ll << 31) && b_span < (1ll << 31) && 256 * ldc * 4 < (1ll << 31);
  const bool vec_ok = bf16 && !no_mfma && aligned16(A) && aligned16(B) && lda % 8 == 0 && ldb % 8 == 0 && k_ok && span_ok;
  if (vec_ok) {
    const uint16_t *a = static_cast<const uint16_t *>(A), *b = static_cast<const uint16_t *>(B);
    int kchunk = K;
    const int ks = (e.splitk_ws && !e.bias && !e.residual && !ctx->gemm_tile) ? choose_ksplit(M, N, K, &kchunk) : 1;
    if (ks > 1 && (size_t)ks * M * N <= e.splitk_floats && aligned16(e.splitk_ws)) {
      const int tm = (M + 255) / 256, tn = (N + 255) / 256;
      Ep part{1.f, nullptr, nullptr, e.splitk_ws, 1, N, N % 4 == 0};
      const dim3 grid(std::min(tm * tn * ks, 256)), block(512);
      switch (lay) {
        case GEMM_NT: hipLaunchKernelGGL((pp::gemm_pp_kernel<1, 1, true>), grid, block, 0, stream, M, N, K, a, lda, b, ldb, part, tm, tn, ks, kchunk); break;
        case GEMM_NN: hipLaunchKernelGGL((pp::gemm_pp_kernel<1, 0, true>), grid, block, 0, stream, M, N, K, a, lda, b, ldb, part, tm, tn, ks, kchunk); break;
        case GEMM_TN: hipLaunchKernelGGL((pp::gemm_pp_kernel<0, 0, true>), grid, block, 0, stream, M, N, K, a, lda, b, ldb, part, tm, tn, ks, kchunk); break;
      }
      TW_HIP(ctx, hipGetLastError());
      const int64_t groups = ((int64_t)M * N + 3) / 4;
      hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, stream, e.splitk_ws, ks, M, N, e.out, ldc, e.out_f32, e.alpha);
      TW_HIP(ctx, hipGetLastError());
      return TWIST_OK;
    }
    switch (lay) {
      case GEMM_NT: launch_mfma<1, 1>(stream, ctx->gemm_tile, M, N, K, a, lda, b, ldb, ep); break;
      case GEMM_NN: launch_mfma<1, 0>(stream, ctx->gemm_tile, M, N, K, a, lda, b, ldb, ep); break;
      case GEMM_TN: launch_mfma<0, 0>(stream, ctx->gemm_tile, M, N, K, a, lda, b, ldb, ep); break;
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
  if (bf16) hipLaunchKernelGGL(gemm_plain_kernel<1>, grid, block, 0, stream, M, N, K, A, sam, sak, B, sbk, sbn, ep);
  else hipLaunchKernelGGL(gemm_plain_kernel<0>, grid, block, 0, stream, M, N, K, A, sam, sak, B, sbk, sbn, ep);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

extern "C" twist_status twist_gemm_raw(twist_ctx *ctx, int32_t layout, int32_t M, int32_t N, int32_t K, const void *A, int64_t lda, const void *B,
                                       int64_t ldb, void *C, int64_t ldc, int32_t out_f32, float alpha) {
  if (!ctx || !A || !B || !C) TW_FAIL(ctx, TWIST_EINVAL, "twist_gemm_raw: null argument");
  if (layout < 0 || layout > 2 || M < 0 || N < 0 || K < 0) TW_FAIL(ctx, TWIST_EINVAL, "twist_gemm_raw: bad layout or size");
  const int64_t need_a = layout == GEMM_TN ? M : K, need_b = layout == GEMM_NT ? K : N;
  if (lda < need_a || ldb < need_b || ldc < N) TW_FAIL(ctx, TWIST_ESHAPE, "twist_gemm_raw: a row stride is smaller than the row it strides");
  GemmEpilogue e;
  e.alpha = alpha;
  e.out = C;
  e.out_f32 = out_f32;
  return twist_gemm(ctx, ctx->d.dtype == TWIST_BF16, (GemmLayout)layout, M, N, K, A, lda, B, ldb, ldc, e);
}

extern "C" twist_status twist_set_overlap(twist_ctx *ctx, int32_t enable) {
  if (!ctx) TW_FAIL(nullptr, TWIST_EINVAL, "twist_set_overlap: null ctx");
  ctx->overlap = enable != 0;
  return TWIST_OK;
}

extern "C" twist_status twist_set_kernel_choice(twist_ctx *ctx, int32_t gemm_tile, int32_t plain_only, int32_t staged_attention) {
  if (!ctx) TW_FAIL(nullptr, TWIST_EINVAL, "twist_set_kernel_choice: null ctx");
  if (gemm_tile != 0 && gemm_tile != 128 && gemm_tile != 256) TW_FAIL(ctx, TWIST_EINVAL, "twist_set_kernel_choice: gemm_tile must be 0, 128 or 256");
  ctx->gemm_tile = gemm_tile;
  ctx->plain_only = plain_only != 0;
  ctx->staged_attention = staged_attention != 0;
  return TWIST_OK;
}

extern "C" twist_status twist_profile_mfma_ceiling(twist_ctx *ctx, int32_t waves_per_simd, int32_t iters, int32_t random_operands, float *sink,
                                                   size_t sink_floats, double *tflops) {
  if (!ctx || !sink || !tflops) TW_FAIL(ctx, TWIST_EINVAL, "twist_profile_mfma_ceiling: null argument");
  if (waves_per_simd < 1 || waves_per_simd > 8 || iters < 1) TW_FAIL(ctx, TWIST_EINVAL, "twist_profile_mfma_ceiling: waves_per_simd in [1, 8], iters >= 1");
  hipDeviceProp_t prop;
  int dev = 0;
  TW_HIP(ctx, hipGetDevice(&dev));
  TW_HIP(ctx, hipGetDeviceProperties(&prop, dev));
  const int blocks = prop.multiProcessorCount * waves_per_simd;  // a workgroup is 4 waves, one per SIMD of a compute unit
  if (sink_floats < (size_t)blocks * 256) TW_FAIL(ctx, TWIST_ESHAPE, "twist_profile_mfma_ceiling: sink needs %zu floats", (size_t)blocks * 256);
  hipEvent_t e0, e1;
  TW_HIP(ctx, hipEventCreate(&e0));
  TW_HIP(ctx, hipEventCreate(&e1));
  hipLaunchKernelGGL(mfma_only_kernel, dim3(blocks), dim3(256), 0, ctx->stream, iters / 8 + 1, sink, random_operands);  // warm-up
  (void)hipEventRecord(e0, ctx->stream);
  hipLaunchKernelGGL(mfma_only_kernel, dim3(blocks), dim3(256), 0, ctx->stream, iters, sink, random_operands);
  (void)hipEventRecord(e1, ctx->stream);
  hipError_t err = hipEventSynchronize(e1);
  float ms = 0.f;
  if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  TW_HIP(ctx, err);
  const double trips = (double)((iters + 3) / 4);  // the kernel runs four iterations per trip
  *tflops = (double)blocks * 4.0 * trips * 16.0 * (2.0 * 32 * 32 * 16) / ((double)ms * 1e-3) / 1e12;
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
