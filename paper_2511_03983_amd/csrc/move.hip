// Dispatcher and aggregator data movement (Sections 3.2 and 3.3): segment gather and pull scatter-average.
//
// Every partitioned tensor is seen as `rows` rows of segments of Q elements.  extract copies, for each row,
// the n_sub segments a blueprint row names into a dense row; aggregate walks the CENTRAL tensor and, for
// each of its segments, pulls the matching segment from every subnet that holds it (through the inverse
// table), sums in fp32 in subnet order, divides by the number of owners and stores once.  No atomics, no
// staging buffer: every byte is read once and written once, so results are run-to-run bit-identical.
//
// All tensors of one layer go into one launch: a workgroup finds its job by its block index.  Two data
// paths: 16-byte vectors when segments are 16-byte multiples (whole matrix rows, head columns), and an
// element path with lane-consecutive elements (neuron columns of the down projection), where a wave's 64
// lanes read a short contiguous span of the source row and write one full 128-byte line.
#include <type_traits>

#include "twist_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 8;  // subnets handled together (loads issued together in the pull, destinations in the push)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int ES> struct VecOf;
template <> struct VecOf<2> { using vec = u32x4; using elem = uint16_t; static constexpr int N = 8; };
template <> struct VecOf<4> { using vec = u32x4; using elem = uint32_t; static constexpr int N = 4; };

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                  // round to nearest even
  return u >> 16;
}

__device__ __forceinline__ int find_job(const MoveLaunch &ml, int blk) {
  int j = 0;
#pragma unroll 1
  for (int i = 1; i < ml.n_jobs; ++i)
    if (blk >= ml.blk_begin[i]) j = i;
  return j;
}

// ------------------------------------------------------------------------------------------- extract
template <int ES, int TR, int TU>
__device__ __forceinline__ void gather_vec(const MoveJob &jb, char *dst_base, int lb) {
  using V = typename VecOf<ES>::vec;
  constexpr int VN = VecOf<ES>::N;
  const int qv = jb.Q / VN;
  const int64_t Ws = (int64_t)jb.n_sub * qv, Wf = (int64_t)jb.n_full * qv;
  const int ct = lb % jb.tiles_per_row, rt = lb / jb.tiles_per_row;
  const V *src = reinterpret_cast<const V *>(jb.full);
  V *dst = reinterpret_cast<V *>(dst_base + jb.sub_off * ES);
  V val[TR][TU];
  int64_t dv[TU], sv[TU];
#pragma unroll
  for (int u = 0; u < TU; ++u) {
    int64_t v = (int64_t)ct * (kThreads * TU) + u * kThreads + threadIdx.x;
    dv[u] = v < Ws ? v : -1;
    if (v < Ws) {
      int k = (int)(v / qv);
      int j = (int)(v - (int64_t)k * qv);
      sv[u] = jb.table ? (int64_t)jb.table[k] * qv + j : v;
    } else {
      sv[u] = 0;
    }
  }
#pragma unroll
  for (int r = 0; r < TR; ++r) {
    int row = rt * TR + r;
#pragma unroll
    for (int u = 0; u < TU; ++u)
      if (row < jb.rows && dv[u] >= 0) val[r][u] = __builtin_nontemporal_load(&src[row * Wf + sv[u]]);
  }
#pragma unroll
  for (int r = 0; r < TR; ++r) {
    int row = rt * TR + r;
#pragma unroll
    for (int u = 0; u < TU; ++u)
      if (row < jb.rows && dv[u] >= 0) __builtin_nontemporal_store(val[r][u], &dst[row * Ws + dv[u]]);
  }
}

// Element path: a thread owns two ADJACENT destination elements of the tile (one packed store when the
// element is 2 bytes), keeps their source columns in registers and walks the rows of the tile, eight at a
// time so that sixteen independent loads are in flight.  Consecutive lanes read a short ascending span of the
// source row and write consecutive bytes.
template <int ES>
__device__ __forceinline__ void gather_elem(const MoveJob &jb, char *dst_base, int lb) {
  using E = typename VecOf<ES>::elem;
  constexpr int RU = 8;
  const int64_t Ws = (int64_t)jb.n_sub * jb.Q, Wf = (int64_t)jb.n_full * jb.Q;
  const int ct = lb % jb.tiles_per_row, rt = lb / jb.tiles_per_row;
  const E *src = reinterpret_cast<const E *>(jb.full);
  E *dst = reinterpret_cast<E *>(dst_base + jb.sub_off * ES);
  const int64_t v0 = (int64_t)ct * (kThreads * 2) + 2 * threadIdx.x;
  if (v0 >= Ws) return;
  const bool two = v0 + 1 < Ws;
  int64_t sv[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int64_t v = two || u == 0 ? v0 + u : v0;
    const int k = (int)(v / jb.Q);
    const int j = (int)(v - (int64_t)k * jb.Q);
    sv[u] = jb.table ? (int64_t)jb.table[k] * jb.Q + j : v;
  }
  const int r0 = rt * jb.tile_rows;
  const int r1 = min(r0 + jb.tile_rows, jb.rows);
  const bool packed = ES == 2 && two && (Ws & 1) == 0 && ((reinterpret_cast<uintptr_t>(dst) & 3) == 0);
  int row = r0;
  for (; row + RU <= r1; row += RU) {
    E val[RU][2];
#pragma unroll
    for (int r = 0; r < RU; ++r) {
      val[r][0] = src[(row + r) * Wf + sv[0]];
      val[r][1] = src[(row + r) * Wf + sv[1]];
    }
#pragma unroll
    for (int r = 0; r < RU; ++r) {
      E *d = dst + (row + r) * Ws + v0;
      if (packed) *reinterpret_cast<uint32_t *>(d) = (uint32_t)val[r][0] | ((uint32_t)val[r][1] << 16);
      else { d[0] = val[r][0]; if (two) d[1] = val[r][1]; }
    }
  }
  for (; row < r1; ++row) {
    E *d = dst + row * Ws + v0;
    d[0] = src[row * Wf + sv[0]];
    if (two) d[1] = src[row * Wf + sv[1]];
  }
}

// Row-block path (jobs whose segments are whole multiples of 256 vectors: blocks of matrix rows).  Every group of
// 256 consecutive destination vectors lies inside one unit, so the blueprint entry is one scalar load per group
// instead of a dependent per-lane lookup, and a thread keeps TU independent 16-byte loads in flight.
template <int ES, int TU>
__device__ __forceinline__ void gather_rows(const MoveJob &jb, char *dst_base, int lb) {
  using V = typename VecOf<ES>::vec;
  constexpr int VN = VecOf<ES>::N;
  const int qv = jb.Q / VN;
  const int64_t Ws = (int64_t)jb.n_sub * qv;
  const V *src = reinterpret_cast<const V *>(jb.full);
  V *dst = reinterpret_cast<V *>(dst_base + jb.sub_off * ES);
  const int64_t g0 = (int64_t)lb * (kThreads * TU);
  V val[TU];
  int64_t sv[TU];
#pragma unroll
  for (int u = 0; u < TU; ++u) {
    const int64_t g = g0 + u * kThreads;  // first vector of the group: uniform over the workgroup
    sv[u] = -1;
    if (g < Ws) {
      const int k = __builtin_amdgcn_readfirstlane((int)(g / qv));
      const int unit = jb.table ? jb.table[k] : k;
      sv[u] = (int64_t)unit * qv + (g - (int64_t)k * qv) + threadIdx.x;
    }
  }
#pragma unroll
  for (int u = 0; u < TU; ++u)
    if (sv[u] >= 0) val[u] = __builtin_nontemporal_load(&src[sv[u]]);
#pragma unroll
  for (int u = 0; u < TU; ++u)
    if (sv[u] >= 0) __builtin_nontemporal_store(val[u], &dst[g0 + u * kThreads + threadIdx.x]);
}

// All subnets at once (row-block jobs): a group of 256 central vectors is read ONCE and written to every subnet whose
// blueprint row names its unit (owners found through the inverse table, scalar loads), instead of once per subnet.
template <int ES, int TU>
__device__ __forceinline__ void push_rows(const MoveLaunch &ml, const MoveJob &jb, int lb) {
  using V = typename VecOf<ES>::vec;
  constexpr int VN = VecOf<ES>::N;
  const int qv = jb.Q / VN;
  const int64_t Wf = (int64_t)jb.n_full * qv;  // a multiple of 256: a group is entirely inside or outside
  const V *full = reinterpret_cast<const V *>(jb.full);
  const int64_t g0 = (int64_t)lb * (kThreads * TU);
  V val[TU];
#pragma unroll
  for (int u = 0; u < TU; ++u)
    if (g0 + u * kThreads < Wf) val[u] = __builtin_nontemporal_load(&full[g0 + u * kThreads + threadIdx.x]);
#pragma unroll
  for (int u = 0; u < TU; ++u) {
    const int64_t g = g0 + u * kThreads;
    if (g >= Wf) continue;
    const int unit = __builtin_amdgcn_readfirstlane((int)(g / qv));
    const int64_t j = g - (int64_t)unit * qv + threadIdx.x;
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
      if (i < ml.n_subs) {
        const int p = jb.table ? jb.table[(int64_t)ml.sub_row[i] * jb.n_full + unit] : 0;
        if (p >= 0) {
          V *dst = reinterpret_cast<V *>(const_cast<char *>(ml.sub_base[i]) + jb.sub_off * ES);
          __builtin_nontemporal_store(val[u], &dst[(int64_t)p * qv + j]);
        }
      }
  }
}

template <int ES, int TU>
__global__ __launch_bounds__(kThreads) void extract_all_rows_kernel(const MoveLaunch ml) {
  const int ji = find_job(ml, blockIdx.x);
  const MoveJob &jb = ml.job[ji];
  push_rows<ES, TU>(ml, jb, blockIdx.x - jb.blk_begin);
}

template <int ES>
__global__ __launch_bounds__(kThreads) void extract_kernel(const MoveLaunch ml) {
  const int ji = find_job(ml, blockIdx.x);
  const MoveJob &jb = ml.job[ji];
  const int lb = blockIdx.x - jb.blk_begin;
  char *dst_base = const_cast<char *>(ml.sub_base[0]);
  if (jb.vec == 2) {
    gather_rows<ES, 8>(jb, dst_base, lb);
  } else if (jb.vec) {
    if (jb.tile_u == 4) gather_vec<ES, 1, 4>(jb, dst_base, lb);
    else if (jb.tile_u == 2) gather_vec<ES, 2, 2>(jb, dst_base, lb);
    else gather_vec<ES, 4, 1>(jb, dst_base, lb);
  } else {
    gather_elem<ES>(jb, dst_base, lb);
  }
}

// ------------------------------------------------------------------------------------------- aggregate
template <int ES> struct Acc;
template <> struct Acc<2> {
  float a[8];
  __device__ __forceinline__ void set(const u32x4 &v) {
    a[0] = bf16_to_f32(v.x & 0xffff); a[1] = bf16_to_f32(v.x >> 16);
    a[2] = bf16_to_f32(v.y & 0xffff); a[3] = bf16_to_f32(v.y >> 16);
    a[4] = bf16_to_f32(v.z & 0xffff); a[5] = bf16_to_f32(v.z >> 16);
    a[6] = bf16_to_f32(v.w & 0xffff); a[7] = bf16_to_f32(v.w >> 16);
  }
  __device__ __forceinline__ void add(const u32x4 &v) {
    a[0] += bf16_to_f32(v.x & 0xffff); a[1] += bf16_to_f32(v.x >> 16);
    a[2] += bf16_to_f32(v.y & 0xffff); a[3] += bf16_to_f32(v.y >> 16);
    a[4] += bf16_to_f32(v.z & 0xffff); a[5] += bf16_to_f32(v.z >> 16);
    a[6] += bf16_to_f32(v.w & 0xffff); a[7] += bf16_to_f32(v.w >> 16);
  }
  __device__ __forceinline__ u32x4 mean(int cnt) const {
    const float c = (float)cnt;
    u32x4 o;
    o.x = f32_to_bf16(a[0] / c) | (f32_to_bf16(a[1] / c) << 16);
    o.y = f32_to_bf16(a[2] / c) | (f32_to_bf16(a[3] / c) << 16);
    o.z = f32_to_bf16(a[4] / c) | (f32_to_bf16(a[5] / c) << 16);
    o.w = f32_to_bf16(a[6] / c) | (f32_to_bf16(a[7] / c) << 16);
    return o;
  }
};
template <> struct Acc<4> {
  float a[4];
  __device__ __forceinline__ void set(const u32x4 &v) {
    a[0] = __uint_as_float(v.x); a[1] = __uint_as_float(v.y); a[2] = __uint_as_float(v.z); a[3] = __uint_as_float(v.w);
  }
  __device__ __forceinline__ void add(const u32x4 &v) {
    a[0] += __uint_as_float(v.x); a[1] += __uint_as_float(v.y); a[2] += __uint_as_float(v.z); a[3] += __uint_as_float(v.w);
  }
  __device__ __forceinline__ u32x4 mean(int cnt) const {
    const float c = (float)cnt;
    u32x4 o;
    o.x = __float_as_uint(a[0] / c); o.y = __float_as_uint(a[1] / c);
    o.z = __float_as_uint(a[2] / c); o.w = __float_as_uint(a[3] / c);
    return o;
  }
};

template <int ES> __device__ __forceinline__ float elem_to_f32(typename VecOf<ES>::elem e);
template <> __device__ __forceinline__ float elem_to_f32<2>(uint16_t e) { return bf16_to_f32(e); }
template <> __device__ __forceinline__ float elem_to_f32<4>(uint32_t e) { return __uint_as_float(e); }
template <int ES> __device__ __forceinline__ typename VecOf<ES>::elem f32_to_elem(float f);
template <> __device__ __forceinline__ uint16_t f32_to_elem<2>(float f) { return (uint16_t)f32_to_bf16(f); }
template <> __device__ __forceinline__ uint32_t f32_to_elem<4>(float f) { return __float_as_uint(f); }


// Vector path of the pull.  Three phases so that the two dependent memory round trips (inverse table, then
// data) are each paid once per thread, not once per vector: all table lookups, then all data loads, then the
// sums and the stores.  With more than kChunk subnets the phases repeat per chunk of subnets.
template <int ES, int TR, int TU>
__device__ __forceinline__ void pull_vec(const MoveLaunch &ml, const MoveJob &jb, int lb) {
  using V = typename VecOf<ES>::vec;
  constexpr int VN = VecOf<ES>::N;
  const int qv = jb.Q / VN;
  const int64_t Ws = (int64_t)jb.n_sub * qv, Wf = (int64_t)jb.n_full * qv;
  const int ct = lb % jb.tiles_per_row, rt = lb / jb.tiles_per_row;
  V *full = reinterpret_cast<V *>(const_cast<void *>(jb.full));
  int64_t v[TU];
  int unit[TU], j[TU];
#pragma unroll
  for (int u = 0; u < TU; ++u) {
    v[u] = (int64_t)ct * (kThreads * TU) + u * kThreads + threadIdx.x;
    const int64_t vc = v[u] < Wf ? v[u] : 0;
    unit[u] = (int)(vc / qv);
    j[u] = (int)(vc - (int64_t)unit[u] * qv);
  }
  Acc<ES> acc[TU][TR];
  int cnt[TU];
#pragma unroll
  for (int u = 0; u < TU; ++u) cnt[u] = 0;
  for (int c0 = 0; c0 < ml.n_subs; c0 += kChunk) {
    int p[TU][kChunk];
#pragma unroll
    for (int u = 0; u < TU; ++u)
#pragma unroll
      for (int i = 0; i < kChunk; ++i) {
        p[u][i] = -1;
        if (c0 + i < ml.n_subs && v[u] < Wf) p[u][i] = jb.table ? jb.table[(int64_t)ml.sub_row[c0 + i] * jb.n_full + unit[u]] : 0;
      }
    V val[TU][kChunk][TR];
#pragma unroll
    for (int u = 0; u < TU; ++u)
#pragma unroll
      for (int i = 0; i < kChunk; ++i)
        if (p[u][i] >= 0) {
          const V *sp = reinterpret_cast<const V *>(ml.sub_base[c0 + i] + jb.sub_off * ES) + (int64_t)p[u][i] * qv + j[u];
#pragma unroll
          for (int r = 0; r < TR; ++r) {
            const int row = rt * TR + r;
            if (row < jb.rows) val[u][i][r] = __builtin_nontemporal_load(&sp[row * Ws]);
          }
        }
#pragma unroll
    for (int u = 0; u < TU; ++u)
#pragma unroll
      for (int i = 0; i < kChunk; ++i)
        if (p[u][i] >= 0) {
#pragma unroll
          for (int r = 0; r < TR; ++r) {
            if (cnt[u] == 0) acc[u][r].set(val[u][i][r]); else acc[u][r].add(val[u][i][r]);
          }
          ++cnt[u];
        }
  }
#pragma unroll
  for (int u = 0; u < TU; ++u)
    if (cnt[u] > 0) {
#pragma unroll
      for (int r = 0; r < TR; ++r) {
        const int row = rt * TR + r;
        if (row < jb.rows) __builtin_nontemporal_store(acc[u][r].mean(cnt[u]), &full[row * Wf + v[u]]);
      }
    }
}

// Element path of the pull: a thread owns two adjacent central elements.  Their positions in every subnet are
// looked up once and reused for all rows of the tile.  Loads are unconditional (a subnet that does not hold the
// unit is read at position 0 and masked out), so no lane diverges and 4 rows x 8 subnets x 2 elements of loads
// are in flight; sums are formed in subnet order, starting from the first owner's value itself so that a
// single-owner element is copied bit for bit.
template <int ES>
__device__ __forceinline__ void pull_elem(const MoveLaunch &ml, const MoveJob &jb, int lb) {
  using E = typename VecOf<ES>::elem;
  constexpr int RU = 2;
  const int64_t Ws = (int64_t)jb.n_sub * jb.Q, Wf = (int64_t)jb.n_full * jb.Q;
  const int ct = lb % jb.tiles_per_row, rt = lb / jb.tiles_per_row;
  E *full = reinterpret_cast<E *>(const_cast<void *>(jb.full));
  const int r0 = rt * jb.tile_rows;
  const int r1 = min(r0 + jb.tile_rows, jb.rows);
  const int64_t v0 = (int64_t)ct * (kThreads * 2) + 2 * threadIdx.x;
  if (v0 >= Wf) return;
  const bool two = v0 + 1 < Wf;
  if (ml.n_subs <= kChunk) {
    int64_t pos[kChunk][2];
    bool ok[kChunk][2];
    int have[2] = {0, 0};
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int64_t v = (two || u == 0) ? v0 + u : v0;
      const int unit = (int)(v / jb.Q);
      const int j = (int)(v - (int64_t)unit * jb.Q);
#pragma unroll
      for (int i = 0; i < kChunk; ++i) {
        int p = -1;
        if (i < ml.n_subs) p = jb.table ? jb.table[(int64_t)ml.sub_row[i] * jb.n_full + unit] : 0;
        ok[i][u] = p >= 0 && (u == 0 || two);
        pos[i][u] = ok[i][u] ? (int64_t)p * jb.Q + j : 0;
        have[u] += ok[i][u] ? 1 : 0;
      }
    }
    if (have[0] == 0 && have[1] == 0) return;  // no owner: the central values stay
    const float c0 = (float)max(have[0], 1), c1 = (float)max(have[1], 1);
    const bool packed = ES == 2 && have[0] > 0 && have[1] > 0 && (Wf & 1) == 0 && ((reinterpret_cast<uintptr_t>(full) & 3) == 0);
    auto reduce_store = [&](const E (&val)[kChunk][2], int row) {
      float acc[2] = {0.f, 0.f};
      bool seen[2] = {false, false};
#pragma unroll
      for (int i = 0; i < kChunk; ++i)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const float x = elem_to_f32<ES>(val[i][u]);
          acc[u] = ok[i][u] ? (seen[u] ? acc[u] + x : x) : acc[u];
          seen[u] = seen[u] || ok[i][u];
        }
      E *d = full + row * Wf + v0;
      const E o0 = f32_to_elem<ES>(acc[0] / c0), o1 = f32_to_elem<ES>(acc[1] / c1);
      if (packed) *reinterpret_cast<uint32_t *>(d) = (uint32_t)o0 | ((uint32_t)o1 << 16);
      else { if (have[0]) d[0] = o0; if (have[1]) d[1] = o1; }
    };
    int row = r0;
    for (; row + RU <= r1; row += RU) {
      E val[RU][kChunk][2];
#pragma unroll
      for (int r = 0; r < RU; ++r)
#pragma unroll
        for (int i = 0; i < kChunk; ++i)
          if (i < ml.n_subs) {
            const E *sp = reinterpret_cast<const E *>(ml.sub_base[i] + jb.sub_off * ES) + (row + r) * Ws;
            val[r][i][0] = sp[pos[i][0]];
            val[r][i][1] = sp[pos[i][1]];
          }
#pragma unroll
      for (int r = 0; r < RU; ++r) reduce_store(val[r], row + r);
    }
    for (; row < r1; ++row) {
      E val[kChunk][2];
#pragma unroll
      for (int i = 0; i < kChunk; ++i)
        if (i < ml.n_subs) {
          const E *sp = reinterpret_cast<const E *>(ml.sub_base[i] + jb.sub_off * ES) + row * Ws;
          val[i][0] = sp[pos[i][0]];
          val[i][1] = sp[pos[i][1]];
        }
      reduce_store(val, row);
    }
  } else {
    // more subnets than one chunk: plain loop over all of them per row
    for (int u = 0; u < (two ? 2 : 1); ++u) {
      const int64_t v = v0 + u;
      const int unit = (int)(v / jb.Q);
      const int j = (int)(v - (int64_t)unit * jb.Q);
      for (int row = r0; row < r1; ++row) {
        float acc = 0.f;
        int cnt = 0;
        for (int i = 0; i < ml.n_subs; ++i) {
          int p = jb.table ? jb.table[(int64_t)ml.sub_row[i] * jb.n_full + unit] : 0;
          if (p >= 0) {
            float x = elem_to_f32<ES>(reinterpret_cast<const E *>(ml.sub_base[i] + jb.sub_off * ES)[row * Ws + (int64_t)p * jb.Q + j]);
            acc = cnt ? acc + x : x;
            ++cnt;
          }
        }
        if (cnt) full[row * Wf + v] = f32_to_elem<ES>(acc / (float)cnt);
      }
    }
  }
}

// Element path of the pull with the subnet rows staged through LDS (at most kChunk subnets).  The blueprint rows are
// ascending, so the elements a subnet contributes to a tile of 512 adjacent central elements are ADJACENT in its own
// row: instead of 2-byte loads scattered by the inverse table, each wave copies whole (row, subnet) spans into LDS
// with aligned 16-byte loads, and the threads then pick their elements out of LDS.  Sums are formed in subnet order
// as in pull_elem: the accumulator starts at -0.0, which leaves the first owner's value (any value, signed zeros
// included) unchanged, and a subnet that does not hold the element reads -0.0 from a dummy block behind the spans, so
// the row loop needs no masks and no branches.  Vector loads start at the 16-byte boundary at or below the span and
// end at the one at or above it; tensors start on 256-byte boundaries of a slab whose end is padded likewise, so they
// stay inside the subnet's slab.  A tile whose spans do not fit (never the case for tables made by twist_sample) is
// read from the subnets directly.  Positions are kept in 32 bits: the caller checks that a subnet row is shorter
// than 2^31 elements.
constexpr int kStageRows = 4;  // rows staged per pass: one per wave
template <int ES> struct StageShape {
  static constexpr int VN = VecOf<ES>::N;
  static constexpr int SEGV = 512 / VN + 1;                   // 16-byte vectors per (row, subnet) span: 512 elements + misalignment
  static constexpr int VECS = kStageRows * kChunk * SEGV + 2; // + the dummy block of -0.0 values (at least VN of them)
};
template <int ES>
__device__ __forceinline__ void pull_elem_staged(const MoveLaunch &ml, const MoveJob &jb, int lb, u32x4 *stage, int *span_lo, int *span_hi) {
  using E = typename VecOf<ES>::elem;
  constexpr int VN = StageShape<ES>::VN, SEGV = StageShape<ES>::SEGV, SEG = SEGV * VN;
  constexpr int DUMMY = kStageRows * kChunk * SEG;  // first element of the dummy block
  static_assert(kStageRows == kThreads / 64, "one staged row per wave");
  // largest LDS element index read: a span holds at most 512 elements behind a misalignment of at most VN - 1, so an owner's
  // index stays below its own SEG-element slot; a non-owner reads DUMMY + (0 .. VN - 1), inside the dummy block's 2 VN elements
  static_assert(SEG >= 512 + VN - 1 + 1 && StageShape<ES>::VECS * VN >= DUMMY + 2 * VN, "staged spans and dummy block fit the LDS array");
  typedef const E __attribute__((address_space(3))) *lds_elems;
  typedef const u32x4 __attribute__((address_space(1))) *global_vecs;  // plain global loads: they leave the LDS counter alone
  const lds_elems stage_e = (lds_elems)stage;
  const int64_t Ws = (int64_t)jb.n_sub * jb.Q, Wf = (int64_t)jb.n_full * jb.Q;
  const int ct = lb % jb.tiles_per_row, rt = lb / jb.tiles_per_row;
  E *full = reinterpret_cast<E *>(const_cast<void *>(jb.full));
  const int r0 = rt * jb.tile_rows;
  const int r1 = min(r0 + jb.tile_rows, jb.rows);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;  // wave-uniform: span arithmetic stays scalar
  const int64_t v0 = (int64_t)ct * (kThreads * 2) + 2 * threadIdx.x;
  const bool in = v0 < Wf, two = v0 + 1 < Wf;
  if (threadIdx.x < kChunk) { span_lo[threadIdx.x] = 0x7fffffff; span_hi[threadIdx.x] = -1; }
  constexpr uint32_t neg0 = ES == 2 ? 0x80008000u : 0x80000000u;  // -0.0 in every element
  if (threadIdx.x < 2) stage[kStageRows * kChunk * SEGV + threadIdx.x] = u32x4{neg0, neg0, neg0, neg0};
  __syncthreads();
  int pos[kChunk][2];
  bool ok[kChunk][2];
  int have[2] = {0, 0};
#pragma unroll
  for (int u = 0; u < 2; ++u) {  // all table lookups first, so that they are in flight together
    const int64_t v = (two || u == 0) ? v0 + u : v0;
    const int unit = in ? (int)(v / jb.Q) : 0;
#pragma unroll
    for (int i = 0; i < kChunk; ++i) {
      pos[i][u] = -1;
      if (in && i < ml.n_subs) pos[i][u] = jb.table ? jb.table[(int64_t)ml.sub_row[i] * jb.n_full + unit] : 0;
    }
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int64_t v = (two || u == 0) ? v0 + u : v0;
    const int unit = in ? (int)(v / jb.Q) : 0;
    const int j = in ? (int)(v - (int64_t)unit * jb.Q) : 0;
#pragma unroll
    for (int i = 0; i < kChunk; ++i) {
      ok[i][u] = pos[i][u] >= 0 && (u == 0 || two);
      pos[i][u] = ok[i][u] ? pos[i][u] * jb.Q + j : 0;
      have[u] += ok[i][u] ? 1 : 0;
    }
  }
#pragma unroll
  for (int i = 0; i < kChunk; ++i) {
    const int first = ok[i][0] ? pos[i][0] : pos[i][1], last = ok[i][1] ? pos[i][1] : pos[i][0];
    if (ok[i][0] || ok[i][1]) { atomicMin(&span_lo[i], min(first, last)); atomicMax(&span_hi[i], max(first, last)); }
  }
  __syncthreads();
  // the spans' bounds and the misalignment of each subnet's row 0 span, wave-uniform
  int lo[kChunk], hi[kChunk];
  uint32_t mis[kChunk];
  bool fits = true;
#pragma unroll
  for (int i = 0; i < kChunk; ++i) {
    lo[i] = __builtin_amdgcn_readfirstlane(span_lo[i]);
    hi[i] = __builtin_amdgcn_readfirstlane(span_hi[i]);
    fits = fits && (hi[i] < lo[i] || hi[i] - lo[i] < 512);
    mis[i] = i < ml.n_subs && hi[i] >= lo[i] ? (uint32_t)((reinterpret_cast<uintptr_t>(ml.sub_base[i]) + (uintptr_t)((jb.sub_off + lo[i]) * ES)) & 15) : 0u;
  }
  const uint32_t row_bytes = (uint32_t)(Ws * ES) & 15u;  // what a step of one row adds to the misalignment
  const float c0 = (float)max(have[0], 1), c1 = (float)max(have[1], 1);
  const bool packed = ES == 2 && have[0] > 0 && have[1] > 0 && (Wf & 1) == 0 && ((reinterpret_cast<uintptr_t>(full) & 3) == 0);
  if (!fits) {
#pragma unroll 1
    for (int row = r0; row < r1; ++row) {
      float acc[2] = {-0.f, -0.f};
#pragma unroll 1
      for (int i = 0; i < ml.n_subs; ++i) {
        const E *direct = reinterpret_cast<const E *>(ml.sub_base[i] + jb.sub_off * ES) + row * Ws;
#pragma unroll
        for (int u = 0; u < 2; ++u) acc[u] += ok[i][u] ? elem_to_f32<ES>(direct[pos[i][u]]) : -0.f;
      }
      if (in) {
        E *d = full + row * Wf + v0;
        if (have[0]) d[0] = f32_to_elem<ES>(acc[0] / c0);
        if (have[1]) d[1] = f32_to_elem<ES>(acc[1] / c1);
      }
    }
    return;
  }
  // LDS element index of each source inside a staged row, without the row's misalignment; subnets that do not hold
  // the element point at the dummy block
  int off[kChunk][2];
  int row_step[kChunk][2];  // LDS elements from one staged row to the next: 0 for the dummy block, which is not per row
#pragma unroll
  for (int i = 0; i < kChunk; ++i)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      off[i][u] = ok[i][u] ? i * SEG + pos[i][u] - lo[i] : DUMMY;
      row_step[i][u] = ok[i][u] ? kChunk * SEG : 0;
    }
  // Rows of a subnet tensor that are a multiple of 16 bytes apart (the usual case) all have the misalignment of row
  // 0, which is then folded into the indices once; otherwise it is recomputed for every row.
  const bool same_shift = row_bytes == 0;
  if (same_shift) {
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
#pragma unroll
      for (int u = 0; u < 2; ++u) off[i][u] += ok[i][u] ? (int)(mis[i] / ES) : 0;
  }
  auto consume = [&](int row0, auto shift_varies) {  // sums and stores of the staged rows row0 .. row0 + kStageRows - 1
#pragma unroll
    for (int r = 0; r < kStageRows; ++r) {
      const int row = row0 + r;
      if (row >= r1) break;
      float acc[2] = {-0.f, -0.f};
#pragma unroll
      for (int i = 0; i < kChunk; ++i) {
        const int sh = decltype(shift_varies)::value ? (int)(((mis[i] + (uint32_t)row * row_bytes) & 15u) / ES) : 0;
#pragma unroll
        // largest index: a staged span's last element, or (dummy) DUMMY + sh < DUMMY + VN, inside the two dummy vectors
        for (int u = 0; u < 2; ++u) acc[u] += elem_to_f32<ES>(stage_e[r * row_step[i][u] + off[i][u] + sh]);
      }
      if (in) {
        E *d = full + row * Wf + v0;
        const E o0 = f32_to_elem<ES>(acc[0] / c0), o1 = f32_to_elem<ES>(acc[1] / c1);
        if (packed) *reinterpret_cast<uint32_t *>(d) = (uint32_t)o0 | ((uint32_t)o1 << 16);
        else { if (have[0]) d[0] = o0; if (have[1]) d[1] = o1; }
      }
    }
  };
  // Copy of the spans of rows row0 .. row0 + kStageRows - 1: wave w takes row row0 + w of every subnet.  issue() starts
  // the loads of each span's first 64 vectors (lanes beyond the span's last vector repeat that vector), commit() puts
  // them into LDS; the loads of one pass are in flight while the pass before it is summed.  Vectors 64 and up exist only
  // for spans of (nearly) all 512 elements and are copied by commit() itself.
  constexpr int SLOTS = (SEGV + 63) / 64;
  u32x4 buf[kChunk];
  int nv[kChunk];
  auto span_start = [&](int i, int row, int &n_vec) -> global_vecs {
    const uintptr_t a = reinterpret_cast<uintptr_t>(ml.sub_base[i]) + (uintptr_t)((jb.sub_off + row * Ws + lo[i]) * ES);
    const uintptr_t a0 = a & ~(uintptr_t)15;
    n_vec = (int)((a - a0) / ES + (hi[i] - lo[i] + 1) + VN - 1) / VN;  // 1 .. SEGV
    return (global_vecs)a0;
  };
  auto issue = [&](int row0) {
#pragma unroll
    for (int i = 0; i < kChunk; ++i) {
      nv[i] = 0;
      if (i < ml.n_subs && row0 + wave < r1 && hi[i] >= lo[i]) {
        const global_vecs src = span_start(i, row0 + wave, nv[i]);
        buf[i] = __builtin_nontemporal_load(src + min(lane, nv[i] - 1));
      }
    }
  };
  auto commit = [&](int row0) {
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
      if (nv[i] > 0) {
        stage[(wave * kChunk + i) * SEGV + min(lane, nv[i] - 1)] = buf[i];
#pragma unroll
        for (int k = 1; k < SLOTS; ++k)
          if (nv[i] > 64 * k) {
            int n;
            const global_vecs src = span_start(i, row0 + wave, n);
            const int idx = min(lane + 64 * k, n - 1);
            stage[(wave * kChunk + i) * SEGV + idx] = __builtin_nontemporal_load(src + idx);
          }
      }
  };
  issue(r0);
  for (int row0 = r0; row0 < r1; row0 += kStageRows) {
    commit(row0);
    __syncthreads();
    if (row0 + kStageRows < r1) issue(row0 + kStageRows);
    if (same_shift) consume(row0, std::false_type());
    else consume(row0, std::true_type());
    __syncthreads();  // the next pass overwrites the staged spans
  }
}

// Row-block path of the pull (see gather_rows): the owners of a group of 256 central vectors are found with
// scalar loads of the inverse table, and only the subnets that hold the unit are read.
template <int ES, int TU>
__device__ __forceinline__ void pull_rows(const MoveLaunch &ml, const MoveJob &jb, int lb) {
  using V = typename VecOf<ES>::vec;
  constexpr int VN = VecOf<ES>::N;
  const int qv = jb.Q / VN;
  const int64_t Wf = (int64_t)jb.n_full * qv;  // a multiple of 256: a group is entirely inside or outside
  V *full = reinterpret_cast<V *>(const_cast<void *>(jb.full));
  const int64_t g0 = (int64_t)lb * (kThreads * TU);
  V val[TU][kChunk];
  int n_own[TU];
  bool own[TU][kChunk];
#pragma unroll
  for (int u = 0; u < TU; ++u) {
    const int64_t g = g0 + u * kThreads;
    n_own[u] = 0;
    const bool in = g < Wf;
    const int unit = in ? __builtin_amdgcn_readfirstlane((int)(g / qv)) : 0;
    const int64_t j = g - (int64_t)unit * qv + threadIdx.x;
#pragma unroll
    for (int i = 0; i < kChunk; ++i) {
      own[u][i] = false;
      if (in && i < ml.n_subs) {
        const int p = jb.table ? jb.table[(int64_t)ml.sub_row[i] * jb.n_full + unit] : 0;
        if (p >= 0) {
          own[u][i] = true;
          ++n_own[u];
          const V *sp = reinterpret_cast<const V *>(ml.sub_base[i] + jb.sub_off * ES);
          val[u][i] = __builtin_nontemporal_load(&sp[(int64_t)p * qv + j]);
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < TU; ++u) {
    if (n_own[u] == 0) continue;  // no owner: the central values stay
    Acc<ES> acc;
    bool first = true;
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
      if (own[u][i]) {
        if (first) acc.set(val[u][i]); else acc.add(val[u][i]);
        first = false;
      }
    __builtin_nontemporal_store(acc.mean(n_own[u]), &full[g0 + u * kThreads + threadIdx.x]);
  }
}

template <int ES>
__global__ __launch_bounds__(kThreads) void aggregate_kernel(const MoveLaunch ml) {
  const int ji = find_job(ml, blockIdx.x);
  const MoveJob &jb = ml.job[ji];
  const int lb = blockIdx.x - jb.blk_begin;
  if (jb.vec) {
    if (jb.tile_u == 4) pull_vec<ES, 1, 4>(ml, jb, lb);
    else if (jb.tile_u == 2 && jb.tile_rows == 1) pull_vec<ES, 1, 2>(ml, jb, lb);
    else if (jb.tile_u == 2) pull_vec<ES, 2, 2>(ml, jb, lb);
    else pull_vec<ES, 4, 1>(ml, jb, lb);
  } else {
    pull_elem<ES>(ml, jb, lb);
  }
}

// launches that hold element-path jobs only
template <int ES>
__global__ __launch_bounds__(kThreads) void aggregate_elem_kernel(const MoveLaunch ml) {
  __shared__ u32x4 stage[StageShape<ES>::VECS];
  __shared__ int span_lo[kChunk], span_hi[kChunk];
  const int ji = find_job(ml, blockIdx.x);
  const MoveJob &jb = ml.job[ji];
  pull_elem_staged<ES>(ml, jb, blockIdx.x - jb.blk_begin, stage, span_lo, span_hi);
}

// launches that hold row-block jobs only: far fewer registers than the general kernel, hence more waves in flight
template <int ES, int TU>
__global__ __launch_bounds__(kThreads) void aggregate_rows_kernel(const MoveLaunch ml) {
  const int ji = find_job(ml, blockIdx.x);
  const MoveJob &jb = ml.job[ji];
  pull_rows<ES, TU>(ml, jb, blockIdx.x - jb.blk_begin);
}

// ------------------------------------------------------------------------------------------- running-sum aggregate
// The aggregation formula of Section 3.3 evaluated one subnet at a time, so that only one subnet has to be resident:
// an fp32 image of the central model receives each subnet's values (stored by the first owner of a block, added by
// later ones, which makes clearing the image unnecessary), and the last pass divides by the number of owners and
// rounds once.  The additions happen in the order of the calls, so the result is bit-identical to the one-shot pull
// over the same subnets in the same order.
template <int ES, int VN, bool FINISH>
__device__ __forceinline__ void accumulate_body(const MoveLaunch &ml, const MoveJob &jb, uint32_t lb) {
  using E = typename VecOf<ES>::elem;
  constexpr int TU = kAccumPerBlock / kThreads;
  const uint32_t q = jb.Q / VN, Wf = (uint32_t)jb.n_full * q, Ws = (uint32_t)jb.n_sub * q;
  const uint32_t total = (uint32_t)jb.rows * Wf;
#pragma unroll
  for (int u = 0; u < TU; ++u) {
    const uint32_t f = lb * (uint32_t)kAccumPerBlock + u * kThreads + threadIdx.x;
    if (f >= total) continue;
    const uint32_t row = f / Wf, v = f - row * Wf;
    const uint32_t unit = v / q, j = v - unit * q;
    float *a = jb.acc + (int64_t)f * VN;
    float x[VN];
    if (!FINISH) {
      const int p = jb.table ? jb.table[(int64_t)ml.sub_row[0] * jb.n_full + unit] : 0;
      if (p < 0) continue;
      bool first = true;
      for (int i = 1; i < ml.n_subs; ++i) first = first && jb.table && jb.table[(int64_t)ml.sub_row[i] * jb.n_full + unit] < 0;
      const E *sp = reinterpret_cast<const E *>(ml.sub_base[0] + jb.sub_off * ES) + ((int64_t)row * Ws + (int64_t)p * q + j) * VN;
      if (VN > 1) {
        const u32x4 raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(sp));
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < VN; ++i) x[i] = ES == 2 ? bf16_to_f32((w[i / 2] >> (16 * (i & 1))) & 0xffff) : __uint_as_float(w[i % 4]);
      } else {
        x[0] = elem_to_f32<ES>(*sp);
      }
      if (VN > 1) {
        f32x4 *a4 = reinterpret_cast<f32x4 *>(a);  // the image is 256-byte aligned and f * VN a multiple of 4
#pragma unroll
        for (int h = 0; h < VN / 4; ++h) {
          f32x4 t = {x[4 * h % VN], x[(4 * h + 1) % VN], x[(4 * h + 2) % VN], x[(4 * h + 3) % VN]};
          if (!first) t = a4[h] + t;
          a4[h] = t;
        }
      } else {
        a[0] = first ? x[0] : a[0] + x[0];
      }
    } else {
      int cnt = 0;
      for (int i = 0; i < ml.n_subs; ++i) cnt += !jb.table || jb.table[(int64_t)ml.sub_row[i] * jb.n_full + unit] >= 0;
      if (cnt == 0) continue;  // no owner: the central values stay
      const float c = (float)cnt;
      E *out = reinterpret_cast<E *>(const_cast<void *>(jb.full)) + (int64_t)f * VN;
      if (VN > 1) {
        const f32x4 *a4 = reinterpret_cast<const f32x4 *>(a);
#pragma unroll
        for (int h = 0; h < VN / 4; ++h) {
          const f32x4 t = a4[h];
          x[4 * h % VN] = t.x / c; x[(4 * h + 1) % VN] = t.y / c; x[(4 * h + 2) % VN] = t.z / c; x[(4 * h + 3) % VN] = t.w / c;
        }
      } else {
        x[0] = a[0] / c;
      }
      if (VN > 1) {
        u32x4 o;
        if (ES == 2) {
          o.x = f32_to_bf16(x[0]) | (f32_to_bf16(x[1 % VN]) << 16);
          o.y = f32_to_bf16(x[2 % VN]) | (f32_to_bf16(x[3 % VN]) << 16);
          o.z = f32_to_bf16(x[4 % VN]) | (f32_to_bf16(x[5 % VN]) << 16);
          o.w = f32_to_bf16(x[6 % VN]) | (f32_to_bf16(x[7 % VN]) << 16);
        } else {
          o.x = __float_as_uint(x[0]); o.y = __float_as_uint(x[1 % VN]); o.z = __float_as_uint(x[2 % VN]); o.w = __float_as_uint(x[3 % VN]);
        }
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(out));
      } else {
        *out = f32_to_elem<ES>(x[0]);
      }
    }
  }
}

template <int ES, bool FINISH>
__global__ __launch_bounds__(kThreads) void accumulate_kernel(const MoveLaunch ml) {
  const int ji = find_job(ml, blockIdx.x);
  const MoveJob &jb = ml.job[ji];
  const uint32_t lb = blockIdx.x - jb.blk_begin;
  if (jb.vec) accumulate_body<ES, VecOf<ES>::N, FINISH>(ml, jb, lb);
  else accumulate_body<ES, 1, FINISH>(ml, jb, lb);
}

// ------------------------------------------------------------------------------------------- helpers
template <int ES>
__global__ __launch_bounds__(kThreads) void to_f32_kernel(const void *src, float *dst, int64_t n) {
  using E = typename VecOf<ES>::elem;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
    dst[i] = elem_to_f32<ES>(reinterpret_cast<const E *>(src)[i]);
}

// bf16 -> fp32, four values per thread and step: one 8-byte load, one 16-byte store, so that a wave's store instruction
// writes 1 KB of consecutive bytes (a bf16 value is the upper half of the fp32 value with the same bits)
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__global__ __launch_bounds__(kThreads) void bf16_to_f32_vec_kernel(const u32x2 *src, u32x4 *dst, int64_t n_vec) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n_vec; i += stride) {
    const u32x2 u = __builtin_nontemporal_load(src + i);
    __builtin_nontemporal_store(u32x4{u.x << 16, u.x & 0xffff0000u, u.y << 16, u.y & 0xffff0000u}, dst + i);
  }
}

__global__ __launch_bounds__(kThreads) void zero_kernel(u32x4 *dst, int64_t n_vec) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n_vec; i += stride) dst[i] = u32x4{0, 0, 0, 0};
}

}  // namespace

twist_status twist_launch_extract(twist_ctx *ctx, const MoveLaunch &ml, int total_blocks) {
  if (total_blocks <= 0) return TWIST_OK;
  if (ctx->esize() == 2) hipLaunchKernelGGL(extract_kernel<2>, dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
  else hipLaunchKernelGGL(extract_kernel<4>, dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_launch_extract_all(twist_ctx *ctx, const MoveLaunch &ml, int total_blocks) {  // row-block jobs, tile_u = 2
  if (total_blocks <= 0) return TWIST_OK;
  if (ctx->esize() == 2) hipLaunchKernelGGL((extract_all_rows_kernel<2, 2>), dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
  else hipLaunchKernelGGL((extract_all_rows_kernel<4, 2>), dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_launch_aggregate(twist_ctx *ctx, const MoveLaunch &ml, int total_blocks) {
  if (total_blocks <= 0) return TWIST_OK;
  bool rows_only = true;
  for (int i = 0; i < ml.n_jobs; ++i) rows_only = rows_only && ml.job[i].vec == 2;
  bool elems_only = ml.n_subs <= kChunk;  // element-path jobs whose subnet rows are short enough for 32-bit positions
  for (int i = 0; i < ml.n_jobs; ++i) elems_only = elems_only && ml.job[i].vec == 0 && (int64_t)ml.job[i].n_sub * ml.job[i].Q < (1ll << 31);
  if (elems_only) {
    if (ctx->esize() == 2) hipLaunchKernelGGL(aggregate_elem_kernel<2>, dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
    else hipLaunchKernelGGL(aggregate_elem_kernel<4>, dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
  } else if (rows_only) {  // the host gives such jobs tile_u = 2
    if (ctx->esize() == 2) hipLaunchKernelGGL((aggregate_rows_kernel<2, 2>), dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
    else hipLaunchKernelGGL((aggregate_rows_kernel<4, 2>), dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
  } else if (ctx->esize() == 2) hipLaunchKernelGGL(aggregate_kernel<2>, dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
  else hipLaunchKernelGGL(aggregate_kernel<4>, dim3(total_blocks), dim3(kThreads), 0, ctx->stream, ml);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_launch_accumulate(twist_ctx *ctx, const MoveLaunch &ml, int total_blocks, bool finish) {
  if (total_blocks <= 0) return TWIST_OK;
  const dim3 g(total_blocks), b(kThreads);
  if (ctx->esize() == 2) {
    if (finish) hipLaunchKernelGGL((accumulate_kernel<2, true>), g, b, 0, ctx->stream, ml);
    else hipLaunchKernelGGL((accumulate_kernel<2, false>), g, b, 0, ctx->stream, ml);
  } else {
    if (finish) hipLaunchKernelGGL((accumulate_kernel<4, true>), g, b, 0, ctx->stream, ml);
    else hipLaunchKernelGGL((accumulate_kernel<4, false>), g, b, 0, ctx->stream, ml);
  }
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_launch_to_f32(twist_ctx *ctx, const void *src, float *dst, int64_t n) {
  if (n <= 0) return TWIST_OK;
  if (ctx->esize() == 2 && n % 8 == 0 && (reinterpret_cast<uintptr_t>(src) % 16) == 0 && (reinterpret_cast<uintptr_t>(dst) % 16) == 0) {
    const int64_t nv = n / 4;
    const int vblocks = (int)std::min<int64_t>((nv + kThreads - 1) / kThreads, 256 * 16);
    hipLaunchKernelGGL(bf16_to_f32_vec_kernel, dim3(vblocks), dim3(kThreads), 0, ctx->stream, static_cast<const u32x2 *>(src), reinterpret_cast<u32x4 *>(dst), nv);
    TW_HIP(ctx, hipGetLastError());
    return TWIST_OK;
  }
  int blocks = (int)std::min<int64_t>((n + kThreads - 1) / kThreads, 256 * 16);
  if (ctx->esize() == 2) hipLaunchKernelGGL(to_f32_kernel<2>, dim3(blocks), dim3(kThreads), 0, ctx->stream, src, dst, n);
  else hipLaunchKernelGGL(to_f32_kernel<4>, dim3(blocks), dim3(kThreads), 0, ctx->stream, src, dst, n);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}

twist_status twist_launch_zero(twist_ctx *ctx, void *dst, size_t bytes) {
  if (bytes == 0) return TWIST_OK;
  int64_t nv = (int64_t)(bytes / 16);  // callers pass multiples of 16
  int blocks = (int)std::min<int64_t>((nv + kThreads - 1) / kThreads, 256 * 16);
  hipLaunchKernelGGL(zero_kernel, dim3(blocks), dim3(kThreads), 0, ctx->stream, reinterpret_cast<u32x4 *>(dst), nv);
  TW_HIP(ctx, hipGetLastError());
  return TWIST_OK;
}
