// Internal declarations shared by the translation units of libtwist (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "twist.h"

#define TWIST_MAX_S 32  // subnets one aggregate launch can average

// ---------------------------------------------------------------------------------------------- errors
void twist_set_error(const twist_ctx *ctx, const char *fmt, ...);

#define TW_FAIL(ctx, code, ...)           \
  do {                                    \
    twist_set_error((ctx), __VA_ARGS__);  \
    return (code);                        \
  } while (0)

#define TW_HIP(ctx, expr)                                                                   \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) TW_FAIL((ctx), TWIST_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

#define TW_TRY(expr)                     \
  do {                                   \
    twist_status s_ = (expr);            \
    if (s_ != TWIST_OK) return s_;       \
  } while (0)

// ---------------------------------------------------------------------------------------------- layout
// Where one tensor lives inside a subnet: an element offset that is the same in the weight slab, the
// fp32 master slab, the gradient slab and the optimizer-moment slabs.
struct Slot {
  int64_t off = -1;  // element offset, -1 = absent
  int32_t rows = 0, cols = 0;
};

struct SubLayout {
  std::vector<Slot> layer;  // [n_layers * TWIST_N_LAYER_TENSORS]
  Slot global[TWIST_N_GLOBAL_TENSORS];
  std::vector<int32_t> heads_sub, ffn_sub;  // per layer kept heads / FFN units
  int64_t n_matrix = 0;  // elements in the matrix region [0, n_matrix): weight decay applies here
  int64_t n_total = 0;   // all elements (multiple of 128)
  const Slot &at(int l, int t) const { return layer[(size_t)l * TWIST_N_LAYER_TENSORS + t]; }
};

struct PlanEntry {
  int32_t n_full = 0, n_sub = 0;
  std::vector<int32_t> idx, inv, count;  // [S*n_sub], [S*n_full], [n_full]
  int32_t *d_idx = nullptr, *d_inv = nullptr, *d_count = nullptr;
};

struct twist_ctx {
  twist_model_desc d;
  hipStream_t stream = nullptr;
  mutable std::string err;
  // optional per-launch timing of the projection kernels (see twist_profile_gemm)
  bool prof_gemm = false;
  std::vector<hipEvent_t> prof_events;  // (start, stop) pairs
  double prof_flops = 0.0;
  // second stream for the weight-gradient projections of the backward pass (created on first use, default
  // priority) and the events that order it against `stream`; overlap can be switched off (twist_set_overlap)
  hipStream_t side = nullptr;
  hipEvent_t ev_ready[4] = {}, ev_done[4] = {};
  bool overlap = true;
  // kernel selection overrides for tests (twist_set_kernel_choice); the defaults let every launcher choose by shape
  int gemm_tile = 0;         // 0 = by shape; 128 / 256 pin the matrix-core projection kernel's tile (and keep the contraction whole)
  bool plain_only = false;   // never use the matrix-core kernels (projections and attention run the plain fp32-arithmetic ones)
  bool staged_attention = false;  // d_head 128: the register-staged tiled attention kernels instead of the direct-to-LDS ones
  int esize() const { return d.dtype == TWIST_BF16 ? 2 : 4; }
  int n_ffn_units() const { return d.d_ff / d.ffn_granule; }
};

struct twist_plan {
  twist_ctx *ctx = nullptr;
  int32_t S = 0, scale_mode = 0;
  std::vector<PlanEntry> e;  // [n_layers * 2], kind-minor
  int32_t *d_tables = nullptr;
  SubLayout layout;
  const PlanEntry &at(int l, int k) const { return e[(size_t)l * 2 + k]; }
};

struct twist_subnet {
  twist_ctx *ctx = nullptr;
  const twist_plan *plan = nullptr;
  int32_t s = 0, store = 0;
  char *base = nullptr;       // caller-owned storage
  char *params = nullptr;     // desc.dtype [n_total]
  float *master = nullptr;    // fp32 [n_total] (bf16 models with gradients), else null
  float *grads = nullptr;     // fp32 [n_total]
  float *adam_m = nullptr, *adam_v = nullptr;
  int64_t step_count = 0;
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------------------------------------- movers
// One tensor's share of a fused gather / pull-average launch.  Every partitioned tensor is viewed as
// `rows` rows, each a sequence of segments of Q elements; a blueprint row picks n_sub of the n_full
// segments.  (A block of whole matrix rows is the rows == 1 case with Q = block_rows * cols.)
struct MoveJob {
  const void *full;     // central tensor [rows][n_full*Q]
  int64_t sub_off;      // element offset of the subnet tensor [rows][n_sub*Q] inside a subnet slab
  const int32_t *table; // extract: idx row of this subnet [n_sub]; aggregate: inv [S][n_full]; null = shared
  int32_t rows, n_full, n_sub, Q;
  int32_t tile_rows, tile_u;  // a workgroup covers tile_rows rows x 256*tile_u vectors (or elements)
  int32_t tiles_per_row;      // ceil(width / (256*tile_u))
  int32_t vec;                // 0 = element path, 1 = 16-byte path, 2 = 16-byte row-block path (segments of whole
                              //     multiples of 256 vectors, one row, at most 8 subnets)
  int32_t blk_begin;          // first workgroup of this job inside the launch
  float *acc;                 // running-sum aggregate only: fp32 image of the central tensor [rows][n_full*Q]
};

// A launch carries the jobs of several layers (as many whole layers as fit): at the 7B shape a layer's extract takes
// about 70 us, and every launch boundary costs about 10 us of drained GPU.  The struct travels as the kernel argument,
// which HIP limits to 4 KB.
#define TWIST_MAX_JOBS 44
struct MoveLaunch {
  MoveJob job[TWIST_MAX_JOBS];
  int32_t blk_begin[TWIST_MAX_JOBS];  // copy of job[i].blk_begin, packed so that a workgroup finds its job with few loads
  int32_t n_jobs;
  int32_t n_subs;                 // aggregate only
  const char *sub_base[TWIST_MAX_S];  // aggregate: weight slab of each given subnet; extract: [0] = destination
  int32_t sub_row[TWIST_MAX_S];   // aggregate: blueprint row of each given subnet
};

static_assert(sizeof(MoveLaunch) <= 4000, "MoveLaunch is passed by value as a kernel argument");

twist_status twist_launch_extract(twist_ctx *ctx, const MoveLaunch &ml, int total_blocks);
twist_status twist_launch_aggregate(twist_ctx *ctx, const MoveLaunch &ml, int total_blocks);
// extract of sub_row[0..n_subs) at once into sub_base[0..n_subs): row-block jobs only, described as for the aggregate
twist_status twist_launch_extract_all(twist_ctx *ctx, const MoveLaunch &ml, int total_blocks);
// Running-sum aggregate: add subnet sub_base[0] (blueprint row sub_row[0]; rows sub_row[1..n_subs) were added before it)
// into the fp32 image, or (finish) write image / owner count over all rows sub_row[0..n_subs) to the central tensors.
constexpr int kAccumPerBlock = 256 * 4;  // vectors (or elements) of the central tensor one workgroup covers
twist_status twist_launch_accumulate(twist_ctx *ctx, const MoveLaunch &ml, int total_blocks, bool finish);
// fp32 master <- weights, zero-fill helpers
twist_status twist_launch_to_f32(twist_ctx *ctx, const void *src, float *dst, int64_t n);
twist_status twist_launch_zero(twist_ctx *ctx, void *dst, size_t bytes);

// ---------------------------------------------------------------------------------------------- training
twist_status twist_train_workspace_bytes(twist_ctx *ctx, const twist_subnet *sub, int B, int N, size_t *bytes);
twist_status twist_train_fwd_bwd(twist_ctx *ctx, twist_subnet *sub, const void *inputs, const void *targets, int B,
                                 int N, void *ws, size_t ws_bytes, float *loss_dev, bool forward_only = false,
                                 const twist_plan *mask_plan = nullptr, int mask_row = 0);
twist_status twist_train_step(twist_ctx *ctx, twist_subnet *sub, const twist_opt_desc *opt);
