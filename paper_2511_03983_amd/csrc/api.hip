// Host side of the C ABI: context, subnet generator (Algorithm 1), subnet layout, and the drivers that
// turn one layer's tensors into a fused gather (dispatcher, Section 3.2) or pull-average (aggregator,
// Section 3.3) launch.
#include <algorithm>
#include <cstring>
#include <atomic>
#include <new>
#include <thread>

#include "twist_internal.h"

// ------------------------------------------------------------------------------------------------ errors
static thread_local std::string g_thread_error;

void twist_set_error(const twist_ctx *ctx, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_thread_error = buf;
  if (ctx) ctx->err = buf;
}

extern "C" const char *twist_last_error(const twist_ctx *ctx) { return ctx ? ctx->err.c_str() : g_thread_error.c_str(); }

// ------------------------------------------------------------------------------------------------ context
extern "C" twist_status twist_create(const twist_model_desc *desc, void *hip_stream, twist_ctx **out) {
  if (!desc || !out) TW_FAIL(nullptr, TWIST_EINVAL, "twist_create: null argument");
  const twist_model_desc &d = *desc;
  if (d.n_layers < 1 || d.d_model < 1 || d.n_heads < 1 || d.d_head < 1 || d.d_ff < 1 || d.ffn_granule < 1 || d.vocab < 0 ||
      d.max_seq < 1)
    TW_FAIL(nullptr, TWIST_ESHAPE, "twist_create: every dimension must be positive");
  if (d.d_ff % d.ffn_granule) TW_FAIL(nullptr, TWIST_ESHAPE, "twist_create: d_ff=%d is not a multiple of ffn_granule=%d", d.d_ff, d.ffn_granule);
  if (d.use_rope && (d.d_head & 1)) TW_FAIL(nullptr, TWIST_ESHAPE, "twist_create: rotary positions need an even d_head");
  if (d.dtype != TWIST_F32 && d.dtype != TWIST_BF16) TW_FAIL(nullptr, TWIST_EINVAL, "twist_create: unknown dtype %d", d.dtype);
  if (d.act < TWIST_ACT_GELU_TANH || d.act > TWIST_ACT_SWIGLU) TW_FAIL(nullptr, TWIST_EINVAL, "twist_create: unknown activation %d", d.act);
  if (d.norm != TWIST_NORM_LN && d.norm != TWIST_NORM_RMS) TW_FAIL(nullptr, TWIST_EINVAL, "twist_create: unknown norm %d", d.norm);
  twist_ctx *c = new (std::nothrow) twist_ctx;
  if (!c) TW_FAIL(nullptr, TWIST_ENOMEM, "twist_create: out of host memory");
  c->d = d;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  *out = c;
  return TWIST_OK;
}

extern "C" void twist_destroy(twist_ctx *ctx) {
  if (!ctx) return;
  for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
  for (int i = 0; i < 4; ++i) {
    if (ctx->ev_ready[i]) (void)hipEventDestroy(ctx->ev_ready[i]);
    if (ctx->ev_done[i]) (void)hipEventDestroy(ctx->ev_done[i]);
  }
  if (ctx->side) (void)hipStreamDestroy(ctx->side);
  delete ctx;
}

// ------------------------------------------------------------------------------------------------ generator
namespace {

// 64-bit counter generator: additive odd constant, then an xor-shift-multiply finaliser.  One stream per
// (seed, round, layer, kind); integers below n by rejection so that draws are exactly uniform.
struct DrawStream {
  uint64_t x;
  static uint64_t finalise(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
  DrawStream(uint64_t seed, uint64_t round, uint64_t layer, uint64_t kind) {
    x = finalise(finalise(finalise(finalise(seed) + round) + layer) + kind);
  }
  uint64_t next() { return finalise(x += 0x9E3779B97F4A7C15ull); }
  uint32_t below(uint32_t n) {
    const uint64_t excess = (0ull - (uint64_t)n) % n;  // 2^64 mod n
    for (;;) {
      uint64_t v = next();
      if (v < 0ull - excess || excess == 0) return (uint32_t)(v % n);
    }
  }
};

// Argument checks of Algorithm 1 (the same for every layer of one kind, so they run once, before any drawing).
twist_status check_blueprint_args(twist_ctx *ctx, int n_full, int S, int n_sub, const int32_t *common, int n_common, bool require_coverage) {
  if (n_common < 0 || (n_common > 0 && !common)) TW_FAIL(ctx, TWIST_EINVAL, "twist_sample: bad common set");
  for (int i = 0; i < n_common; ++i)
    if (common[i] < 0 || common[i] >= n_full || (i > 0 && common[i] <= common[i - 1]))
      TW_FAIL(ctx, TWIST_EINVAL, "twist_sample: common set must be sorted, unique and within [0, %d)", n_full);
  if (n_sub < 1 || n_sub > n_full || n_sub < n_common)
    TW_FAIL(ctx, TWIST_ECONSTRAINT, "twist_sample: need |C|=%d <= N_sub=%d <= N_full=%d", n_common, n_sub, n_full);
  if (require_coverage && (int64_t)n_full - n_common > (int64_t)S * (n_sub - n_common))
    TW_FAIL(ctx, TWIST_ECONSTRAINT, "twist_sample: N_full - |C| = %d exceeds S (N_sub - |C|) = %lld: not every block can be assigned",
            n_full - n_common, (long long)S * (n_sub - n_common));
  return TWIST_OK;
}

// Algorithm 1 on checked arguments.  Row s of idx receives subnet s's block ids in ascending order.  Touches nothing
// but its arguments, so the (layer, kind) entries of a plan can be drawn on separate host threads.
void generate_blueprint(int n_full, int S, int n_sub, const int32_t *common, int n_common, bool require_coverage, DrawStream &rng,
                        std::vector<int32_t> &idx) {
  std::vector<uint8_t> is_common(n_full, 0);
  for (int i = 0; i < n_common; ++i) is_common[common[i]] = 1;
  // fill level of each row; the common blocks come first
  std::vector<int> fill(S, n_common);
  idx.assign((size_t)S * n_sub, -1);
  for (int s = 0; s < S; ++s) std::copy(common, common + n_common, idx.begin() + (size_t)s * n_sub);

  if (require_coverage) {
    // the non-common blocks in random order, dealt round-robin: block i of the order goes to row i mod S
    std::vector<int32_t> rest;
    rest.reserve(n_full - n_common);
    for (int b = 0; b < n_full; ++b)
      if (!is_common[b]) rest.push_back(b);
    for (size_t i = rest.size(); i-- > 1;) std::swap(rest[i], rest[rng.below((uint32_t)i + 1)]);
    for (size_t i = 0; i < rest.size(); ++i) {
      int s = (int)(i % S);
      idx[(size_t)s * n_sub + fill[s]++] = rest[i];
    }
  }
  // top every row up with distinct blocks it does not hold yet, drawn uniformly
  std::vector<uint8_t> held(n_full);
  std::vector<int32_t> pool;
  for (int s = 0; s < S; ++s) {
    int32_t *row = idx.data() + (size_t)s * n_sub;
    const int missing = n_sub - fill[s];
    std::fill(held.begin(), held.end(), 0);
    for (int k = 0; k < fill[s]; ++k) held[row[k]] = 1;
    if (missing > 0) {
      pool.clear();
      for (int b = 0; b < n_full; ++b)
        if (!held[b]) pool.push_back(b);
      for (int t = 0; t < missing; ++t) {
        uint32_t j = t + rng.below((uint32_t)(pool.size() - t));
        std::swap(pool[t], pool[j]);
        held[pool[t]] = 1;
      }
    }
    // the row in ascending order: its blocks are distinct, so reading the membership flags in order sorts it
    int k = 0;
    for (int b = 0; b < n_full; ++b)
      if (held[b]) row[k++] = b;
  }
}

// tensors and how the blueprint cuts them: kind, and whether blocks are rows (0) or columns (1)
struct Cut { int kind; int axis; };
const Cut *cut_of(const twist_model_desc &d, int t) {
  static const Cut head_rows{TWIST_KIND_HEAD, 0}, head_cols{TWIST_KIND_HEAD, 1}, ffn_rows{TWIST_KIND_FFN, 0}, ffn_cols{TWIST_KIND_FFN, 1};
  switch (t) {
    case TWIST_WQ: case TWIST_WK: case TWIST_WV: case TWIST_BQ: case TWIST_BK: case TWIST_BV: return &head_rows;
    case TWIST_WO: return d.out_unit_major ? &head_rows : &head_cols;
    case TWIST_W_GATE: case TWIST_W_UP: case TWIST_B_UP: return &ffn_rows;
    case TWIST_W_DOWN: return d.out_unit_major ? &ffn_rows : &ffn_cols;
    default: return nullptr;
  }
}

bool layer_tensor_present(const twist_model_desc &d, int t) {
  switch (t) {
    case TWIST_WQ: case TWIST_WK: case TWIST_WV: case TWIST_WO: case TWIST_W_UP: case TWIST_W_DOWN:
    case TWIST_NORM1_W: case TWIST_NORM2_W: return true;
    case TWIST_W_GATE: return d.act == TWIST_ACT_SWIGLU;
    case TWIST_NORM1_B: case TWIST_NORM2_B: return d.norm == TWIST_NORM_LN;
    default: return d.has_bias != 0;  // the six biases
  }
}

bool global_tensor_present(const twist_model_desc &d, int t) {
  if (d.vocab == 0) return false;
  switch (t) {
    case TWIST_TOK_EMBED: case TWIST_FINAL_NORM_W: return true;
    case TWIST_POS_EMBED: return !d.use_rope;
    case TWIST_FINAL_NORM_B: return d.norm == TWIST_NORM_LN;
    case TWIST_LM_HEAD: return !d.tied_head;
  }
  return false;
}

// full-model shape of a layer tensor
void full_shape(const twist_model_desc &d, int t, int &rows, int &cols) {
  const int hd = d.n_heads * d.d_head;
  switch (t) {
    case TWIST_WQ: case TWIST_WK: case TWIST_WV: rows = hd; cols = d.d_model; break;
    case TWIST_WO: rows = d.d_model; cols = hd; if (d.out_unit_major) std::swap(rows, cols); break;
    case TWIST_W_GATE: case TWIST_W_UP: rows = d.d_ff; cols = d.d_model; break;
    case TWIST_W_DOWN: rows = d.d_model; cols = d.d_ff; if (d.out_unit_major) std::swap(rows, cols); break;
    case TWIST_BQ: case TWIST_BK: case TWIST_BV: rows = hd; cols = 1; break;
    case TWIST_B_UP: rows = d.d_ff; cols = 1; break;
    default: rows = d.d_model; cols = 1; break;
  }
}

void global_shape(const twist_model_desc &d, int t, int &rows, int &cols) {
  switch (t) {
    case TWIST_TOK_EMBED: case TWIST_LM_HEAD: rows = d.vocab; cols = d.d_model; break;
    case TWIST_POS_EMBED: rows = d.max_seq; cols = d.d_model; break;
    default: rows = d.d_model; cols = 1; break;
  }
}

// Subnet layout: matrices first (so that weight decay covers one contiguous range), vectors after.  Q,K,V
// and gate,up are adjacent with no padding, so that each group is one dense matrix for the projections.
void build_layout(const twist_ctx *ctx, twist_plan *plan) {
  const twist_model_desc &d = ctx->d;
  SubLayout &L = plan->layout;
  L.layer.assign((size_t)d.n_layers * TWIST_N_LAYER_TENSORS, Slot());
  L.heads_sub.resize(d.n_layers);
  L.ffn_sub.resize(d.n_layers);
  int64_t off = 0;
  auto pad = [&]() { off = (int64_t)align_up((size_t)off, 128); };
  auto place = [&](Slot &s, int rows, int cols) { s.off = off; s.rows = rows; s.cols = cols; off += (int64_t)rows * cols; };
  static const int mat_groups[][3] = {{TWIST_WQ, TWIST_WK, TWIST_WV}, {TWIST_WO, -1, -1}, {TWIST_W_GATE, TWIST_W_UP, -1}, {TWIST_W_DOWN, -1, -1}};
  static const int vec_groups[][3] = {{TWIST_BQ, TWIST_BK, TWIST_BV}, {TWIST_BO, -1, -1}, {TWIST_B_UP, -1, -1}, {TWIST_B_DOWN, -1, -1},
                                      {TWIST_NORM1_W, -1, -1}, {TWIST_NORM1_B, -1, -1}, {TWIST_NORM2_W, -1, -1}, {TWIST_NORM2_B, -1, -1}};
  auto sub_shape = [&](int l, int t, int &rows, int &cols) {
    full_shape(d, t, rows, cols);
    if (const Cut *c = cut_of(d, t)) {
      const PlanEntry &pe = plan->at(l, c->kind);
      const int q = c->kind == TWIST_KIND_HEAD ? d.d_head : d.ffn_granule;
      (c->axis == 0 ? rows : cols) = pe.n_sub * q;
    }
  };
  for (int pass = 0; pass < 2; ++pass) {
    for (int l = 0; l < d.n_layers; ++l) {
      L.heads_sub[l] = plan->at(l, TWIST_KIND_HEAD).n_sub;
      L.ffn_sub[l] = plan->at(l, TWIST_KIND_FFN).n_sub;
      const auto *groups = pass == 0 ? mat_groups : vec_groups;
      const int ng = pass == 0 ? 4 : 8;
      for (int g = 0; g < ng; ++g) {
        pad();
        for (int i = 0; i < 3 && groups[g][i] >= 0; ++i) {
          int t = groups[g][i], r, c;
          if (!layer_tensor_present(d, t)) continue;
          sub_shape(l, t, r, c);
          place(L.layer[(size_t)l * TWIST_N_LAYER_TENSORS + t], r, c);
        }
      }
    }
    for (int t = 0; t < TWIST_N_GLOBAL_TENSORS; ++t) {
      int r, c;
      if (!global_tensor_present(d, t)) continue;
      global_shape(d, t, r, c);
      if ((c > 1) != (pass == 0)) continue;
      pad();
      place(L.global[t], r, c);
    }
    pad();
    if (pass == 0) L.n_matrix = off;
  }
  L.n_total = off;
}

}  // namespace

extern "C" twist_status twist_sample(twist_ctx *ctx, const twist_sample_desc *sd, twist_plan **out) {
  if (!ctx || !sd || !out) TW_FAIL(ctx, TWIST_EINVAL, "twist_sample: null argument");
  if (sd->S < 1 || sd->S > TWIST_MAX_S) TW_FAIL(ctx, TWIST_EINVAL, "twist_sample: S=%d outside [1, %d]", sd->S, TWIST_MAX_S);
  if (sd->scale_mode != TWIST_SCALE_NONE && sd->scale_mode != TWIST_SCALE_SQRT_RATIO) TW_FAIL(ctx, TWIST_EINVAL, "twist_sample: unknown scale_mode");
  const twist_model_desc &d = ctx->d;
  twist_plan *plan = new (std::nothrow) twist_plan;
  if (!plan) TW_FAIL(ctx, TWIST_ENOMEM, "twist_sample: out of host memory");
  plan->ctx = ctx;
  plan->S = sd->S;
  plan->scale_mode = sd->scale_mode;
  plan->e.resize((size_t)d.n_layers * 2);
  bool any_drawn = false;  // false when every layer is kept whole
  for (int l = 0; l < d.n_layers; ++l) any_drawn = any_drawn || !(sd->layer_shared && sd->layer_shared[l]);
  for (int kind = 0; any_drawn && kind < 2; ++kind) {
    const bool head = kind == TWIST_KIND_HEAD;
    twist_status st = check_blueprint_args(ctx, head ? d.n_heads : ctx->n_ffn_units(), sd->S, head ? sd->heads_sub : sd->ffn_units_sub,
                                           head ? sd->common_heads : sd->common_ffn, head ? sd->n_common_heads : sd->n_common_ffn, sd->require_coverage != 0);
    if (st != TWIST_OK) { delete plan; return st; }
  }
  // Every (layer, kind) entry has a draw stream of its own, so the entries are drawn on a few host threads (entry e
  // on thread e mod n); the result does not depend on how many there are.
  const int n_entries = d.n_layers * 2;
  auto draw_entry = [&](int e) {
    const int l = e / 2, kind = e % 2;
    PlanEntry &pe = plan->e[(size_t)e];
    pe.n_full = kind == TWIST_KIND_HEAD ? d.n_heads : ctx->n_ffn_units();
    const bool shared = sd->layer_shared && sd->layer_shared[l];
    if (shared) {
      pe.n_sub = pe.n_full;
      pe.idx.resize((size_t)sd->S * pe.n_full);
      for (int s = 0; s < sd->S; ++s)
        for (int b = 0; b < pe.n_full; ++b) pe.idx[(size_t)s * pe.n_full + b] = b;
    } else {
      pe.n_sub = kind == TWIST_KIND_HEAD ? sd->heads_sub : sd->ffn_units_sub;
      DrawStream rng(sd->seed, sd->round, (uint64_t)l, (uint64_t)kind);
      generate_blueprint(pe.n_full, sd->S, pe.n_sub, kind == TWIST_KIND_HEAD ? sd->common_heads : sd->common_ffn,
                         kind == TWIST_KIND_HEAD ? sd->n_common_heads : sd->n_common_ffn, sd->require_coverage != 0, rng, pe.idx);
    }
    // inverse positions and owner counts
    pe.inv.assign((size_t)sd->S * pe.n_full, -1);
    pe.count.assign(pe.n_full, 0);
    for (int s = 0; s < sd->S; ++s)
      for (int k = 0; k < pe.n_sub; ++k) {
        int32_t u = pe.idx[(size_t)s * pe.n_sub + k];
        pe.inv[(size_t)s * pe.n_full + u] = k;
        pe.count[u] += 1;
      }
  };
  // threads only when there is enough to draw to pay for starting them
  const int64_t draw_work = (int64_t)n_entries * sd->S * ctx->n_ffn_units();
  const int hw = (int)std::thread::hardware_concurrency();
  const int n_threads = draw_work < (1 << 18) ? 1 : std::max(1, std::min({8, hw > 0 ? hw : 1, n_entries}));
  std::atomic<bool> failed{false};
  auto draw_share = [&](int t) {  // entries t, t + n_threads, ...
    try {
      for (int e = t; e < n_entries; e += n_threads) draw_entry(e);
    } catch (...) {
      failed = true;  // out of host memory
    }
  };
  std::vector<std::thread> pool;
  int started = 1;  // share 0 is the calling thread's
  try {
    pool.reserve(n_threads);
    for (; started < n_threads; ++started) pool.emplace_back(draw_share, started);
  } catch (...) {  // no more threads to be had: the caller draws the remaining shares itself
  }
  draw_share(0);
  for (int t = started; t < n_threads; ++t) draw_share(t);
  for (std::thread &th : pool) th.join();
  if (failed) { delete plan; TW_FAIL(ctx, TWIST_ENOMEM, "twist_sample: out of host memory while drawing the blueprints"); }
  size_t table_ints = 0;
  for (const PlanEntry &pe : plan->e) {
    table_ints += pe.idx.size() + pe.inv.size() + pe.count.size();
    table_ints = align_up(table_ints, 64);
  }
  // one device allocation for all tables
  hipError_t e = hipMalloc(reinterpret_cast<void **>(&plan->d_tables), table_ints * sizeof(int32_t));
  if (e != hipSuccess) { delete plan; TW_FAIL(ctx, TWIST_ENOMEM, "twist_sample: hipMalloc of %zu bytes failed: %s", table_ints * 4, hipGetErrorString(e)); }
  std::vector<int32_t> host(table_ints, 0);
  size_t pos = 0;
  for (PlanEntry &pe : plan->e) {
    pe.d_idx = plan->d_tables + pos;   std::copy(pe.idx.begin(), pe.idx.end(), host.begin() + pos);     pos += pe.idx.size();
    pe.d_inv = plan->d_tables + pos;   std::copy(pe.inv.begin(), pe.inv.end(), host.begin() + pos);     pos += pe.inv.size();
    pe.d_count = plan->d_tables + pos; std::copy(pe.count.begin(), pe.count.end(), host.begin() + pos); pos += pe.count.size();
    pos = align_up(pos, 64);
  }
  e = hipMemcpy(plan->d_tables, host.data(), table_ints * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e != hipSuccess) { (void)hipFree(plan->d_tables); delete plan; TW_FAIL(ctx, TWIST_EHIP, "twist_sample: upload failed: %s", hipGetErrorString(e)); }
  build_layout(ctx, plan);
  *out = plan;
  return TWIST_OK;
}

extern "C" twist_status twist_plan_view(const twist_plan *plan, int32_t layer, int32_t kind, const int32_t **idx, const int32_t **inv,
                                        const int32_t **count, int32_t *n_sub, int32_t *n_full, int32_t on_device) {
  if (!plan) TW_FAIL(nullptr, TWIST_EINVAL, "twist_plan_view: null plan");
  if (layer < 0 || layer >= plan->ctx->d.n_layers || kind < 0 || kind > 1) TW_FAIL(plan->ctx, TWIST_EINVAL, "twist_plan_view: layer %d / kind %d out of range", layer, kind);
  const PlanEntry &pe = plan->at(layer, kind);
  if (idx) *idx = on_device ? pe.d_idx : pe.idx.data();
  if (inv) *inv = on_device ? pe.d_inv : pe.inv.data();
  if (count) *count = on_device ? pe.d_count : pe.count.data();
  if (n_sub) *n_sub = pe.n_sub;
  if (n_full) *n_full = pe.n_full;
  return TWIST_OK;
}

extern "C" twist_status twist_plan_read_device(const twist_plan *plan, int32_t layer, int32_t kind, int32_t *idx, int32_t *inv, int32_t *count) {
  if (!plan) TW_FAIL(nullptr, TWIST_EINVAL, "twist_plan_read_device: null plan");
  if (layer < 0 || layer >= plan->ctx->d.n_layers || kind < 0 || kind > 1)
    TW_FAIL(plan->ctx, TWIST_EINVAL, "twist_plan_read_device: layer %d / kind %d out of range", layer, kind);
  const PlanEntry &pe = plan->at(layer, kind);
  if (idx) TW_HIP(plan->ctx, hipMemcpy(idx, pe.d_idx, pe.idx.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
  if (inv) TW_HIP(plan->ctx, hipMemcpy(inv, pe.d_inv, pe.inv.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
  if (count) TW_HIP(plan->ctx, hipMemcpy(count, pe.d_count, pe.count.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
  return TWIST_OK;
}

extern "C" void twist_plan_destroy(twist_plan *plan) {
  if (!plan) return;
  if (plan->d_tables) (void)hipFree(plan->d_tables);
  delete plan;
}

// ------------------------------------------------------------------------------------------------ subnets
static size_t region_bytes(const twist_plan *plan, int esize) { return align_up((size_t)plan->layout.n_total * esize, 256); }

extern "C" twist_status twist_subnet_bytes(twist_ctx *ctx, const twist_plan *plan, int32_t store, size_t *bytes) {
  if (!ctx || !plan || !bytes) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_bytes: null argument");
  if (store < TWIST_STORE_PARAMS || store > TWIST_STORE_ADAMW) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_bytes: unknown store mode %d", store);
  size_t b = region_bytes(plan, ctx->esize());
  const size_t f32 = region_bytes(plan, 4);
  if (store >= TWIST_STORE_GRADS) b += f32 + (ctx->d.dtype == TWIST_BF16 ? f32 : 0);
  if (store >= TWIST_STORE_ADAMW) b += 2 * f32;
  *bytes = b;
  return TWIST_OK;
}

namespace {

// Describe tensor t of layer l (or global t when l < 0) as a MoveJob; returns false if the model lacks it.
bool make_job(const twist_ctx *ctx, const twist_plan *plan, int l, int t, const void *full_ptr, int s, bool for_aggregate, int n_subs, MoveJob &jb) {
  const twist_model_desc &d = ctx->d;
  const Slot &slot = l >= 0 ? plan->layout.at(l, t) : plan->layout.global[t];
  if (slot.off < 0) return false;
  const int es = ctx->esize();
  const int VN = 16 / es;
  jb.full = full_ptr;
  jb.sub_off = slot.off;
  const Cut *c = l >= 0 ? cut_of(d, t) : nullptr;
  int frows, fcols;
  if (l >= 0) full_shape(d, t, frows, fcols); else global_shape(d, t, frows, fcols);
  if (c) {
    const PlanEntry &pe = plan->at(l, c->kind);
    const int q = c->kind == TWIST_KIND_HEAD ? d.d_head : d.ffn_granule;
    jb.n_full = pe.n_full;
    jb.n_sub = pe.n_sub;
    jb.table = for_aggregate ? pe.d_inv : pe.d_idx + (size_t)s * pe.n_sub;
    if (c->axis == 0) { jb.rows = 1; jb.Q = q * fcols; }   // a block of whole rows is one long segment
    else { jb.rows = frows; jb.Q = q; }
  } else {
    jb.n_full = jb.n_sub = 1;
    jb.table = nullptr;
    jb.rows = 1;
    jb.Q = frows * fcols;
  }
  jb.vec = ((int64_t)jb.Q * es) % 16 == 0 && (reinterpret_cast<uintptr_t>(full_ptr) % 16) == 0;
  const int64_t width = (int64_t)(for_aggregate ? jb.n_full : jb.n_sub) * (jb.vec ? jb.Q / VN : jb.Q);
  if (jb.vec && jb.rows == 1 && (jb.Q / VN) % 256 == 0 && (!for_aggregate || n_subs <= 8)) {
    jb.vec = 2;
    jb.tile_u = for_aggregate ? 2 : 8;
    jb.tile_rows = 1;
  } else if (jb.vec && for_aggregate) {
    // the pull keeps up to 8 subnets' vectors per output vector in registers: fewer vectors per thread
    jb.tile_u = jb.rows == 1 ? (width >= 1024 ? 4 : (width >= 512 ? 2 : 1)) : (width >= 512 ? 2 : 1);
    jb.tile_rows = jb.tile_u == 4 ? 1 : (jb.tile_u == 2 ? (jb.rows > 1 ? 2 : 1) : 4);
  } else if (jb.vec) {
    jb.tile_u = width >= 1024 ? 4 : (width >= 512 ? 2 : 1);
    jb.tile_rows = 4 / jb.tile_u;
  } else {
    jb.tile_u = 2;
    // element path: the pull's per-tile set-up (16 table look-ups per thread, span bounds through LDS) is paid once per tile, so its
    // tiles are tall (128 rows: 12.2 instead of 14.4 ms for the [out, in] aggregate of the 7B-shaped stack); the gather's are not
    jb.tile_rows = std::min(for_aggregate ? 128 : 32, jb.rows);
  }
  jb.tiles_per_row = (int32_t)((width + 256 * jb.tile_u - 1) / (256 * jb.tile_u));
  return true;
}

int job_blocks(const MoveJob &jb) { return jb.tiles_per_row * ((jb.rows + jb.tile_rows - 1) / jb.tile_rows); }

twist_status check_full(twist_ctx *ctx, const twist_full_weights *full, const char *who) {
  if (!full || !full->layer_tensors) TW_FAIL(ctx, TWIST_EINVAL, "%s: null weights", who);
  const twist_model_desc &d = ctx->d;
  for (int l = 0; l < d.n_layers; ++l)
    for (int t = 0; t < TWIST_N_LAYER_TENSORS; ++t)
      if (layer_tensor_present(d, t) && !full->layer_tensors[(size_t)l * TWIST_N_LAYER_TENSORS + t])
        TW_FAIL(ctx, TWIST_EINVAL, "%s: layer %d tensor %d is required by this model but NULL", who, l, t);
  for (int t = 0; t < TWIST_N_GLOBAL_TENSORS; ++t)
    if (global_tensor_present(d, t) && !full->global_tensors[t]) TW_FAIL(ctx, TWIST_EINVAL, "%s: model-level tensor %d is required but NULL", who, t);
  return TWIST_OK;
}

// Run `launch` over the model-level tensors and every layer, as many whole layers per launch as the job table holds.
// When aggregating, the row-block jobs, the other 16-byte jobs and the element-path jobs go into launches of their own
// (each kind has a kernel of its own).
enum JobFilter { JOBS_ALL = 0, JOBS_ROW_BLOCKS = 1, JOBS_NOT_ROW_BLOCKS = 2 };
template <class F>
twist_status for_each_group(twist_ctx *ctx, const twist_plan *plan, const twist_full_weights *full, int s, bool for_aggregate, MoveLaunch &ml, F launch,
                            JobFilter filter = JOBS_ALL) {
  const twist_model_desc &d = ctx->d;
  for (int pass = 0; pass < (for_aggregate ? 3 : 1); ++pass) {
    ml.n_jobs = 0;
    int64_t blocks = 0;
    auto flush = [&]() -> twist_status {
      twist_status st = ml.n_jobs ? launch(ml, (int)blocks) : TWIST_OK;
      ml.n_jobs = 0;
      blocks = 0;
      return st;
    };
    for (int l = -1; l < d.n_layers; ++l) {
      const int nt = l < 0 ? TWIST_N_GLOBAL_TENSORS : TWIST_N_LAYER_TENSORS;
      if (ml.n_jobs + nt > TWIST_MAX_JOBS || blocks > (1 << 30)) TW_TRY(flush());
      for (int t = 0; t < nt; ++t) {
        const void *fp = l < 0 ? full->global_tensors[t] : full->layer_tensors[(size_t)l * TWIST_N_LAYER_TENSORS + t];
        MoveJob &jb = ml.job[ml.n_jobs];
        if (!make_job(ctx, plan, l, t, fp, s, for_aggregate, ml.n_subs, jb)) continue;
        if (for_aggregate && jb.vec != 2 - pass) continue;
        if ((filter == JOBS_ROW_BLOCKS && jb.vec != 2) || (filter == JOBS_NOT_ROW_BLOCKS && jb.vec == 2)) continue;
        jb.blk_begin = (int32_t)blocks;
        ml.blk_begin[ml.n_jobs] = jb.blk_begin;
        blocks += job_blocks(jb);
        ++ml.n_jobs;
      }
    }
    TW_TRY(flush());
  }
  return TWIST_OK;
}

}  // namespace

namespace {

// checks and the subnet object over caller storage (no device work)
twist_status bind_subnet(twist_ctx *ctx, const twist_plan *plan, int32_t s, void *storage, size_t storage_bytes, int32_t store, const char *who,
                         twist_subnet **out) {
  if (s < 0 || s >= plan->S) TW_FAIL(ctx, TWIST_EINVAL, "%s: subnet %d outside [0, %d)", who, s, plan->S);
  size_t need;
  TW_TRY(twist_subnet_bytes(ctx, plan, store, &need));
  if (storage_bytes < need) TW_FAIL(ctx, TWIST_ESHAPE, "%s: storage of %zu bytes is smaller than the %zu needed", who, storage_bytes, need);
  if (reinterpret_cast<uintptr_t>(storage) % 256) TW_FAIL(ctx, TWIST_ESHAPE, "%s: storage must be 256-byte aligned", who);
  twist_subnet *sub = new (std::nothrow) twist_subnet;
  if (!sub) TW_FAIL(ctx, TWIST_ENOMEM, "%s: out of host memory", who);
  sub->ctx = ctx; sub->plan = plan; sub->s = s; sub->store = store;
  sub->base = static_cast<char *>(storage);
  const size_t pb = region_bytes(plan, ctx->esize()), fb = region_bytes(plan, 4);
  char *p = sub->base;
  sub->params = p; p += pb;
  if (store >= TWIST_STORE_GRADS) {
    if (ctx->d.dtype == TWIST_BF16) { sub->master = reinterpret_cast<float *>(p); p += fb; }
    sub->grads = reinterpret_cast<float *>(p); p += fb;
  }
  if (store >= TWIST_STORE_ADAMW) {
    sub->adam_m = reinterpret_cast<float *>(p); p += fb;
    sub->adam_v = reinterpret_cast<float *>(p); p += fb;
  }
  *out = sub;
  return TWIST_OK;
}

// After the weights are in place: the fp32 master copy.  The gradient region is not cleared (twist_subnet_fwd_bwd
// overwrites every gradient) and neither are the AdamW moments: the first step of a subnet takes them as zero without
// reading them (twist_adamw with step = 1), which saves three sweeps over the subnet per extract.
twist_status finish_subnet(twist_ctx *ctx, const twist_plan *plan, twist_subnet *sub) {
  if (sub->master) TW_TRY(twist_launch_to_f32(ctx, sub->params, sub->master, plan->layout.n_total));
  return TWIST_OK;
}

}  // namespace

extern "C" twist_status twist_extract(twist_ctx *ctx, const twist_plan *plan, const twist_full_weights *full, int32_t s, void *storage,
                                      size_t storage_bytes, int32_t store, twist_subnet **out) {
  if (!ctx || !plan || !storage || !out) TW_FAIL(ctx, TWIST_EINVAL, "twist_extract: null argument");
  if (plan->ctx != ctx) TW_FAIL(ctx, TWIST_EINVAL, "twist_extract: plan belongs to another context");
  if (s < 0 || s >= plan->S) TW_FAIL(ctx, TWIST_EINVAL, "twist_extract: subnet %d outside [0, %d)", s, plan->S);
  TW_TRY(check_full(ctx, full, "twist_extract"));
  twist_subnet *sub = nullptr;
  TW_TRY(bind_subnet(ctx, plan, s, storage, storage_bytes, store, "twist_extract", &sub));
  // The few elements of padding between tensors are never read by any kernel except the optimizer
  // sweeps, whose results there are never used, so the weight slab is not cleared (clearing it would
  // add a full extra write of the subnet).
  MoveLaunch ml;
  std::memset(&ml, 0, sizeof ml);
  ml.sub_base[0] = sub->params;
  twist_status st = for_each_group(ctx, plan, full, s, false, ml, [&](const MoveLaunch &m, int blocks) { return twist_launch_extract(ctx, m, blocks); });
  if (st == TWIST_OK) st = finish_subnet(ctx, plan, sub);
  if (st != TWIST_OK) { delete sub; return st; }
  *out = sub;
  return TWIST_OK;
}

extern "C" twist_status twist_extract_all(twist_ctx *ctx, const twist_plan *plan, const twist_full_weights *full, void *const *storages,
                                          size_t storage_bytes, int32_t store, twist_subnet **out) {
  if (!ctx || !plan || !storages || !out) TW_FAIL(ctx, TWIST_EINVAL, "twist_extract_all: null argument");
  if (plan->ctx != ctx) TW_FAIL(ctx, TWIST_EINVAL, "twist_extract_all: plan belongs to another context");
  TW_TRY(check_full(ctx, full, "twist_extract_all"));
  const int S = plan->S;
  for (int s = 0; s < S; ++s)
    if (!storages[s]) TW_FAIL(ctx, TWIST_EINVAL, "twist_extract_all: storage %d is NULL", s);
  std::vector<twist_subnet *> subs(S, nullptr);
  twist_status st = TWIST_OK;
  for (int s = 0; s < S && st == TWIST_OK; ++s) st = bind_subnet(ctx, plan, s, storages[s], storage_bytes, store, "twist_extract_all", &subs[s]);
  const bool fused = S <= 8;  // the one-pass kernel keeps up to 8 destinations per group of central vectors
  if (st == TWIST_OK && fused) {
    // tensors cut into blocks of whole rows (and the shared matrices): one pass over the central tensor writes every subnet
    MoveLaunch ml;
    std::memset(&ml, 0, sizeof ml);
    ml.n_subs = S;
    for (int s = 0; s < S; ++s) { ml.sub_base[s] = subs[s]->params; ml.sub_row[s] = s; }
    st = for_each_group(ctx, plan, full, 0, true, ml, [&](const MoveLaunch &m, int blocks) { return twist_launch_extract_all(ctx, m, blocks); },
                        JOBS_ROW_BLOCKS);
  }
  for (int s = 0; s < S && st == TWIST_OK; ++s) {  // everything else (or everything, beyond 8 subnets): per-subnet gathers
    MoveLaunch ml;
    std::memset(&ml, 0, sizeof ml);
    ml.n_subs = S;  // same job classification as above
    ml.sub_base[0] = subs[s]->params;
    st = for_each_group(ctx, plan, full, s, false, ml, [&](const MoveLaunch &m, int blocks) { return twist_launch_extract(ctx, m, blocks); },
                        fused ? JOBS_NOT_ROW_BLOCKS : JOBS_ALL);
    if (st == TWIST_OK) st = finish_subnet(ctx, plan, subs[s]);
  }
  if (st != TWIST_OK) {
    for (twist_subnet *p : subs) delete p;
    return st;
  }
  for (int s = 0; s < S; ++s) out[s] = subs[s];
  return TWIST_OK;
}

extern "C" twist_status twist_subnet_view(const twist_subnet *sub, int32_t layer, int32_t tensor, int32_t what, void **dev, int64_t shape[2]) {
  if (!sub || !dev || !shape) TW_FAIL(sub ? sub->ctx : nullptr, TWIST_EINVAL, "twist_subnet_view: null argument");
  twist_ctx *ctx = sub->ctx;
  const int nl = ctx->d.n_layers;
  if (layer < -1 || layer >= nl || tensor < 0 || tensor >= (layer < 0 ? TWIST_N_GLOBAL_TENSORS : TWIST_N_LAYER_TENSORS))
    TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_view: layer %d / tensor %d out of range", layer, tensor);
  const Slot &slot = layer < 0 ? sub->plan->layout.global[tensor] : sub->plan->layout.at(layer, tensor);
  if (slot.off < 0) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_view: this model has no such tensor (layer %d, tensor %d)", layer, tensor);
  if (what == TWIST_PARAM) *dev = sub->params + slot.off * ctx->esize();
  else if (what == TWIST_GRAD) {
    if (!sub->grads) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_view: subnet was extracted without gradient storage");
    *dev = sub->grads + slot.off;
  } else if (what == TWIST_MASTER) {
    // fp32 models keep no separate master copy: the parameters are the fp32 weights the optimizer updates
    if (ctx->d.dtype == TWIST_BF16 && !sub->master) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_view: subnet was extracted without master weights");
    *dev = ctx->d.dtype == TWIST_BF16 ? static_cast<void *>(sub->master + slot.off) : static_cast<void *>(sub->params + slot.off * 4);
  } else if (what == TWIST_ADAM_M || what == TWIST_ADAM_V) {
    if (!sub->adam_m) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_view: subnet was extracted without AdamW moments");
    if (sub->step_count == 0) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_view: the AdamW moments hold nothing before the first step");
    *dev = (what == TWIST_ADAM_M ? sub->adam_m : sub->adam_v) + slot.off;
  } else TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_view: unknown selector %d", what);
  shape[0] = slot.rows;
  shape[1] = slot.cols;
  return TWIST_OK;
}

extern "C" void twist_subnet_destroy(twist_subnet *sub) { delete sub; }

extern "C" twist_status twist_aggregate(twist_ctx *ctx, const twist_plan *plan, twist_subnet *const *subs, int32_t n_subs, const twist_full_weights *inout) {
  if (!ctx || !plan || !subs) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate: null argument");
  if (plan->ctx != ctx) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate: plan belongs to another context");
  if (n_subs < 1 || n_subs > plan->S) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate: n_subs=%d outside [1, S=%d]", n_subs, plan->S);
  TW_TRY(check_full(ctx, inout, "twist_aggregate"));
  MoveLaunch ml;
  std::memset(&ml, 0, sizeof ml);
  ml.n_subs = n_subs;
  for (int i = 0; i < n_subs; ++i) {
    if (!subs[i] || subs[i]->plan != plan) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate: subnet %d was not extracted from this plan", i);
    for (int k = 0; k < i; ++k)
      if (subs[k]->s == subs[i]->s) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate: blueprint row %d passed twice", subs[i]->s);
    ml.sub_base[i] = subs[i]->params;
    ml.sub_row[i] = subs[i]->s;
  }
  return for_each_group(ctx, plan, inout, 0, true, ml, [&](const MoveLaunch &m, int blocks) { return twist_launch_aggregate(ctx, m, blocks); });
}

// ------------------------------------------------------------------------------------------------ running-sum aggregate
struct twist_accum {
  twist_ctx *ctx = nullptr;
  const twist_plan *plan = nullptr;
  float *base = nullptr;
  std::vector<int64_t> layer_off;                 // [n_layers * TWIST_N_LAYER_TENSORS] element offsets, -1 = absent
  int64_t global_off[TWIST_N_GLOBAL_TENSORS];
  int32_t rows[TWIST_MAX_S];                      // blueprint rows added so far, in order
  int32_t n_rows = 0;
};

namespace {

// Offsets of every central tensor inside the fp32 image (each tensor starts on a 256-byte boundary); returns the
// image's size in elements.
int64_t image_layout(const twist_model_desc &d, std::vector<int64_t> *layer_off, int64_t *global_off) {
  int64_t n = 0;
  int r, c;
  if (layer_off) layer_off->assign((size_t)d.n_layers * TWIST_N_LAYER_TENSORS, -1);
  for (int l = 0; l < d.n_layers; ++l)
    for (int t = 0; t < TWIST_N_LAYER_TENSORS; ++t) {
      if (!layer_tensor_present(d, t)) continue;
      full_shape(d, t, r, c);
      if (layer_off) (*layer_off)[(size_t)l * TWIST_N_LAYER_TENSORS + t] = n;
      n += (int64_t)align_up((size_t)r * c, 64);
    }
  for (int t = 0; t < TWIST_N_GLOBAL_TENSORS; ++t) {
    if (global_off) global_off[t] = -1;
    if (!global_tensor_present(d, t)) continue;
    global_shape(d, t, r, c);
    if (global_off) global_off[t] = n;
    n += (int64_t)align_up((size_t)r * c, 64);
  }
  return n;
}

// Launches over the central layout, as many whole layers per launch as the job table holds.  `full` is null for an add.
twist_status for_each_image_group(twist_accum *acc, const twist_full_weights *full, MoveLaunch &ml, bool finish) {
  twist_ctx *ctx = acc->ctx;
  const twist_model_desc &d = ctx->d;
  const int VN = 16 / ctx->esize();
  ml.n_jobs = 0;
  int64_t blocks = 0;
  auto flush = [&]() -> twist_status {
    twist_status st = ml.n_jobs ? twist_launch_accumulate(ctx, ml, (int)blocks, finish) : TWIST_OK;
    ml.n_jobs = 0;
    blocks = 0;
    return st;
  };
  for (int l = -1; l < d.n_layers; ++l) {
    const int nt = l < 0 ? TWIST_N_GLOBAL_TENSORS : TWIST_N_LAYER_TENSORS;
    if (ml.n_jobs + nt > TWIST_MAX_JOBS || blocks > (1 << 30)) TW_TRY(flush());
    for (int t = 0; t < nt; ++t) {
      const int64_t off = l < 0 ? acc->global_off[t] : acc->layer_off[(size_t)l * TWIST_N_LAYER_TENSORS + t];
      if (off < 0) continue;
      float *img = acc->base + off;
      const void *fp = finish ? (l < 0 ? full->global_tensors[t] : full->layer_tensors[(size_t)l * TWIST_N_LAYER_TENSORS + t]) : img;
      MoveJob &jb = ml.job[ml.n_jobs];
      if (!make_job(ctx, acc->plan, l, t, fp, 0, true, ml.n_subs, jb)) continue;
      if (jb.vec) jb.vec = 1;
      jb.acc = img;
      const int64_t total = (int64_t)jb.rows * jb.n_full * (jb.vec ? jb.Q / VN : jb.Q);
      if (total >= (int64_t)1 << 31) TW_FAIL(ctx, TWIST_ESHAPE, "running-sum aggregate: a tensor of %lld vectors exceeds the 32-bit index range", (long long)total);
      jb.blk_begin = (int32_t)blocks;
      ml.blk_begin[ml.n_jobs] = jb.blk_begin;
      blocks += (total + kAccumPerBlock - 1) / kAccumPerBlock;
      ++ml.n_jobs;
    }
  }
  return flush();
}

}  // namespace

extern "C" twist_status twist_aggregate_image_bytes(twist_ctx *ctx, size_t *bytes) {
  if (!ctx || !bytes) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate_image_bytes: null argument");
  *bytes = (size_t)image_layout(ctx->d, nullptr, nullptr) * sizeof(float);
  return TWIST_OK;
}

extern "C" twist_status twist_aggregate_begin(twist_ctx *ctx, const twist_plan *plan, void *image, size_t image_bytes, twist_accum **out) {
  if (!ctx || !plan || !image || !out) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate_begin: null argument");
  if (plan->ctx != ctx) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate_begin: plan belongs to another context");
  if (reinterpret_cast<uintptr_t>(image) % 256) TW_FAIL(ctx, TWIST_ESHAPE, "twist_aggregate_begin: image must be 256-byte aligned");
  twist_accum *acc = new (std::nothrow) twist_accum;
  if (!acc) TW_FAIL(ctx, TWIST_ENOMEM, "twist_aggregate_begin: out of host memory");
  acc->ctx = ctx; acc->plan = plan; acc->base = static_cast<float *>(image);
  const size_t need = (size_t)image_layout(ctx->d, &acc->layer_off, acc->global_off) * sizeof(float);
  if (image_bytes < need) {
    delete acc;
    TW_FAIL(ctx, TWIST_ESHAPE, "twist_aggregate_begin: image of %zu bytes is smaller than the %zu needed", image_bytes, need);
  }
  *out = acc;
  return TWIST_OK;
}

extern "C" twist_status twist_aggregate_add(twist_accum *acc, const twist_subnet *sub) {
  if (!acc || !sub) TW_FAIL(acc ? acc->ctx : nullptr, TWIST_EINVAL, "twist_aggregate_add: null argument");
  twist_ctx *ctx = acc->ctx;
  if (sub->plan != acc->plan) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate_add: subnet was not extracted from this plan");
  for (int i = 0; i < acc->n_rows; ++i)
    if (acc->rows[i] == sub->s) TW_FAIL(ctx, TWIST_EINVAL, "twist_aggregate_add: blueprint row %d added twice", sub->s);
  MoveLaunch ml;
  std::memset(&ml, 0, sizeof ml);
  ml.n_subs = acc->n_rows + 1;
  ml.sub_base[0] = sub->params;
  ml.sub_row[0] = sub->s;
  for (int i = 0; i < acc->n_rows; ++i) ml.sub_row[1 + i] = acc->rows[i];
  TW_TRY(for_each_image_group(acc, nullptr, ml, false));
  acc->rows[acc->n_rows++] = sub->s;
  return TWIST_OK;
}

extern "C" twist_status twist_aggregate_finish(twist_accum *acc, const twist_full_weights *inout) {
  if (!acc) TW_FAIL(nullptr, TWIST_EINVAL, "twist_aggregate_finish: null argument");
  twist_ctx *ctx = acc->ctx;
  TW_TRY(check_full(ctx, inout, "twist_aggregate_finish"));
  if (acc->n_rows == 0) return TWIST_OK;  // nothing reported: the central model stays
  MoveLaunch ml;
  std::memset(&ml, 0, sizeof ml);
  ml.n_subs = acc->n_rows;
  for (int i = 0; i < acc->n_rows; ++i) ml.sub_row[i] = acc->rows[i];
  TW_TRY(for_each_image_group(acc, inout, ml, true));
  acc->n_rows = 0;
  return TWIST_OK;
}

extern "C" void twist_aggregate_destroy(twist_accum *acc) { delete acc; }

// ------------------------------------------------------------------------------------------------ one whole round
namespace {
size_t batch_elems(const twist_ctx *ctx, int B, int N) { return (size_t)B * N * (ctx->d.vocab > 0 ? 1 : ctx->d.d_model); }
size_t batch_esize(const twist_ctx *ctx) { return ctx->d.vocab > 0 ? sizeof(int32_t) : (size_t)ctx->esize(); }
int store_of(const twist_opt_desc &o) { return o.kind == TWIST_OPT_ADAMW ? TWIST_STORE_ADAMW : TWIST_STORE_GRADS; }
}  // namespace

extern "C" twist_status twist_round_bytes(twist_ctx *ctx, const twist_round_desc *rd, size_t *subnet_bytes, size_t *workspace_bytes,
                                          size_t *image_bytes) {
  if (!ctx || !rd || !subnet_bytes || !workspace_bytes || !image_bytes) TW_FAIL(ctx, TWIST_EINVAL, "twist_round_bytes: null argument");
  // Sizes depend on the widths only, not on the draw: a plan without tables (host object only, nothing sampled,
  // nothing allocated on the device) carries the subnet layout the two size queries read.
  const twist_sample_desc &sd = rd->sample;
  const twist_model_desc &d = ctx->d;
  if (sd.S < 1 || sd.S > TWIST_MAX_S) TW_FAIL(ctx, TWIST_EINVAL, "twist_round_bytes: S=%d outside [1, %d]", sd.S, TWIST_MAX_S);
  twist_plan widths;
  widths.ctx = ctx;
  widths.S = sd.S;
  widths.e.resize((size_t)d.n_layers * 2);
  bool any_drawn = false;
  for (int l = 0; l < d.n_layers; ++l) any_drawn = any_drawn || !(sd.layer_shared && sd.layer_shared[l]);
  for (int kind = 0; any_drawn && kind < 2; ++kind) {
    const bool head = kind == TWIST_KIND_HEAD;
    TW_TRY(check_blueprint_args(ctx, head ? d.n_heads : ctx->n_ffn_units(), sd.S, head ? sd.heads_sub : sd.ffn_units_sub,
                                head ? sd.common_heads : sd.common_ffn, head ? sd.n_common_heads : sd.n_common_ffn, sd.require_coverage != 0));
  }
  for (int l = 0; l < d.n_layers; ++l)
    for (int kind = 0; kind < 2; ++kind) {
      PlanEntry &pe = widths.e[(size_t)l * 2 + kind];
      pe.n_full = kind == TWIST_KIND_HEAD ? d.n_heads : ctx->n_ffn_units();
      pe.n_sub = (sd.layer_shared && sd.layer_shared[l]) ? pe.n_full : (kind == TWIST_KIND_HEAD ? sd.heads_sub : sd.ffn_units_sub);
    }
  build_layout(ctx, &widths);
  size_t sb = 0, wb = 0, ib = 0;
  twist_status st = twist_subnet_bytes(ctx, &widths, store_of(rd->opt), &sb);
  if (st == TWIST_OK) {
    twist_subnet probe;
    probe.ctx = ctx; probe.plan = &widths;
    st = twist_train_workspace_bytes(ctx, &probe, rd->B, rd->N, &wb);
  }
  if (st == TWIST_OK) st = twist_aggregate_image_bytes(ctx, &ib);
  if (st != TWIST_OK) return st;
  *subnet_bytes = sb; *workspace_bytes = wb; *image_bytes = ib;
  return TWIST_OK;
}

extern "C" twist_status twist_round(twist_ctx *ctx, const twist_round_desc *rd, const twist_full_weights *inout, const void *inputs,
                                    const void *targets, void *subnet_storage, size_t subnet_bytes, void *workspace, size_t workspace_bytes,
                                    void *image, size_t image_bytes, float *loss_dev) {
  if (!ctx || !rd || !inputs || !targets || !subnet_storage || !workspace || !image || !loss_dev) TW_FAIL(ctx, TWIST_EINVAL, "twist_round: null argument");
  if (rd->local_steps < 1) TW_FAIL(ctx, TWIST_EINVAL, "twist_round: local_steps=%d must be at least 1", rd->local_steps);
  TW_TRY(check_full(ctx, inout, "twist_round"));
  twist_plan *plan = nullptr;
  TW_TRY(twist_sample(ctx, &rd->sample, &plan));
  twist_accum *acc = nullptr;
  twist_status st = twist_aggregate_begin(ctx, plan, image, image_bytes, &acc);
  const size_t step_bytes = batch_elems(ctx, rd->B, rd->N) * batch_esize(ctx);
  for (int s = 0; st == TWIST_OK && s < plan->S; ++s) {
    twist_subnet *sub = nullptr;
    st = twist_extract(ctx, plan, inout, s, subnet_storage, subnet_bytes, store_of(rd->opt), &sub);
    for (int j = 0; st == TWIST_OK && j < rd->local_steps; ++j) {
      const size_t b = (size_t)s * rd->local_steps + j;
      st = twist_train_fwd_bwd(ctx, sub, static_cast<const char *>(inputs) + b * step_bytes, static_cast<const char *>(targets) + b * step_bytes,
                               rd->B, rd->N, workspace, workspace_bytes, loss_dev + b);
      if (st == TWIST_OK) st = twist_train_step(ctx, sub, &rd->opt);
    }
    if (st == TWIST_OK) st = twist_aggregate_add(acc, sub);
    twist_subnet_destroy(sub);
  }
  if (st == TWIST_OK) st = twist_aggregate_finish(acc, inout);
  // the plan's device tables are read by kernels still in flight: drain the stream before releasing them
  if (hipStreamSynchronize(ctx->stream) != hipSuccess && st == TWIST_OK) st = TWIST_EHIP;
  twist_aggregate_destroy(acc);
  twist_plan_destroy(plan);
  return st;
}

// ------------------------------------------------------------------------------------------------ training entry points
extern "C" twist_status twist_workspace_bytes(twist_ctx *ctx, const twist_subnet *sub, int32_t B, int32_t N, size_t *bytes) {
  if (!ctx || !sub || !bytes) TW_FAIL(ctx, TWIST_EINVAL, "twist_workspace_bytes: null argument");
  return twist_train_workspace_bytes(ctx, sub, B, N, bytes);
}

extern "C" twist_status twist_subnet_fwd_bwd(twist_ctx *ctx, twist_subnet *sub, const void *inputs, const void *targets, int32_t B, int32_t N,
                                             void *workspace, size_t workspace_bytes, float *loss_dev) {
  if (!ctx || !sub || !inputs || !targets || !workspace || !loss_dev) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_fwd_bwd: null argument");
  if (sub->ctx != ctx) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_fwd_bwd: subnet belongs to another context");
  return twist_train_fwd_bwd(ctx, sub, inputs, targets, B, N, workspace, workspace_bytes, loss_dev);
}

extern "C" twist_status twist_subnet_fwd_bwd_masked(twist_ctx *ctx, twist_subnet *full_sub, const twist_plan *plan, int32_t s, const void *inputs,
                                                    const void *targets, int32_t B, int32_t N, void *workspace, size_t workspace_bytes, float *loss_dev) {
  if (!ctx || !full_sub || !plan || !inputs || !targets || !workspace || !loss_dev) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_fwd_bwd_masked: null argument");
  if (full_sub->ctx != ctx || plan->ctx != ctx) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_fwd_bwd_masked: subnet or plan belongs to another context");
  if (s < 0 || s >= plan->S) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_fwd_bwd_masked: blueprint row %d outside [0, %d)", s, plan->S);
  return twist_train_fwd_bwd(ctx, full_sub, inputs, targets, B, N, workspace, workspace_bytes, loss_dev, false, plan, s);
}

extern "C" twist_status twist_subnet_forward(twist_ctx *ctx, twist_subnet *sub, const void *inputs, const void *targets, int32_t B, int32_t N,
                                             void *workspace, size_t workspace_bytes, float *loss_dev) {
  if (!ctx || !sub || !inputs || !targets || !workspace || !loss_dev) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_forward: null argument");
  if (sub->ctx != ctx) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_forward: subnet belongs to another context");
  return twist_train_fwd_bwd(ctx, sub, inputs, targets, B, N, workspace, workspace_bytes, loss_dev, true);
}

extern "C" twist_status twist_subnet_step(twist_ctx *ctx, twist_subnet *sub, const twist_opt_desc *opt) {
  if (!ctx || !sub || !opt) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_step: null argument");
  if (sub->ctx != ctx) TW_FAIL(ctx, TWIST_EINVAL, "twist_subnet_step: subnet belongs to another context");
  return twist_train_step(ctx, sub, opt);
}
