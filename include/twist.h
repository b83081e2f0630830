/*
 * twist.h - C ABI of the TwIST hot path on one AMD MI355X (gfx950).
 *
 * One training round of "Transformers with Independent Subnetwork Training" on one device:
 *
 *     twist_sample  ->  twist_extract (x S)  ->  { twist_subnet_fwd_bwd, twist_subnet_step }*  ->  twist_aggregate
 *
 * i.e. the subnet generator (Section 3.1, Algorithm 1), the dispatcher (Section 3.2), local training of
 * each physically smaller dense subnet ("True TwIST", Section 4.1, with the activation-shift correction of
 * Section 3.4) and the aggregator (Section 3.3).  The S subnets a cluster would spread over workers are
 * run back-to-back on the one GPU.
 *
 * Conventions
 *  - Every call returns a twist_status; nothing throws or aborts across this boundary.  On error the
 *    out-parameters are left untouched and twist_last_error() describes the failure.
 *  - "dev" pointers are HIP device pointers, "host" pointers ordinary host memory.  The library never
 *    takes ownership of caller memory: full weights, subnet storage, workspace, inputs, targets and the
 *    loss scalar stay owned by the caller (normally torch tensors) and must outlive the calls and the
 *    handles that reference them.  The library owns only its handles (ctx, plan, subnet) and the small
 *    index tables inside a plan, all released by the matching *_destroy call.
 *  - All device work is enqueued on the HIP stream given to twist_create, asynchronously; calls do not
 *    synchronise unless stated.
 *  - Matrices are row-major [out_features, in_features]; element type is desc.dtype (fp32 or bf16).
 *    A block ("unit") of kind TWIST_KIND_HEAD is one attention head: d_head rows of W^Q, W^K, W^V and of
 *    their biases, and d_head columns of C^attn.  A block of kind TWIST_KIND_FFN is ffn_granule rows of
 *    W^ffn (and of the gate matrix and the first bias) and ffn_granule columns of C^ffn.  Everything else
 *    (output biases, norms, embeddings, final projection) is shared by all subnets (Section 3.1).
 */
#ifndef TWIST_H
#define TWIST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TWIST_API __attribute__((visibility("default")))

typedef enum {
  TWIST_OK = 0,
  TWIST_EINVAL = 1,      /* bad argument (null pointer, unknown enum, out-of-range index)           */
  TWIST_ECONSTRAINT = 2, /* the size bound of Section 3.1 is violated                               */
  TWIST_ESHAPE = 3,      /* a shape the kernels do not support, or a buffer that is too small        */
  TWIST_ENOMEM = 4,      /* host or device allocation failed                                        */
  TWIST_EHIP = 5         /* a HIP runtime call failed                                                */
} twist_status;

enum { TWIST_F32 = 0, TWIST_BF16 = 1 };                            /* desc.dtype        */
enum { TWIST_ACT_GELU_TANH = 0, TWIST_ACT_RELU = 1, TWIST_ACT_SWIGLU = 2 }; /* desc.act  */
enum { TWIST_NORM_LN = 0, TWIST_NORM_RMS = 1 };                    /* desc.norm         */
enum { TWIST_KIND_HEAD = 0, TWIST_KIND_FFN = 1 };                  /* block kinds       */
enum { TWIST_SCALE_NONE = 0, TWIST_SCALE_SQRT_RATIO = 1 };         /* sample.scale_mode */
enum { TWIST_OPT_SGD = 0, TWIST_OPT_ADAMW = 1 };
/* twist_subnet_view `what`: the weights in desc.dtype; the fp32 gradient; the fp32 weights the optimizer updates (bf16
 * models: the master copy; fp32 models: the weights themselves); the two fp32 AdamW moment estimates */
enum { TWIST_PARAM = 0, TWIST_GRAD = 1, TWIST_MASTER = 2, TWIST_ADAM_M = 3, TWIST_ADAM_V = 4 };
/* storage a subnet needs: weights only; + fp32 gradients (and fp32 master weights for bf16 models);
 * + the two AdamW moment buffers. */
enum { TWIST_STORE_PARAMS = 0, TWIST_STORE_GRADS = 1, TWIST_STORE_ADAMW = 2 };

/* per-layer tensors, in the order of twist_full_weights.layer_tensors */
enum {
  TWIST_WQ = 0, TWIST_WK, TWIST_WV, TWIST_WO, TWIST_W_GATE, TWIST_W_UP, TWIST_W_DOWN,
  TWIST_BQ, TWIST_BK, TWIST_BV, TWIST_BO, TWIST_B_UP, TWIST_B_DOWN,
  TWIST_NORM1_W, TWIST_NORM1_B, TWIST_NORM2_W, TWIST_NORM2_B,
  TWIST_N_LAYER_TENSORS
};
/* model-level tensors, all shared */
enum {
  TWIST_TOK_EMBED = 0, TWIST_POS_EMBED, TWIST_FINAL_NORM_W, TWIST_FINAL_NORM_B, TWIST_LM_HEAD,
  TWIST_N_GLOBAL_TENSORS
};

/* The central model's shape (Section 2, "Problem formulation"; Appendix A.1-A.2 for the layer). */
typedef struct {
  int32_t n_layers, d_model, n_heads, d_head, d_ff;
  int32_t ffn_granule; /* neurons per FFN block, d_ff / R                                            */
  int32_t vocab;       /* 0 = block-stack mode: activations in, mean-squared-error loss, no embedding */
  int32_t max_seq;
  int32_t act, norm;
  int32_t has_bias;    /* linear layers carry biases (GPT-style)                                     */
  int32_t tied_head;   /* final projection shares the token embedding                                */
  int32_t use_rope;    /* rotary positions on Q,K (half-split pairing) instead of learned positions  */
  int32_t dtype;
  int32_t out_unit_major; /* storage of the two output projections C^attn (TWIST_WO) and C^ffn (TWIST_W_DOWN), in the
                           * central model and in every subnet.  0: [d_model, H*d_head] and [d_model, d_ff]
                           * ([out, in] like every other matrix; their blocks are columns).  1: unit-major,
                           * [H*d_head, d_model] and [d_ff, d_model] (the orientation of Section 2's C^attn): their
                           * blocks are rows, so every partitioned tensor is gathered and averaged in whole rows. */
  float norm_eps, rope_theta;
} twist_model_desc;

/* Device pointers of the central model.  layer_tensors is a HOST array of n_layers*TWIST_N_LAYER_TENSORS
 * device pointers (layer-major); entries the architecture does not have are NULL. */
typedef struct {
  void *const *layer_tensors;
  void *global_tensors[TWIST_N_GLOBAL_TENSORS];
} twist_full_weights;

/* Inputs of Algorithm 1, for every layer and both block kinds. */
typedef struct {
  int32_t S;                   /* number of subnets                                                  */
  int32_t heads_sub;           /* N_sub for attention heads                                          */
  int32_t ffn_units_sub;       /* N_sub for FFN blocks                                               */
  const int32_t *common_heads; /* host, sorted unique, may be NULL when n_common_heads == 0          */
  int32_t n_common_heads;
  const int32_t *common_ffn;   /* host                                                               */
  int32_t n_common_ffn;
  const uint8_t *layer_shared; /* host [n_layers] or NULL; non-zero = layer kept whole in every subnet */
  int32_t require_coverage;    /* 1 = training heuristic (every block assigned); 0 = deployment      */
  int32_t scale_mode;
  uint64_t seed, round;
} twist_sample_desc;

typedef struct {
  int32_t kind;
  float lr, beta1, beta2, eps, weight_decay; /* weight decay applies to matrices only */
} twist_opt_desc;

typedef struct twist_ctx twist_ctx;
typedef struct twist_plan twist_plan;
typedef struct twist_subnet twist_subnet;
typedef struct twist_accum twist_accum;

/* One TwIST round (Section 3: sample, dispatch, local training for the repartition interval, aggregate). */
typedef struct {
  twist_sample_desc sample; /* blueprint of this round; advance sample.round from one round to the next  */
  twist_opt_desc opt;       /* local optimizer; AdamW moments start at zero in every round                */
  int32_t local_steps;      /* batches each subnet trains on before aggregation (repartition interval)  */
  int32_t B, N;             /* batch shape of every local step                                          */
} twist_round_desc;

/* Create a context for one model shape.  hip_stream is a hipStream_t (NULL = the default stream).
 * TWIST_ESHAPE if a dimension is not positive, d_ff is not a multiple of ffn_granule, or d_head is odd
 * with rotary positions. */
TWIST_API twist_status twist_create(const twist_model_desc *desc, void *hip_stream, twist_ctx **out);
TWIST_API void twist_destroy(twist_ctx *ctx);
/* Message of the last failing call on this ctx (or, with ctx == NULL, of the last failing call of the
 * calling thread).  The string is owned by the library and valid until the next call. */
TWIST_API const char *twist_last_error(const twist_ctx *ctx);

/* Subnet generator, Algorithm 1 (Section 3.1): one blueprint A (S x N_sub, rows sorted) per layer and
 * block kind, each from its own random stream keyed by (seed, round, layer, kind); plus, derived from A,
 * inv[s][u] = position of block u in row s or -1, and count[u] = number of rows holding u (the denominator
 * of the aggregation formula, Section 3.3).  Host integer work, spread over up to 8 host threads for large models
 * (the streams are independent, so the tables do not depend on the thread count); the tables are also uploaded to
 * the device (synchronous copy).  TWIST_ECONSTRAINT unless |C| <= N_sub <= N_full and, with require_coverage,
 * N_full - |C| <= S (N_sub - |C|)  (the bound stated below Algorithm 1). */
TWIST_API twist_status twist_sample(twist_ctx *ctx, const twist_sample_desc *desc, twist_plan **out);
/* Borrowed views of one blueprint: idx [S][n_sub], inv [S][n_full], count [n_full], int32, host or device
 * copies (on_device).  Any of the out pointers may be NULL.  Valid until twist_plan_destroy. */
TWIST_API twist_status twist_plan_view(const twist_plan *plan, int32_t layer, int32_t kind, const int32_t **idx,
                             const int32_t **inv, const int32_t **count, int32_t *n_sub, int32_t *n_full,
                             int32_t on_device);
/* Copies the DEVICE copies of one blueprint's tables into host arrays of S*n_sub, S*n_full and n_full int32 (any may be
 * NULL): what the gather and pull kernels actually read.  Synchronous copies. */
TWIST_API twist_status twist_plan_read_device(const twist_plan *plan, int32_t layer, int32_t kind, int32_t *idx, int32_t *inv, int32_t *count);
TWIST_API void twist_plan_destroy(twist_plan *plan);

/* Bytes of caller-provided device storage a subnet of this plan needs (same for every s). */
TWIST_API twist_status twist_subnet_bytes(twist_ctx *ctx, const twist_plan *plan, int32_t store, size_t *bytes);

/* Dispatcher (Section 3.2): materialise subnet s.  For every partitioned tensor the blocks named by row s
 * of the blueprint are concatenated, in row order, into a smaller dense matrix; shared tensors are copied.
 * `storage` (dev, 256-byte aligned, storage_bytes >= twist_subnet_bytes) receives the subnet and stays
 * owned by the caller; fp32 master weights, if requested, are initialised from the extracted values.  The gradient
 * region is left as it is (twist_subnet_fwd_bwd overwrites every gradient, so gradients are undefined until its first
 * call) and so are the AdamW moments, which count as zero: a subnet's first twist_subnet_step does not read them.
 * Inside the subnet W^Q,W^K,W^V are stored as one [3 H' d_head, d]
 * matrix and gate/up as one [2 F', d] matrix; twist_subnet_view hides that. */
TWIST_API twist_status twist_extract(twist_ctx *ctx, const twist_plan *plan, const twist_full_weights *full, int32_t s,
                           void *storage, size_t storage_bytes, int32_t store, twist_subnet **out);
/* The dispatcher for all S subnets of the plan at once (Section 3.2; on one device all subnets are resident together):
 * same result as twist_extract for s = 0..S-1 into storages[s] (each dev, 256-byte aligned, storage_bytes large), but
 * every tensor that is cut into blocks of whole rows, and every shared matrix, is read ONCE and written to each subnet
 * that holds the block, instead of once per subnet (up to 8 subnets; beyond that the per-subnet gathers run).
 * out[0..S) receives the handles; on error none is created. */
TWIST_API twist_status twist_extract_all(twist_ctx *ctx, const twist_plan *plan, const twist_full_weights *full, void *const *storages,
                                         size_t storage_bytes, int32_t store, twist_subnet **out);
/* Device pointer and [rows, cols] shape (cols = 1 for vectors) of one subnet tensor; layer = -1 selects the
 * model-level tensors.  what = TWIST_PARAM gives desc.dtype data, TWIST_GRAD the fp32 gradient, TWIST_MASTER the fp32
 * weights the optimizer updates, TWIST_ADAM_M / TWIST_ADAM_V the AdamW moments (TWIST_EINVAL before the first step, or
 * when the subnet was extracted without that storage). */
TWIST_API twist_status twist_subnet_view(const twist_subnet *sub, int32_t layer, int32_t tensor, int32_t what,
                               void **dev, int64_t shape[2]);
TWIST_API void twist_subnet_destroy(twist_subnet *sub);

/* Bytes of device workspace twist_subnet_fwd_bwd needs for a batch of B sequences of N tokens. */
TWIST_API twist_status twist_workspace_bytes(twist_ctx *ctx, const twist_subnet *sub, int32_t B, int32_t N, size_t *bytes);

/* One forward + backward pass of the dense subnet (Section 4.1 "True TwIST"; layer of Appendix A.2, causal
 * attention).  Each module's output is multiplied by sqrt(N_full / N_sub) before its residual add when the
 * plan was sampled with TWIST_SCALE_SQRT_RATIO (Section 3.4).
 *   vocab > 0 : inputs  = int32 token ids [B, N] (dev), targets = int32 ids [B, N] (dev, already shifted);
 *               loss = mean cross-entropy over the B*N positions.
 *   vocab = 0 : inputs  = activations [B, N, d_model] in desc.dtype, targets likewise; loss = mean squared
 *               error over all B*N*d_model elements of the last layer's output.
 * Writes the fp32 loss to loss_dev and OVERWRITES the subnet's gradient buffers with dLoss/dparam.
 * bf16 models: bf16 operands, fp32 accumulation, fp32 residual stream, softmax and norm statistics.
 * TWIST_ESHAPE if the subnet has no gradient storage, N > max_seq, the workspace is too small, or a
 * dimension is outside what the kernels cover (d_head in {32, 64, 128}; d_model, widths multiples of 8). */
TWIST_API twist_status twist_subnet_fwd_bwd(twist_ctx *ctx, twist_subnet *sub, const void *inputs, const void *targets,
                                  int32_t B, int32_t N, void *workspace, size_t workspace_bytes, float *loss_dev);

/* Masked TwIST (Section 4.1): forward+backward of the FULL-width model `full_sub` (a subnet extracted from a plan
 * that keeps every block) with the blocks that row s of `plan` does not name masked out, and the module scales of
 * row s's widths.  Loss and the gradients of the kept blocks equal those of the subnet twist_extract(plan, s)
 * would give; gradients of masked blocks are zero; shared tensors get their usual gradients.  Other arguments as
 * for twist_subnet_fwd_bwd.  TWIST_ESHAPE if full_sub does not hold every block. */
TWIST_API twist_status twist_subnet_fwd_bwd_masked(twist_ctx *ctx, twist_subnet *full_sub, const twist_plan *plan, int32_t s,
                                                   const void *inputs, const void *targets, int32_t B, int32_t N, void *workspace,
                                                   size_t workspace_bytes, float *loss_dev);

/* Evaluation of an extracted subnet (Section 4.2, deployment: a pruned model is used as is): the forward half of
 * twist_subnet_fwd_bwd only; *loss_dev receives the same loss.  Works on subnets extracted with any storage mode
 * (no gradients are written); arguments, workspace and errors as for twist_subnet_fwd_bwd. */
TWIST_API twist_status twist_subnet_forward(twist_ctx *ctx, twist_subnet *sub, const void *inputs, const void *targets,
                                            int32_t B, int32_t N, void *workspace, size_t workspace_bytes, float *loss_dev);

/* Local optimizer step on every subnet parameter from the current gradients: SGD  w -= lr g,  or AdamW
 * (bias-corrected, decoupled decay on matrices only; needs TWIST_STORE_ADAMW).  bf16 models update fp32
 * master weights and re-round the bf16 copy. */
TWIST_API twist_status twist_subnet_step(twist_ctx *ctx, twist_subnet *sub, const twist_opt_desc *opt);

/* Aggregator (Section 3.3): for every central parameter p,  p <- sum_i p_i [p in W_i] / sum_i [p in W_i]
 * over the given subnets (a parameter held by none of them keeps its value); shared tensors become the
 * mean over the given subnets.  subs[i] must have been extracted from this plan; any subset of the S
 * subnets may be passed (n_subs >= 1).  Sums are formed in fp32 in the order given, divided, and rounded
 * once to desc.dtype; a parameter with a single owner is copied bit-exactly.  Updates `inout` in place. */
TWIST_API twist_status twist_aggregate(twist_ctx *ctx, const twist_plan *plan, twist_subnet *const *subs, int32_t n_subs,
                             const twist_full_weights *inout);

/* The same aggregation (Section 3.3) one subnet at a time, so that only one subnet needs to be resident: an fp32
 * image of the central model accumulates p_i for every subnet added; finish divides by the number of added
 * owners, rounds once to desc.dtype and writes the central tensors (a parameter none of the added subnets holds
 * keeps its value), then forgets the added rows so the object can serve the next round of the same plan.
 * Additions happen in the order of the add calls, hence the result is bit-identical to twist_aggregate over
 * the same subnets in the same order.  `image` (dev, 256-byte aligned, >= twist_aggregate_image_bytes, caller-owned,
 * need not be cleared) must stay valid until finish; a subnet's storage may be reused as soon as its add call has
 * returned (stream order).  TWIST_EINVAL if a blueprint row is added twice or the subnet is from another plan. */
TWIST_API twist_status twist_aggregate_image_bytes(twist_ctx *ctx, size_t *bytes);
TWIST_API twist_status twist_aggregate_begin(twist_ctx *ctx, const twist_plan *plan, void *image, size_t image_bytes, twist_accum **out);
TWIST_API twist_status twist_aggregate_add(twist_accum *acc, const twist_subnet *sub);
TWIST_API twist_status twist_aggregate_finish(twist_accum *acc, const twist_full_weights *inout);
TWIST_API void twist_aggregate_destroy(twist_accum *acc);

/* One whole round on the persistent central model `inout` (Section 3; Section 5 resamples every few batches):
 * sample the round's blueprint, then for s = 0..S-1: extract subnet s, run local_steps x {fwd_bwd, step} on its own
 * batches, add it to the running aggregate; finally write the averaged parameters back.  One subnet is resident at
 * a time, in `subnet_storage`.  inputs/targets (dev) hold S * local_steps batches back to back, subnet-major
 * ([S][local_steps][B][N] token ids, or [..][B][N][d_model] activations when vocab = 0); loss_dev (dev) receives
 * the S * local_steps losses in the same order.  Buffer sizes from twist_round_bytes; all buffers caller-owned.
 * Synchronises the context's stream before returning (the round's index tables are released). */
TWIST_API twist_status twist_round_bytes(twist_ctx *ctx, const twist_round_desc *rd, size_t *subnet_bytes, size_t *workspace_bytes,
                                         size_t *image_bytes);
TWIST_API twist_status twist_round(twist_ctx *ctx, const twist_round_desc *rd, const twist_full_weights *inout, const void *inputs,
                                   const void *targets, void *subnet_storage, size_t subnet_bytes, void *workspace,
                                   size_t workspace_bytes, void *image, size_t image_bytes, float *loss_dev);

/* Kernel-level entry point for tests and benchmarks: one projection of the subnet forward/backward pass in
 * isolation, C = alpha * op(A) op(B), fp32 accumulation, on the ctx's stream (Appendix A.1: Q_h = X W^Q_h etc.;
 * the backward pass uses the two transposed forms).  layout 0: A [M,K], B [N,K] (y = x W^T); 1: A [M,K], B [K,N]
 * (dx = dy W); 2: A stored [K,M], B stored [K,N] (dW = dy^T x).  All row-major device pointers of desc.dtype
 * with row strides lda/ldb/ldc in elements; C is fp32 when out_f32 != 0, else desc.dtype. */
TWIST_API twist_status twist_gemm_raw(twist_ctx *ctx, int32_t layout, int32_t M, int32_t N, int32_t K, const void *A, int64_t lda,
                                      const void *B, int64_t ldb, void *C, int64_t ldc, int32_t out_f32, float alpha);

/* Kernel-level entry point for tests: causal multi-head attention of Appendix A.1 in isolation, forward and (when
 * dout is not NULL) backward, on a fused activation buffer qkv [B*N, 3*Hs*d_head] (q | k | v, desc.dtype).
 * Outputs: o [B*N, Hs*d_head] (desc.dtype), lse [B, Hs, N] fp32 (log-sum-exp of the scaled scores), and dqkv
 * [B*N, 3*Hs*d_head] from dout [B*N, Hs*d_head].  o32 [B*N, Hs*d_head] fp32 and delta [B, Hs, N] fp32 are
 * caller-provided scratch (o32 receives the unrounded output of bf16 models).  keep (dev int32 [Hs], may be NULL) is the
 * head mask of Masked TwIST (Section 4.1): heads with keep[h] < 0 give zero output and zero gradients.  rope_tab (scratch
 * of N * d_head floats, may be NULL): when given, q and k are taken to be already rotated by the rotary embedding and
 * their gradients in dqkv are turned back through it, as the training pass does (inside the attention kernels where they
 * cover the shape).  All device pointers, caller-owned; work is enqueued on the ctx's stream.  TWIST_ESHAPE if d_head
 * exceeds 256. */
TWIST_API twist_status twist_attention_raw(twist_ctx *ctx, const void *qkv, const void *dout, int32_t B, int32_t N, int32_t Hs,
                                           void *o, float *o32, float *lse, float *delta, void *dqkv, const int32_t *keep,
                                           float *rope_tab);

/* Kernel-level entry points for tests: the memory-bound steps of twist_subnet_fwd_bwd in isolation, run by the same
 * kernels, on the ctx's stream.  Shapes and kinds come from the ctx's model description (d_model, d_head, norm, act,
 * vocab, dtype).  All pointers are device pointers owned by the caller; "dtype" means desc.dtype.
 *
 * twist_norm_raw   f_ln of Appendix A.1 (LayerNorm, or RMSNorm for desc.norm = TWIST_NORM_RMS): y [T, d_model] (dtype) from
 *                  x [T, d_model] (fp32 residual stream), gain w and bias b ([d_model], dtype; b NULL for RMSNorm);
 *                  stats [2 T] fp32 receives (mean, 1/std) per row.  With dy (dtype) not NULL also the backward half:
 *                  dx [T, d_model] fp32 (overwritten), dxb (dtype copy of dx, may be NULL), dw and db ([d_model] fp32, db
 *                  may be NULL); scratch: at least ceil(T / 16) * 2 * d_model floats (TWIST_ESHAPE if smaller).
 * twist_rope_raw   rotary positions (half-split pairing, desc.rope_theta) applied in place to the q and k heads of a
 *                  fused [B*N, 3*Hs*d_head] buffer (dtype); sign = +1 forward, -1 the backward rotation; tab: scratch
 *                  of N * d_head floats (receives the cos/sin table).
 * twist_act_raw    FFN activation of Appendix A.1 (desc.act): a [T, F] from gu [T, F] (GELU, ReLU) or gu [T, 2F] (gate | up
 *                  for SwiGLU); with da not NULL also dgu (shape of gu) from da [T, F].  keep (int32, one entry per block
 *                  of `unit` neurons, may be NULL): blocks with keep[b] < 0 are masked (Section 4.1): a = 0, dgu = 0 there.
 * twist_ce_raw     mean cross-entropy over T rows of logits [T, ld] (dtype; ld >= vocab, columns beyond vocab are
 *                  padding): loss (fp32 scalar), rowloss [T] fp32, and logits are overwritten by dLoss/dlogits.
 * twist_embed_raw  x [B*N, d_model] fp32 = tok_embed[tok] (+ pos_embed[position], pos_embed may be NULL); with dx not NULL
 *                  also the backward half: dx rows are ADDED into d_tok [vocab, d_model] fp32 (caller clears it) and
 *                  d_pos [N, d_model] fp32 (overwritten, may be NULL) receives the sum over the batch. */
TWIST_API twist_status twist_norm_raw(twist_ctx *ctx, const float *x, const void *w, const void *b, int32_t T, void *y, float *stats,
                                      const void *dy, float *dx, void *dxb, float *dw, float *db, float *scratch, size_t scratch_floats);
/* twist_norm_raw for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): same arguments, results and kernels, but the scratch of the backward half is a
 * built-in device array of 2 Mi floats (8 MiB, held on every GPU the library runs on until the process ends) instead of
 * a caller buffer; the call allocates nothing.  TWIST_ESHAPE when ceil(T / 16) * 2 * d_model exceeds 2 Mi floats (use
 * twist_norm_raw then).  All calls on one GPU share the array: calls that may overlap there (different streams, different
 * contexts) race on it; calls on one stream are ordered and safe.  Nothing in the array has to start at zero. */
TWIST_API twist_status twist_norm_raw_static(twist_ctx *ctx, const float *x, const void *w, const void *b, int32_t T, void *y, float *stats,
                                             const void *dy, float *dx, void *dxb, float *dw, float *db);
TWIST_API twist_status twist_rope_raw(twist_ctx *ctx, void *qkv, int32_t B, int32_t N, int32_t Hs, float sign, float *tab);
TWIST_API twist_status twist_act_raw(twist_ctx *ctx, const void *gu, int32_t T, int32_t F, void *a, const void *da, void *dgu,
                                     const int32_t *keep, int32_t unit);
TWIST_API twist_status twist_ce_raw(twist_ctx *ctx, void *logits, int64_t ld, const int32_t *targets, int32_t T, float *rowloss, float *loss);
TWIST_API twist_status twist_embed_raw(twist_ctx *ctx, const int32_t *tok, int32_t B, int32_t N, const void *tok_embed, const void *pos_embed,
                                       float *x, const float *dx, float *d_tok, float *d_pos);

/* Measurement aid for benchmarks (not part of the method): while enabled, every projection (GEMM) launch on
 * this ctx is bracketed by two HIP events on the ctx's stream.  twist_profile_gemm_read synchronises the
 * stream, returns the number of launches, their summed duration in milliseconds and their summed algorithmic
 * floating-point operations (2 M N K each) since enabling, and resets the counters. */
TWIST_API twist_status twist_profile_gemm(twist_ctx *ctx, int32_t enable);
TWIST_API twist_status twist_profile_gemm_read(twist_ctx *ctx, int64_t *launches, double *ms, double *flops);

/* Measurement aid: the rate of the projection kernels' matrix instruction alone (v_mfma_f32_32x32x16_bf16, operands in
 * registers, no loads, four independent accumulator tiles per wave), with `waves_per_simd` waves on every SIMD of the
 * chip for `iters` iterations of four instructions: the ceiling any kernel built on that instruction has on this chip at
 * the clock it holds under that load.  random_operands = 0 feeds small constants, 1 pseudo-random values of magnitude
 * about one (the chip's power limit, hence its clock, depends on how many operand bits toggle).  sink (dev, at least
 * compute units * waves_per_simd * 256 floats) receives the accumulators.  Synchronises the ctx's stream; *tflops
 * (host) receives the rate. */
TWIST_API twist_status twist_profile_mfma_ceiling(twist_ctx *ctx, int32_t waves_per_simd, int32_t iters, int32_t random_operands, float *sink,
                                                  size_t sink_floats, double *tflops);

/* The weight-gradient projections of twist_subnet_fwd_bwd run on a second stream that the library creates
 * (default priority), next to the input-gradient kernels on the context's stream; the call still returns with
 * all of its work ordered before anything enqueued on the context's stream afterwards.  enable = 0 puts every
 * kernel on the context's stream (needed when per-kernel durations are to be measured one at a time).
 * Default: enabled. */
TWIST_API twist_status twist_set_overlap(twist_ctx *ctx, int32_t enable);

/* Kernel selection for tests (not part of the method): by default every launcher picks its kernel from the shape.
 *   gemm_tile        0 = by shape; 128 or 256 pins the tile of the matrix-core projection kernel and keeps the
 *                    contraction in one piece (TWIST_EINVAL for other values);
 *   plain_only       non-zero: projections and attention never use the matrix-core kernels (the plain fp32-arithmetic
 *                    kernels that serve fp32 models and unaligned shapes run instead);
 *   staged_attention non-zero: d_head = 128 attention runs the register-staged tiled kernels instead of the ones fed by
 *                    loads straight into LDS.
 * Results stay within the same tolerances under every choice; only speed changes. */
TWIST_API twist_status twist_set_kernel_choice(twist_ctx *ctx, int32_t gemm_tile, int32_t plain_only, int32_t staged_attention);

#ifdef __cplusplus
}
#endif
#endif /* TWIST_H */
