/*
 * zb_stage.h — C ABI of one Zero-Bubble pipeline stage on one MI355X (gfx950).
 *
 * Method: "Zero Bubble Pipeline Parallelism", arXiv 2401.10241.  One pipeline
 * stage holds L pre-LN GPT decoder layers (Sec. 2.3: FFN inner size 4h, head
 * size h/a) and executes, per microbatch, the paper's three passes (Sec. 1):
 *   F  forward
 *   B  input-gradient backward   grad_x f(x,W)^T dl/dy
 *   W  parameter-gradient backward grad_W f(x,W)^T dl/dy, accumulated over
 *      microbatches from what B kept for it (Sec. 2.3, Table 1)
 * in the per-stage order of the handcrafted schedules ZB-H1 (Sec. 2.1) and
 * ZB-H2 (Sec. 2.2), followed by the post-validated optimizer step (Sec. 4)
 * with the in-place AdamW step / rollback of Appendix C, Algorithm 1.
 *
 * Conventions
 *  - Every function returns a zb_status and never throws or aborts.
 *  - "host" pointers are ordinary CPU memory owned by the caller; "device"
 *    pointers are HIP device memory.  The stage allocates nothing on the device:
 *    all its device memory is carved from the caller's `arena` (device pointer,
 *    256-byte aligned, at least zb_stage_arena_bytes() long), which must stay
 *    valid until zb_stage_free.  Kernels run on `hip_stream` (a hipStream_t
 *    passed as void*; NULL = the default stream).
 *  - Calls enqueue work and return without waiting for the device, except
 *    zb_get_tensor / zb_set_tensor / zb_synchronize / zb_profile_read and
 *    zb_optimizer_step_validated when a report is requested.
 *  - External tensor layout is fp32, row-major.  Token matrices are
 *    [seq*mb_size, hidden] (sample-major rows).  Weight matrices are [in, out];
 *    the QKV projection's columns are [Q | K | V], each head-major.
 *  - Data type ZB_BF16: fp32 master parameters, Adam moments and accumulated
 *    gradients; bf16 working weights, activations and activation gradients;
 *    fp32 accumulation everywhere.  ZB_FP32: everything fp32.
 *  - There is no CPU fallback: every pass runs in HIP kernels of this library.
 */
#ifndef ZB_STAGE_H
#define ZB_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct zb_stage zb_stage; /* opaque */

typedef enum {
  ZB_OK = 0,
  ZB_EINVAL = 1,  /* bad argument or configuration */
  ZB_EORDER = 2,  /* F -> B -> W dependency of a microbatch violated, or pass repeated (Sec. 2) */
  ZB_ENOMEM = 3,  /* arena too small, or a stash pool is exhausted */
  ZB_EDEVICE = 4, /* a HIP call failed; see zb_last_error */
  ZB_ESTATE = 5   /* call not valid in the stage's current state */
} zb_status;

typedef enum { ZB_FP32 = 0, ZB_BF16 = 1 } zb_dtype;
typedef enum { ZB_1F1B = 0, ZB_H1 = 1, ZB_H2 = 2 } zb_kind;
typedef enum { ZB_PASS_F = 0, ZB_PASS_B = 1, ZB_PASS_W = 2 } zb_pass;
/* Sec. 5.1: the first stage of the pipeline also does the embedding lookup, the last one the loss
 * computation (each holds one transformer layer fewer to make up for it: pass that count as `layers`). */
typedef enum { ZB_ROLE_MIDDLE = 0, ZB_ROLE_FIRST = 1, ZB_ROLE_LAST = 2 } zb_role;
typedef struct { int32_t pass, mb; } zb_op;

/* Per-layer parameters, in the order used by every "param index" below. */
enum {
  ZB_P_LN1_G = 0, ZB_P_LN1_B, ZB_P_WQKV, ZB_P_BQKV, ZB_P_WO, ZB_P_BO,
  ZB_P_LN2_G, ZB_P_LN2_B, ZB_P_W1, ZB_P_B1, ZB_P_W2, ZB_P_B2, ZB_P_COUNT
};

/* Stage-level parameters of a first stage (token table [vocab, hidden], position table [seq, hidden]) and of
 * a last stage (final LayerNorm gamma / beta [hidden], head matrix [hidden, vocab], no bias, not tied to the
 * token table). */
enum { ZB_SP_EMB_TOK = 0, ZB_SP_EMB_POS = 1, ZB_SP_LNF_G = 2, ZB_SP_LNF_B = 3, ZB_SP_W_HEAD = 4, ZB_SP_COUNT = 5 };

/* `what` of zb_get_tensor / zb_set_tensor.  For the four per-parameter groups
 * add the param index (ZB_T_PARAM + ZB_P_WO ...); `layer` selects the layer and
 * `mb` is ignored.  For the per-microbatch tensors `layer` is ignored. */
enum {
  ZB_T_PARAM = 0,    /* fp32 master parameter                               get/set */
  ZB_T_GRAD = 16,    /* fp32 gradient accumulated over this iteration's W   get/set */
  ZB_T_ADAM_M = 32,  /* first moment                                        get/set */
  ZB_T_ADAM_V = 48,  /* second moment                                       get/set */
  ZB_T_INPUT_X = 64, /* activation received from the previous stage, [tokens, hidden]  get/set */
  ZB_T_INPUT_DY = 65,  /* output gradient received from the next stage               get/set */
  ZB_T_OUTPUT_Y = 66,  /* activation sent to the next stage (written by F)           get */
  ZB_T_OUTPUT_DX = 67, /* input gradient sent to the previous stage (written by B)   get */
  ZB_T_INPUT_IDS = 68,  /* first stage: token ids of microbatch mb; the host buffer holds int32 [tokens],
                           bytes = 4 * tokens, every id in [0, vocab) (ZB_EINVAL otherwise)            get/set */
  ZB_T_TARGET_IDS = 69, /* last stage: target ids, same format                                         get/set */
  ZB_T_LOSS = 70,       /* last stage: mean over the tokens of microbatch mb of its cross-entropy loss
                           (written by F), one fp32                                                    get */
  ZB_T_STAGE_PARAM = 96,    /* + ZB_SP_*: stage-level master parameter (layer, mb ignored)              get/set */
  ZB_T_STAGE_GRAD = 104,    /* + ZB_SP_*: its accumulated gradient                                      get/set */
  ZB_T_STAGE_ADAM_M = 112,  /* + ZB_SP_*                                                                get/set */
  ZB_T_STAGE_ADAM_V = 120,  /* + ZB_SP_*                                                                get/set */
  ZB_T_FLAT_PARAMS = 80, /* all master parameters of the stage, layer-major, param order, each
                            tensor padded to a multiple of 64 floats (zb_stage_flat_count)   get */
  ZB_T_FLAT_GRADS = 81, ZB_T_FLAT_ADAM_M = 82, ZB_T_FLAT_ADAM_V = 83
};

typedef struct {
  int32_t layers, hidden, heads, ffn, seq, mb_size;
  int32_t max_microbatches; /* capacity of the per-microbatch input/output buffers */
  int32_t max_pending_b;    /* microbatches that have done F but not B at once */
  int32_t max_pending_w;    /* microbatches that have done B but not W at once */
  int32_t max_inflight;     /* microbatches that have done F but not W at once */
  int32_t dtype;            /* zb_dtype */
  int32_t journal;          /* 1: the step keeps an undo journal so that rollback restores
                               theta, m, v bit for bit (12 B/parameter); 0: rollback is
                               Algorithm 1's arithmetic inverse only (exact to rounding) */
  int32_t group_w;          /* 1: zb_run_schedule / zb_run_order run consecutive W passes of the order as
                               one grouped W (zb_backward_weight_group); 0: one by one.  Same bits. */
  int32_t fuse_bw;          /* 1: where an order has W_k directly after B_k (1F1B), zb_run_schedule /
                               zb_run_order run the two as one zb_backward_fused; 0 (default): separately */
  int32_t chunks;           /* 1, or 2 for ZB-V (Sec. 6): the first half of the layers is chunk 0, the second
                               half chunk 1; microbatch indices are then VIRTUAL, v = chunk * (m/2) + microbatch
                               for zb_begin_iteration's (even) m, each with its own INPUT_X / INPUT_DY /
                               OUTPUT_Y / OUTPUT_DX, and a pass on v runs through the layers of its chunk only */
  int32_t role;             /* zb_role.  ZB_ROLE_FIRST: F of a microbatch starts from INPUT_IDS (X0 = token row +
                               position row; INPUT_X is then written by F), W also adds the two tables' gradients
                               (a table row receives the OUTPUT_DX rows of its tokens in increasing token order).
                               ZB_ROLE_LAST: F ends with the final LayerNorm, the head and the softmax cross-entropy
                               against TARGET_IDS (LOSS); B starts from the gradient of
                               (1/m) * sum over the iteration's microbatches of their mean token loss (INPUT_DY is
                               then written by B) and adds the final LayerNorm's gamma / beta gradients; W also adds
                               the head's gradient.  Not with chunks = 2. */
  int32_t vocab;            /* rows of the token table / columns of the head (first and last stage), <= 2^18;
                               the first stage takes at most 8192 tokens per microbatch */
  float ln_eps;             /* 1e-5 */
  float lr, beta1, beta2, adam_eps, weight_decay; /* Algorithm 1's gamma, beta1, beta2, eps, lambda */
  float clip;               /* global gradient-norm clipping threshold (Sec. 4) */
  void* hip_stream;         /* hipStream_t or NULL */
  void* arena;              /* device memory, 256-byte aligned */
  size_t arena_bytes;
} zb_config;

/* Fills the numeric fields of *cfg with defaults (ln_eps 1e-5, lr 1e-4, betas 0.9/0.95,
 * eps 1e-8, weight decay 0.01, clip 1.0, journal 1, group_w 1, dtype bf16); shapes are left 0. */
zb_status zb_config_defaults(zb_config* cfg);

/* Device bytes zb_stage_init needs for this configuration (arena fields ignored). */
zb_status zb_stage_arena_bytes(const zb_config* cfg, size_t* bytes);

/* Creates a stage.  Parameters, moments and gradients start at zero, t = 0; load
 * parameters with zb_set_tensor.  *out is NULL on failure. */
zb_status zb_stage_init(const zb_config* cfg, zb_stage** out);
zb_status zb_stage_free(zb_stage* st);

/* Number of floats in the ZB_T_FLAT_* vectors. */
zb_status zb_stage_flat_count(const zb_stage* st, size_t* count);

/* Starts an iteration of m microbatches (m <= max_microbatches): forgets which passes
 * have run, releases all stash slots and zeroes the accumulated gradients (on the stream).
 * `iter` is recorded for error messages only.  Inputs keep their contents. */
zb_status zb_begin_iteration(zb_stage* st, int32_t iter, int32_t m);

/* The three passes of microbatch mb (Sec. 1).  F reads INPUT_X[mb] and writes OUTPUT_Y[mb];
 * B reads INPUT_DY[mb], writes OUTPUT_DX[mb] and adds the LayerNorm gamma/beta gradients;
 * W adds the weight and bias gradients of the four linears of every layer.
 * ZB_EORDER unless F(mb) precedes B(mb) precedes W(mb), each at most once per iteration. */
zb_status zb_forward(zb_stage* st, int32_t mb);
zb_status zb_backward_input(zb_stage* st, int32_t mb);
zb_status zb_backward_weight(zb_stage* st, int32_t mb);

/* B and W of microbatch mb as the traditional single backward (Sec. 1: 1F1B's backward, before the split):
 * layer by layer from the last to the first, the input gradient of a layer and right after it that layer's
 * parameter gradients.  Same results, bit for bit, as zb_backward_input(mb) then zb_backward_weight(mb);
 * it is here to measure what the split costs or gains on one GPU.  Needs a free B->W stash slot. */
zb_status zb_backward_fused(zb_stage* st, int32_t mb);

/* W of n microbatches at once, mbs[0..n) (host) in that order, grouped by parameter (Appendix A groups
 * the deferred W passes by parameter; Sec. 2: W may run anywhere after its B): every weight gradient is
 * read once, receives the n products one after the other and is written once.  The gradients are bit for
 * bit those of zb_backward_weight(mbs[0]), ..., zb_backward_weight(mbs[n-1]).  Each mbs[i] must have
 * done B and not W (ZB_EORDER otherwise, nothing is run then); n >= 1. */
zb_status zb_backward_weight_group(zb_stage* st, const int32_t* mbs, int32_t n);

/* Per-stage pass order (host only; `stage` is 0-based, the paper's worker i = stage+1).
 * Writes 3m entries to out (host, capacity cap) and their number to *n. */
zb_status zb_schedule_order(int32_t p, int32_t stage, int32_t m, int32_t kind,
                            zb_op* out, int32_t cap, int32_t* n);

/* Largest number of pending-B, pending-W and in-flight microbatches of that order
 * (the sizes the stash pools of zb_config need).  Any out pointer may be NULL. */
zb_status zb_schedule_stash_need(int32_t p, int32_t stage, int32_t m, int32_t kind,
                                 int32_t* max_pending_b, int32_t* max_pending_w, int32_t* max_inflight);

/* zb_begin_iteration(m) must have been called; runs all 3m passes in schedule order. */
zb_status zb_run_schedule(zb_stage* st, int32_t p, int32_t stage, int32_t m, int32_t kind);

/* Same for an explicit order of n entries (host), e.g. one stage's row of zb_auto_schedule's result.
 * ZB_EORDER if the list is not a valid stage order (F before B before W, nothing twice). */
zb_status zb_order_stash_need(const zb_op* ops, int32_t n, int32_t* max_pending_b, int32_t* max_pending_w,
                              int32_t* max_inflight);

/* zb_begin_iteration(m) must have been called; runs the n = 3m passes of an explicit order (host array).
 * The same dependency rule as the single pass calls applies (ZB_EORDER); the stash pools of the stage
 * must hold what zb_order_stash_need reports for this order (ZB_ENOMEM from the pass that does not fit). */
zb_status zb_run_order(zb_stage* st, const zb_op* ops, int32_t n);

/* ---- p-stage timing model and automatic scheduling (host only, no device needed) --------------------
 * Pass times of one stage (any unit) and the transfer time between neighbouring stages (Sec. 3). */
typedef struct { double t_f, t_b, t_w, t_comm; } zb_pass_times;
/* Activation memory (Appendix G): F adds m_b, B adds m_w - m_b, W releases m_w; a stage may never
 * hold more than m_limit.  0 <= m_w <= m_b <= m_limit. */
typedef struct { double m_limit, m_b, m_w; } zb_memory_model;

/* Timing model of Sec. 5.3 / Appendix G for p stage orders, orders[stage*3m + q] (host): a pass starts
 * when its stage is free and its input has arrived (F from stage-1, B from stage+1, t_comm after the
 * producer ended; fused_backward != 0: the gradient leaves a stage after the W of that microbatch, the
 * single backward of 1F1B).  *cost = largest stage span, *bubble_rate = (cost - m(T_F+T_B+T_W)) / cost,
 * stage_span[p] = every stage's span.  Out pointers may be NULL.  ZB_EORDER for invalid or deadlocking
 * orders. */
zb_status zb_simulate_pipeline(int32_t p, int32_t m, const zb_op* orders, const zb_pass_times* times,
                               int32_t fused_backward, double* cost, double* bubble_rate, double* stage_span);

/* Heuristic scheduler of Sec. 3.1 for one setting of its two binary options: extra_warmup_f = a stage that
 * would idle before its first backward takes one more warm-up forward although that delays the backward;
 * skip_f = a stage that leads its successor by more than one forward leaves a round's forward out when it has a
 * W to run instead.  The steps run as the section lists them: warm-up forwards within the memory limit (stage
 * i+1 at most one fewer than stage i), rounds of one B and one F per stage with W filling the gaps and
 * releasing memory, the remaining W.  Writes all p stage orders to orders[p*3m] (host).  ZB_ENOMEM if
 * m_limit admits no schedule. */
zb_status zb_auto_schedule(int32_t p, int32_t m, const zb_pass_times* times, const zb_memory_model* mem,
                           int32_t extra_warmup_f, int32_t skip_f, zb_op* orders);

/* Grid search over the two options (Sec. 3.1): the cheapest of the four schedules under the timing model
 * above, the first of (0,0) (0,1) (1,0) (1,1) on ties.  Out pointers other than orders may be NULL. */
zb_status zb_auto_schedule_search(int32_t p, int32_t m, const zb_pass_times* times, const zb_memory_model* mem,
                                  zb_op* orders, double* cost, double* bubble_rate, int32_t* extra_warmup_f,
                                  int32_t* skip_f);

/* ZB-V (Sec. 6): every worker holds two chunks, chunk 0 of workers 1..p followed by chunk 1 of workers
 * p..1 makes the model.  An entry names a VIRTUAL microbatch v = chunk * m + microbatch, so a worker's
 * order has 6m entries over 2m virtual microbatches; orders[p * 6m] (host) receives all workers' orders
 * (warm-up of 2p-1 forwards, F-B-W groups per chunk, then the remaining B and W with B first and W filling
 * the gaps, built for equal pass times).  With m >= 2p-1 and equal pass times no worker idles, and no
 * worker holds more than 2p chunk activations (= p M_B). */
zb_status zb_schedule_order_v(int32_t p, int32_t m, zb_op* orders);

/* Timing model for such orders: F of chunk 0 waits for worker-1, F of chunk 1 for worker+1 (the last
 * worker: for its own chunk 0), B of chunk 1 for worker-1 (the first worker: for its own F of chunk 1),
 * B of chunk 0 for worker+1 (the last worker: for its own B of chunk 1).  times are those of ONE chunk's
 * pass; *bubble_rate = (cost - 2m(T_F+T_B+T_W)) / cost.  Out pointers may be NULL. */
zb_status zb_simulate_pipeline_v(int32_t p, int32_t m, const zb_op* orders, const zb_pass_times* times, double* cost,
                                 double* bubble_rate, double* stage_span);

/* The same stage order with the W passes of its 1F1B-shaped steady state run `group` at a time (Sec. 2: a W
 * may run anywhere after its B; Appendix A regroups W the same way): wherever the order reads
 * B W F_j B W F B W ... B W  (group times B W, a forward between each two) with the first forward's
 * microbatch j a multiple of group, the W wait for the last of them:  B F_j B F ... B W W ... W.  Keyed on the
 * forward's microbatch, all stages of a pipeline group around the same forwards, so no stage wants a tensor
 * earlier than its neighbour, grouping the same way, sends it: at zero transfer time the timing model's cost
 * does not grow (at most one t_comm per group otherwise), while W side by side read and write every gradient
 * once (zb_backward_weight_group; zb_run_order runs consecutive W that way).  F, B and W each keep their
 * sequence, so results keep every bit; group - 1 more W stashes are pending at the peak
 * (zb_order_stash_need / zb_order_memory_peak on the result).  ops and out: n entries each (host), group >= 1
 * (1: a copy). */
zb_status zb_order_group_w(const zb_op* ops, int32_t n, int32_t group, zb_op* out);

/* zb_simulate_pipeline's model with one more time: a W that directly follows another W on its stage takes
 * t_w_next >= 0 (measured: the later W of a grouped launch).  No fused backward; *cost = largest stage span. */
zb_status zb_simulate_pipeline_w_runs(int32_t p, int32_t m, const zb_op* orders, const zb_pass_times* times,
                                      double t_w_next, double* cost, double* stage_span);

/* Peak of Appendix G's memory walk over one stage order of n entries. */
zb_status zb_order_memory_peak(const zb_op* ops, int32_t n, double m_b, double m_w, double* peak);

/* Global optimizer state contributed by the other stages (Sec. 4): the partially reduced
 * state received from the previous stage and what the stages after this one add to it. */
typedef struct {
  double prev_sq, rest_sq;                 /* squared gradient norms */
  int32_t prev_nonfinite, rest_nonfinite;  /* NaN/Inf seen there */
  int32_t force_optimistic;                /* take the optimistic step whatever the partial state */
} zb_global_state;

enum { /* zb_step_report.outcome */
  ZB_COMMITTED = 0,             /* optimistic step taken and confirmed by the full state */
  ZB_SKIPPED_LOCAL = 1,         /* partial state non-finite: no step, iteration skipped */
  ZB_ROLLED_BACK_NONFINITE = 2, /* step taken, full state non-finite: rolled back, skipped */
  ZB_ROLLED_BACK_RECLIPPED = 3, /* step taken, full norm above threshold: rolled back, redone clipped */
  ZB_DEFERRED_CLIPPED = 4,      /* partial norm already above threshold: one clipped step after validation */
  ZB_DEFERRED_SKIPPED = 5       /* waited for the full state, which was non-finite: skipped */
};

typedef struct {
  int32_t outcome;
  int32_t stepped_optimistically;
  double local_sq;     /* this stage's squared gradient norm */
  double global_norm;  /* sqrt(prev_sq + local_sq + rest_sq); NaN if non-finite */
  double clip_coef;    /* min(1, clip / (global_norm + 1e-6)); 0 if skipped */
  int64_t t;           /* Algorithm 1's time stamp after the call */
  uint64_t alg1_mismatch_elems; /* journal mode, on rollback: elements where Algorithm 1's
                                   arithmetic inverse differs in any bit from the journal */
} zb_step_report;

/* Sec. 4 on the device, with no host round trip between the steps: local sum of squares and
 * non-finite flag; partial = prev (+) local; AdamW Step predicated on the partial state;
 * full = partial (+) rest; if the step taken was not the legitimate one, Rollback and redo
 * Step with the full state.  All decisions are taken by the device from device-resident
 * predicates.  report may be NULL (then the call does not wait for the device). */
zb_status zb_optimizer_step_validated(zb_stage* st, const zb_global_state* gs, zb_step_report* report);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the first step of zb_optimizer_step_validated, the squared norm and the
 * non-finite flag of a gradient vector, with the partial sums of its reduction levels in a fixed array
 * inside the library (about 3.2 MB per GPU, held until the process ends) instead of a stage's arena.
 *   grads          device, n floats, 16-byte aligned; n > 0, n % 4 == 0, n <= ZB_GRAD_NORM_STATIC_MAX_FLOATS
 *   sq_out         device, one double: sum of squares, accumulated in fp64 in the same fixed order as
 *                  zb_step_report.local_sq (bit-identical for the same n and values)
 *   nonfinite_out  device, one int32: 1 if any element is NaN or Inf, else 0
 *   hip_stream     hipStream_t or NULL; the call only enqueues kernels (no synchronisation, no memset,
 *                  no hipMalloc / hipFree), so it may be captured into a graph
 * ZB_EINVAL for null pointers, misaligned grads or n outside the range above (nothing is launched then);
 * ZB_EDEVICE if a HIP call fails.  All calls on one GPU share the array: calls that overlap on one GPU
 * (different streams without ordering between them) race; calls on one stream are safe. */
#define ZB_GRAD_NORM_STATIC_MAX_FLOATS ((size_t)1 << 30)
zb_status zb_grad_norm_static(const float* grads, size_t n, double* sq_out, int32_t* nonfinite_out,
                              void* hip_stream);

/* Copies between host fp32 buffers and stage tensors (converting to/from the stage's
 * data type).  bytes must equal 4 * number of elements.  Both wait for the device. */
zb_status zb_get_tensor(zb_stage* st, int32_t what, int32_t layer, int32_t mb, void* host_dst, size_t bytes);
zb_status zb_set_tensor(zb_stage* st, int32_t what, int32_t layer, int32_t mb, const void* host_src, size_t bytes);

/* What B keeps for W (Table 1: the inputs and the output gradients of the four linears of a layer), as a
 * debug read-out: columns cols[0..ncols) (host) of one such [tokens, width] matrix of microbatch mb, converted
 * to fp32, into host_dst as a dense [tokens, ncols] matrix.  Valid between B(mb) and W(mb) (ZB_EORDER
 * otherwise).  Widths: hidden, except FC2's input and FC1's output gradient (ffn) and the QKV projection's
 * output gradient (3 hidden).  The weight gradient of a linear is the sum over microbatches of
 * input^T * output-gradient, so an accumulated gradient entry can be recomputed from these.  Waits for the
 * device. */
enum {
  ZB_S_QKV_IN = 0, ZB_S_PROJ_IN = 1, ZB_S_FC1_IN = 2, ZB_S_FC2_IN = 3,         /* A, C, U, G of the forward */
  ZB_S_QKV_DOUT = 4, ZB_S_PROJ_DOUT = 5, ZB_S_FC1_DOUT = 6, ZB_S_FC2_DOUT = 7  /* their output gradients */
};
zb_status zb_get_stash_columns(zb_stage* st, int32_t which, int32_t layer, int32_t mb, const int32_t* cols,
                               int32_t ncols, float* host_dst);

/* Overwrites one element of INPUT_X / INPUT_DY of microbatch mb (e.g. with NaN). */
zb_status zb_inject(zb_stage* st, int32_t what, int32_t mb, int64_t elem, float value);

zb_status zb_synchronize(zb_stage* st);
const char* zb_last_error(const zb_stage* st); /* "" if none; valid until the next call on st */

/* Model FLOPs of Table 1 for this stage and m microbatches: L*m*(F + B + W) with
 * F = sbh(24h+4s), B = sbh(24h+8s), W = 24sbh^2 (no causal discount); a last stage adds its head's three
 * matmuls, m * 6 sbh * vocab (Table 1 covers transformer layers only). */
zb_status zb_stage_model_flops(const zb_stage* st, int32_t m, double* flops);

/* Activation bytes this stage really holds per microbatch, in the terms of Appendix G's memory model:
 * *m_b after F (what B and W will read), *m_w after B (what is kept for W: the inputs and output
 * gradients of the four linears of every layer, Table 1).  Feeds zb_memory_model. */
zb_status zb_stage_stash_bytes(const zb_stage* st, double* m_b, double* m_w);

/* Per-kernel timing.  While enabled, every kernel launch is bracketed by HIP events on the
 * stage's stream (this slows the stream down: measure throughput with profiling off).
 * zb_profile_read waits for the device and fills up to cap rows, one per kernel class. */
typedef struct {
  char name[48];
  int64_t launches;
  double total_ms;
  double flops;  /* algorithmic FLOPs summed over those launches (0 for bandwidth kernels) */
  double bytes;  /* algorithmic HBM bytes summed over those launches */
} zb_kernel_stat;
zb_status zb_profile_enable(zb_stage* st, int32_t on); /* on=1 also clears the statistics */
zb_status zb_profile_read(zb_stage* st, zb_kernel_stat* out, int32_t cap, int32_t* n);

#ifdef __cplusplus
}
#endif
#endif /* ZB_STAGE_H */
