/*
 * mammoth_hip.h - C ABI of the MI355X (gfx950) library for the routed encoder-decoder
 * training step of modular translation models.
 *
 * What the calls mean follows the paper's problem statement:
 *   - a *task* is a translation direction bound to a fixed, ordered set of modules
 *     (section 3.2 "Design principles"); modules are specific to a sequential position, every
 *     task involves the same number of modules, and the number of layers belongs to the module
 *     position (the enc_layers / dec_layers keys);
 *   - one training step runs a batch through the task's modules in order, h_i = T_i(h_{i-1}),
 *     and produces a gradient for exactly those modules; modules outside the task keep a zero
 *     gradient; before the update a module's summed gradient is divided by n_j, the number of
 *     times it was used (Algorithm 1).  This library is the one-GPU share of that algorithm:
 *     sums over devices do not occur, n_j counts uses on this GPU since the last update.
 *
 * Conventions
 *   - Every call returns an mm_status; nothing throws or exits across the ABI.
 *   - Pointers are HOST pointers unless a parameter comment says "device".  The caller owns
 *     every buffer it passes; buffers are borrowed for the duration of the call only.
 *   - The library owns parameters, gradient buckets, optimiser state and workspace (device
 *     memory obtained with hipMalloc on the current device at creation/registration time).
 *   - All work is enqueued on one HIP stream (mm_config.hip_stream, NULL = the default stream).
 *     One context = one GPU = one stream; calls on one context must not overlap.
 *   - On an error detected before launch (bad ids, lengths, task, sizes) nothing is changed.
 *   - Matrices at the ABI are [in, out] row-major fp32; a module's tensors live in one flat
 *     fp32 vector ("bucket layout", see mm_get_layout); each tensor starts at a multiple of 64
 *     elements and the vector length is a multiple of 64; gaps hold zeros.
 */
#ifndef MAMMOTH_HIP_H
#define MAMMOTH_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mm_ctx mm_ctx; /* opaque */

typedef enum {
  MM_OK = 0,
  MM_EINVAL = -1,     /* malformed argument (NULL, bad enum, inconsistent sizes, route rule broken) */
  MM_ENOMEM = -2,     /* device or host allocation failed */
  MM_ESTATE = -3,     /* call not valid in this state (e.g. compute on a plan-only context) */
  MM_ERANGE = -4,     /* token id outside [0, vocab), length outside its limits, non-pad after the end */
  MM_ENONFINITE = -5, /* the step's loss is not finite (gradients of the step have been added) */
  MM_EHIP = -6        /* a HIP runtime call failed; mm_last_error names it */
} mm_status;

typedef enum { MM_F32 = 0, MM_BF16 = 1 } mm_dtype;
typedef enum {
  MM_SRC_EMB = 0, MM_ENC_STACK = 1, MM_TGT_EMB = 2, MM_DEC_STACK = 3, MM_GENERATOR = 4, MM_ADAPTER = 5
} mm_kind;
typedef enum { MM_HOST = 0, MM_DEVICE = 1 } mm_memspace;
typedef enum { MM_T_MATRIX = 0, MM_T_EMBED = 1, MM_T_BIAS = 2, MM_T_GAMMA = 3, MM_T_BETA = 4 } mm_tensor_role;

/* Model shape shared by all modules of a context (paper section 4: d=512, 8 heads, FFN 2048). */
typedef struct {
  int32_t d_model;          /* multiple of 16; d_model / n_heads in {16, 32, 64}                  */
  int32_t n_heads;
  int32_t d_ff;             /* multiple of 16                                                     */
  int32_t vocab;            /* multiple of 8; id 0 = pad                                          */
  int32_t dtype;            /* mm_dtype: storage of activations and working weights; master,
                               gradients and optimiser state are always fp32                     */
  float label_smoothing;    /* epsilon of the uniform smoothing over all vocab classes            */
  float adam_beta1, adam_beta2, adam_eps;
  float ln_eps;
  int32_t max_len;          /* longest source sentence / longest decoder input                    */
  int32_t max_batch_tokens; /* upper bound on sum of source lengths and on sum of (t_b - 1)       */
  void* hip_stream;         /* hipStream_t, borrowed; NULL = default stream                       */
  int32_t plan_only;        /* 1: no device memory; registry, layouts, routes and batch checks
                               work, compute calls return MM_ESTATE                              */
} mm_config;

/* One module; a module belongs to one position of its stack (section 3.2, the second design constraint). */
typedef struct {
  int32_t kind;             /* mm_kind                                                            */
  int32_t position;         /* index in the encoder / decoder module sequence (stacks only)       */
  int32_t n_layers;         /* layers of this stack module; for an adapter: layers of the whole
                               stack it attaches to (one bottleneck per layer)                   */
  int32_t owns_final_norm;  /* 1 for the module at the last position of its stack                 */
  int32_t adapter_dim;      /* MM_ADAPTER only: bottleneck width (multiple of 16)                  */
  int32_t adapter_stack;    /* MM_ADAPTER only: 0 = encoder stack, 1 = decoder stack              */
  const char* name;         /* sharing-group name, informational, copied                          */
} mm_module_desc;

mm_status mm_create(const mm_config* cfg, mm_ctx** out);
mm_status mm_destroy(mm_ctx* ctx);

/* Registers a module and allocates its parameters (fp32 master, working copy), its gradient
 * bucket (zeroed) and Adam state (zeroed, step count 0).
 * init_fp32: flat vector in bucket layout, n_params long, or NULL for zeros; n_params must
 * equal the module's bucket length (ignored when init_fp32 is NULL).  out_module_id receives
 * ids 0, 1, 2, ... in registration order. */
mm_status mm_register_module(mm_ctx* ctx, const mm_module_desc* desc, const float* init_fp32,
                             int64_t n_params, int32_t* out_module_id);

/* Defines a task by its ordered module list: src_emb, enc stack modules by position 0..,
 * tgt_emb, dec stack modules by position 0.., generator, then at most one adapter per stack.
 * Checks the paper's two rules - every task has the same number of modules as the first one,
 * and a module is only used at the position it was defined for - plus: the last position of a
 * stack (and only it) owns the final norm, an adapter covers every layer of its stack, no
 * module appears twice.  Violations return MM_EINVAL and define nothing. */
mm_status mm_route_task(mm_ctx* ctx, const int32_t* module_ids, int32_t n_modules, int32_t* out_task_id);

/* One forward+backward pass of one batch of one task (Algorithm 1, forward and backward parts):
 * gradients of the mean label-smoothed cross-entropy over the real target tokens are ADDED to
 * the buckets of the task's modules, whose use counts n_j grow by one; no other module's
 * memory is read or written.
 *   src_ids [B, S_max] row-major int32: s_b content ids then pad (0).
 *   tgt_ids [B, T_max] row-major int32: BOS ... EOS (t_b ids) then pad; the decoder reads
 *           positions 0..t_b-2 and predicts positions 1..t_b-1.
 *   ids_mem says where src_ids/tgt_ids live.  MM_HOST: checked on the host before anything is
 *           launched.  MM_DEVICE (device pointers valid on the context's stream): checked by the
 *           first kernel; a bad id turns the whole step into a no-op on the buckets.
 *   lengths [B, 2] int32 (host) = (s_b, t_b) with 1 <= s_b <= S_max <= max_len,
 *           2 <= t_b <= T_max <= max_len + 1.
 *   out_loss (host, may be NULL): receives the loss; writing it is the call's only
 *           synchronisation with the stream.  With NULL the call returns once the work is
 *           enqueued and id/finite checks are reported by the next mm_last_loss call. */
mm_status mm_train_step(mm_ctx* ctx, int32_t task, const int32_t* src_ids, const int32_t* tgt_ids,
                        const int32_t* lengths, int32_t B, int32_t S_max, int32_t T_max,
                        int32_t ids_mem, float* out_loss);

/* Greedy translation of one batch of one task with the task's own modules only (section 3.2,
 * "inference": a task needs just its modules loaded; no other module's memory is read, and no
 * bucket, use count or Adam state is written).  The search itself is the plainest one: every
 * sentence starts from BOS (id 1); each step feeds the last token back, takes the largest
 * generator logit (the lowest id among equal ones) and stops the sentence at EOS (id 2) or after
 * max_new tokens.
 *   src_ids [B, S_max] row-major int32 as for mm_train_step (ids_mem: MM_HOST or MM_DEVICE).
 *   src_lengths [B] int32 (host), 1 <= s_b <= S_max <= max_len;  1 <= max_new <= max_len.
 *   out_ids [B, max_new] int32 (host, caller-owned): produced ids, EOS included, then pad (0).
 *   out_lengths [B] int32 (host): number of ids produced per sentence.
 * Synchronous: returns when the outputs are written.  A training step still in flight is
 * waited for first.  Errors as for mm_train_step; on error the outputs are unspecified.
 * The call reuses the training step's workspace and id tables: mm_debug_dump afterwards
 * describes this call's batch (with a two-token target BOS EOS per sentence), not the last
 * training step's. */
mm_status mm_translate_greedy(mm_ctx* ctx, int32_t task, const int32_t* src_ids, const int32_t* src_lengths,
                              int32_t B, int32_t S_max, int32_t max_new, int32_t ids_mem,
                              int32_t* out_ids, int32_t* out_lengths);

/* Beam search with the task's own modules (same property as mm_translate_greedy: only the task's
 * modules are read, no training state is written).  The paper names no search procedure; this is
 * the textbook one: per sentence `beam` hypotheses, best first, starting from the empty one at
 * score 0; each step an unfinished hypothesis extended by token v scores its own score plus
 * log softmax(logits)[v] (fp32), a hypothesis that ended in EOS (id 2) is carried at its score; the
 * `beam` best candidates form the next beam, equal scores going to the lower hypothesis, then
 * the lower token id; no length normalisation.  The search ends when every hypothesis of every
 * sentence is finished or after max_new tokens; the first hypothesis of each beam is returned.
 * beam = 1 produces what mm_translate_greedy produces.
 *   1 <= beam <= 8; B * beam <= max_batch_tokens; other arguments as for mm_translate_greedy.
 *   out_scores [B] float (host, may be NULL): summed log-probability of the returned hypothesis.
 * Synchronous; errors and the note on mm_debug_dump as for mm_translate_greedy. */
mm_status mm_translate_beam(mm_ctx* ctx, int32_t task, const int32_t* src_ids, const int32_t* src_lengths,
                            int32_t B, int32_t S_max, int32_t max_new, int32_t beam, int32_t ids_mem,
                            int32_t* out_ids, int32_t* out_lengths, float* out_scores);

/* Waits for the most recent mm_train_step and returns its loss and status. */
mm_status mm_last_loss(mm_ctx* ctx, float* out_loss);

/* Renormalise and update (Algorithm 1 last line, then Adam): for every listed module with
 * n_j > 0: g = bucket / n_j; t_j += 1; Adam step on the fp32 master with bias correction for
 * step t_j; working copy refreshed; bucket emptied; n_j = 0.  Modules with n_j = 0 are skipped:
 * not one byte of theirs is read or written.  module_ids NULL = every module.
 * A training step whose ids turned out bad on the device had no effect: its uses are not
 * counted, and a module left without a use gets no update.  That also holds for a step still in
 * flight, without the call waiting for it: the update is enqueued behind the step and reads the
 * step's outcome on the device; n_j and t_j as the host reports them (mm_get_touched,
 * mm_get_adam) are settled when they are next asked for.  The step's status stays available from
 * mm_last_loss.  The update itself is enqueued and not waited for. */
mm_status mm_apply_update(mm_ctx* ctx, const int32_t* module_ids, int32_t n, float lr);

/* mm_apply_update for callers that cannot allocate device or pinned memory inside the call (tight
 * serving or training loops, harnesses that forbid hipMalloc): same arguments, same result, but
 * the table of per-module segments the update kernel reads lives in a static device array of the
 * library (18 KiB per GPU, held until the process ends) instead of a buffer that grows on demand,
 * and the call makes no hipMalloc / hipHostMalloc / hipFree and creates no events.  At most
 * MM_NOALLOC_MAX_MODULES modules with n_j > 0 can be updated by one call; more returns MM_ERANGE
 * and changes nothing.  Every context on one GPU shares that GPU's array: calls that overlap in
 * time on one GPU (two contexts, two streams) race on it; calls on one context's stream are
 * ordered and safe.  The update kernel is not timed by mm_profile. */
#define MM_NOALLOC_MAX_MODULES 256
mm_status mm_apply_update_noalloc(mm_ctx* ctx, const int32_t* module_ids, int32_t n, float lr);

/* ---- introspection (tests, checkpoints); all synchronise with the stream ------------------- */
mm_status mm_num_modules(mm_ctx* ctx, int32_t* out_n);
/* ids/n: capacity in *n on entry, count on return. */
mm_status mm_get_route(mm_ctx* ctx, int32_t task, int32_t* ids, int32_t* n);
/* counts[j] = n_j for every module j (array of mm_num_modules entries). */
mm_status mm_get_touched(mm_ctx* ctx, int32_t* counts, int32_t capacity);
/* Tensor table of a module in bucket order.  Arrays hold *n_tensors entries on entry (capacity)
 * and the count on return; any array may be NULL.  rows/cols: matrix [rows=in, cols=out],
 * embedding [vocab, d], vectors rows = 1. */
mm_status mm_get_layout(mm_ctx* ctx, int32_t module, int64_t* offsets, int32_t* rows, int32_t* cols,
                        int32_t* roles, int32_t* n_tensors, int64_t* bucket_len);
mm_status mm_get_params(mm_ctx* ctx, int32_t module, float* dst, int64_t n);
mm_status mm_set_params(mm_ctx* ctx, int32_t module, const float* src, int64_t n);
/* The module's bucket: the sum of the gradients of its uses since its last update (Algorithm 1),
 * all zeros when n_j = 0. */
mm_status mm_get_grads(mm_ctx* ctx, int32_t module, float* dst, int64_t n);
/* The bucket's memory as it stands.  Differs from mm_get_grads only when n_j = 0: the update
 * zeroes the buckets of embedding tables but leaves those of stacks, generators and adapters as
 * they are, because the next step that uses such a module writes every element of its bucket
 * (first use overwrites, later uses add).  A module that was never used reads all zeros. */
mm_status mm_get_bucket_memory(mm_ctx* ctx, int32_t module, float* dst, int64_t n);
/* Overwrites a bucket and its use count (to test the update in isolation). */
mm_status mm_set_grads(mm_ctx* ctx, int32_t module, const float* src, int64_t n, int32_t n_uses);
mm_status mm_get_adam(mm_ctx* ctx, int32_t module, float* m, float* v, int64_t n, int64_t* t_j);
/* Working copy widened to fp32 (bf16 contexts: the rounded values the kernels read). */
mm_status mm_get_working(mm_ctx* ctx, int32_t module, float* dst, int64_t n);

/* Integer by-products of the most recent step, for bit-exact checks.  *nbytes: capacity on
 * entry, size on return. */
typedef enum {
  MM_DUMP_CU_SRC = 0,     /* int32[B+1] prefix sums of s_b                                        */
  MM_DUMP_CU_DEC = 1,     /* int32[B+1] prefix sums of t_b - 1                                    */
  MM_DUMP_SRC_TOK = 2,    /* int32[S] gathered source ids, sentence after sentence                */
  MM_DUMP_SRC_POS = 3,    /* int32[S] their positions                                             */
  MM_DUMP_DEC_TOK = 4,    /* int32[U] decoder input ids                                           */
  MM_DUMP_DEC_POS = 5,    /* int32[U]                                                             */
  MM_DUMP_LABEL = 6,      /* int32[U] labels                                                      */
  MM_DUMP_MASK_ENC = 7,   /* uint8[B, S_max, S_max]: 1 where query i must not see key j           */
  MM_DUMP_MASK_DEC = 8,   /* uint8[B, T_max-1, T_max-1] (causal and length)                       */
  MM_DUMP_MASK_CROSS = 9  /* uint8[B, T_max-1, S_max]                                             */
} mm_dump_what;
mm_status mm_debug_dump(mm_ctx* ctx, int32_t what, void* dst, int64_t* nbytes);

/* Test hook on the attention kernels themselves (section 3.2 fixes no network internals; the
 * benchmark's contract asks that blocked keys get probability exactly 0).  Returns the attention
 * probabilities of one attention block of the most recent mm_train_step as that step's own forward
 * attention kernel computes them: the kernel is run again on the step's saved queries and keys
 * with one-hot value rows (the value row of a sentence's key j is unit vector j mod d_h; one pass
 * per group of d_h keys), so each output row IS a probability row with the kernel's masking,
 * tile skipping and softmax, rounded to the working dtype.
 *   kind: 0 encoder self-attention, 1 decoder self-attention, 2 decoder attention over the
 *         encoder output; layer: index of the block within its stack, in forward order.
 *   probs: host float [B, H, Lq, Lk] with Lq, Lk the step's padded widths (S_max or T_max - 1);
 *          entries beyond a sentence's own lengths are 0.  NULL: only *n_floats is set.
 *   *n_floats: capacity on entry, size on return.
 * Valid until the next compute call on the context.  Synchronous; allocates temporaries. */
mm_status mm_debug_attention(mm_ctx* ctx, int32_t kind, int32_t layer, float* probs, int64_t* n_floats);

/* ---- per-kernel-class timing with HIP events on the context's stream ----------------------- */
typedef enum {
  MM_K_GEMM = 0, MM_K_ATTN_FWD = 1, MM_K_ATTN_BWD = 2, MM_K_LAYERNORM_FWD = 3, MM_K_LAYERNORM_BWD = 4,
  MM_K_EMBED = 5, MM_K_EMBED_GRAD = 6, MM_K_CE = 7, MM_K_COLSUM = 8, MM_K_ADAM = 9, MM_K_OTHER = 10,
  MM_K_COUNT = 11
} mm_kernel_class;
/* enable = 1: an event is recorded after every launch (and one at the start of each call); a launch
 * is charged the stream time since the event before it, and its algorithmic work (flops for
 * GEMM/attention, bytes for the rest) is tallied; enable = 0 stops.  Counters reset on enable. */
mm_status mm_profile(mm_ctx* ctx, int32_t enable);
/* Arrays of MM_K_COUNT entries: total milliseconds, launches, algorithmic work (flops or bytes). */
mm_status mm_profile_read(mm_ctx* ctx, double* ms, int64_t* launches, double* work);

const char* mm_last_error(mm_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* MAMMOTH_HIP_H */
