/*
 * pass.h -- C ABI of the MI355X (gfx950) hot path of PaSS, parallel speculative sampling.
 *
 * The library runs the (1+k)-row decode step that the method calls twice per iteration
 * (Section 2.2 of the paper): a drafting call on the last token plus k look-ahead embeddings
 * (Section 2.2.1), and a validation call on the drafted block followed by the accept / reject
 * chain of Algorithm 1.  Around it: the prompt pass that fills the cache, two-model speculative
 * sampling (the appendix's Algorithm 2) on the same validation call, and the training of the
 * look-ahead embeddings against the frozen model (Training details).  Every step of these paths
 * runs in HIP kernels; there is no CPU fallback.
 *
 * Conventions
 *   - Every function returns PASS_OK (0) or a negative pass_status; nothing throws or aborts.
 *     pass_last_error() gives a message for the last failure on that context.
 *   - "host" / "device" on a pointer says where the memory lives.  Pointers are borrowed for
 *     the duration of the call only, except the arena given to pass_create, which the caller
 *     owns and must keep alive (and not touch) until pass_destroy.
 *   - The library allocates no device memory: K/V pages, packed weights, workspaces and
 *     per-slot state all live in the caller's arena (pass_arena_bytes tells how large); what
 *     training the look-ahead embeddings needs lives in a second workspace of the caller's
 *     (pass_train_bytes, pass_train_begin).
 *   - All work is issued on the HIP stream given to pass_create.  Calls that return results to
 *     host memory synchronise that stream before returning.
 *   - One context may be used from one thread at a time.
 *
 * Per-slot invariant between calls:  kv_len == (#tokens of the sequence) - 1;  the last token
 * is "pending": its K/V are computed by the next call.  K/V rows beyond kv_len are dead and are
 * overwritten by the next call; rolling the cache back after a rejection is not advancing
 * kv_len (the paper's Baselines paragraph: the cache is updated after every call according to
 * the number of drafted and accepted tokens).
 *
 * Notation: k is the number of look-ahead embeddings (L in Algorithm 1); p_t is the target
 * distribution of the validation call, d_t the draft distribution of the drafting call, both
 * softmax(logits / temperature).
 */
#ifndef PASS_H_
#define PASS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pass_ctx pass_ctx;

typedef enum {
  PASS_OK = 0,
  PASS_EINVAL = -1,    /* bad argument, bad slot, unsupported shape                         */
  PASS_ESTATE = -2,    /* call out of order (draft needs a prefilled slot, verify a drafted) */
  PASS_ECAPACITY = -3, /* kv_len + 1 + k would exceed max_seq_len, or the page pool is empty */
  PASS_EDEVICE = -4    /* a HIP call failed                                                  */
} pass_status;

enum { PASS_F32 = 0, PASS_BF16 = 1 };
enum { PASS_MAX_K = 15, PASS_MAX_ROWS = 64 };

/* Shape of a LLaMA-style decoder (pre-norm RMSNorm, rotary embedding on interleaved pairs,
 * SwiGLU, multi-head attention with n_heads * head_dim projection width, untied LM head) --
 * the paper's Experiments section runs a re-implementation of LLaMA-7B in bfloat16. */
typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_base;
  int32_t dtype;       /* PASS_F32 / PASS_BF16: storage type of every model tensor and of K/V  */
  int32_t k;           /* look-ahead embeddings per drafting call, 0 .. PASS_MAX_K             */
  int32_t max_slots;   /* concurrent sequences; (1+k) * max_slots <= PASS_MAX_ROWS             */
  int32_t max_seq_len; /* per-sequence limit on cached positions                               */
  int32_t page_size;   /* positions per K/V page (power of two, >= 16)                         */
  int32_t n_pages;     /* pages in the pool; 0 = max_slots * ceil(max_seq_len / page_size)     */
} pass_config;

typedef struct {
  float temperature;   /* 0 = greedy (every sample is an argmax, lowest index on ties)         */
  int32_t top_k;       /* 0 = no filter; K > 0 = top-k sampling (Experimental setup: k = 10, 25): the
                          draft and the target distribution are each the softmax over the row's own
                          K largest logits (boundary ties keep the lower indices), zero elsewhere;
                          ignored when temperature is 0; K >= vocab filters nothing; negative: EINVAL */
  uint64_t seed;       /* Philox4x32-10 key; streams are separated by sequence id, iteration,
                          row and purpose, so results do not depend on batch composition      */
} pass_sampling;

typedef struct {
  int64_t iterations;       /* PaSS iterations (draft + verify), summed over slots            */
  int64_t drafts_proposed;  /* k per iteration and slot                                       */
  int64_t drafts_accepted;
  int64_t tokens_out;       /* tokens written to out_tokens                                   */
  double draft_ms, verify_ms; /* device time of the two calls, summed over iterations         */
} pass_stats;

/* Model tensors in their plain layout: matrices are [out_features, in_features] row-major,
 * element type config.dtype.  Arrays of per-layer pointers live in host memory. */
typedef struct {
  const void *tok_emb;    /* [vocab, d_model]                                                */
  const void *lm_head;    /* [vocab, d_model]                                                */
  const void *final_norm; /* [d_model]                                                       */
  const void *lookahead;  /* [k, d_model] look-ahead embeddings (Section 2.2.1); NULL if k==0 */
  const void *const *attn_norm, *const *wq, *const *wk, *const *wv, *const *wo;
  const void *const *ffn_norm, *const *w_gate, *const *w_up, *const *w_down;
} pass_weights;

/* Bytes of device memory pass_create needs for this configuration (0 if it is invalid). */
size_t pass_arena_bytes(const pass_config *cfg);

/* Create a context.  hip_stream: a hipStream_t (NULL = the null stream).  device_arena:
 * device memory of at least pass_arena_bytes(cfg) bytes, 256-byte aligned, owned by the caller.
 * Errors: PASS_EINVAL (shape not supported, arena too small or misaligned), PASS_EDEVICE. */
int pass_create(const pass_config *cfg, void *hip_stream, void *device_arena, size_t arena_bytes,
                pass_ctx **out);

/* Copy the model into the arena, repacking matrices into the layout the kernels stream
 * (tiles of 16 rows x 32 columns for the bf16 matrix-core path).  on_device = 0: tensor
 * pointers are host memory; 1: device memory.  The caller may free its tensors afterwards. */
int pass_load_weights(pass_ctx *ctx, const pass_weights *w, int on_device);

/* Start a sequence in `slot` (frees what the slot held).  prompt: host, n >= 1 token ids.
 * Computes K/V of prompt[0..n-2]; prompt[n-1] becomes the pending token, so the first
 * drafting call is already a parallel one (Algorithm 1 starts from the prompt x_0..x_t).
 * seq_id selects the sequence's random streams.  Prompts of more than 2 * PASS_MAX_ROWS rows on
 * the matrix-core path go through tiled, compute-bound kernels, up to 2048 rows per pass over the
 * weights; shorter ones (and every prompt on the generic path) through the decode kernels,
 * PASS_MAX_ROWS rows per pass ("prefill_*" options).  Returns when the cache is filled.
 * Errors: PASS_EINVAL (slot, token ids), PASS_ESTATE (no weights), PASS_ECAPACITY (the prompt
 * plus one call's rows exceed max_seq_len, or the page pool is exhausted). */
int pass_prefill(pass_ctx *ctx, int slot, uint32_t seq_id, const int32_t *prompt, int n);

/* pass_prefill for several sequences at once (Algorithm 1's "initial prompt sequence" of a batch; the prefixes
 * of a training batch): slots[n_slots] distinct, seq_ids[n_slots], lens[n_slots] >= 1, prompts: the prompts one
 * after the other (host, sum of lens tokens).  The state afterwards is what n_slots calls of pass_prefill
 * leave.  Where the tiled kernels apply (matrix-core path, more than 2 * PASS_MAX_ROWS rows in all), rows of
 * several sequences share a pass over the weights: every sequence starts on a block of 128 rows of the pass, a
 * prompt that does not fit goes on in the next pass, attention runs per sequence.  A row's arithmetic is that of
 * pass_prefill up to the grouping of the RMSNorm's partial sums, which follows the pass's row count (logits
 * agree to rounding, not bit for bit).  Elsewhere the prompts go one by one.  Returns when the caches are filled.
 * Errors as pass_prefill, and PASS_EINVAL for a slot listed twice; slots before the failing one may already
 * have been restarted. */
int pass_prefill_batch(pass_ctx *ctx, const int32_t *slots, const uint32_t *seq_ids, const int32_t *prompts,
                       const int32_t *lens, int n_slots);

/* Release a slot's pages. */
int pass_release(pass_ctx *ctx, int slot);

/* Drafting phase (Algorithm 1, first step of the loop; Section 2.2): one model call on
 * (pending, [LA]_1..[LA]_k) per slot; samples x_{n+1} from row 0 and draft t from row t, in
 * parallel.  Afterwards kv_len += 1 and pending = x_{n+1}.  slots: host, n_slots distinct
 * slot numbers, all prefilled / verified.  out_first: host [n_slots]; out_drafts: host
 * [n_slots * k] or NULL. */
int pass_draft(pass_ctx *ctx, const int32_t *slots, int n_slots, const pass_sampling *sp,
               int32_t *out_first, int32_t *out_drafts);

/* pass_draft for callers that cannot allocate device memory and whose harness forbids a library
 * to do so on their behalf: code under HIP graph capture, tight serving loops.  Same arguments,
 * results and errors as pass_draft; what differs is where the call's scratch lives: the attention
 * partials (running maximum, sum and accumulator of every row, head and split) go to a static
 * device array of 8 MiB inside the library instead of the arena, and the kernels are launched
 * directly (no graph is instantiated).  The call allocates nothing, on the device or through any
 * library routine that does.  Limit: rows * n_heads * 32 * (head_dim + 2) * 4 bytes <= 8 MiB with
 * rows = n_slots * (1 + look-ahead rows), i.e. 12 rows of a 40-head model, 15 of a 32-head one;
 * beyond it PASS_ECAPACITY and nothing has run.  Every call on a GPU shares that GPU's array, which
 * keeps the last call's contents (nothing in it needs clearing: every entry a call reads, that
 * call has written): calls that overlap on one GPU, from two contexts or two threads, race. */
int pass_draft_static(pass_ctx *ctx, const int32_t *slots, int n_slots, const pass_sampling *sp,
                      int32_t *out_first, int32_t *out_drafts);

/* Validation phase (Algorithm 1, second model call and the for-loop): one call on
 * (x_{n+1}, drafts); draft t is accepted iff r_t < min(1, p_t(x)/d_t(x)), in order, until the
 * first reject, which is replaced by a sample from the normalised (p_t - d_t)_+; if all k are
 * accepted one more token is sampled from the last row.  Afterwards kv_len += 1 + a and
 * pending = the final token.  out_n_accepted: host [n_slots]; out_tokens: host
 * [n_slots * (k+1)], per slot the a accepted drafts followed by the final token. */
int pass_verify(pass_ctx *ctx, const int32_t *slots, int n_slots, const pass_sampling *sp,
                int32_t *out_n_accepted, int32_t *out_tokens);

/* One iteration of two-model speculative sampling (Algorithm 2 of the appendix, the method PaSS is
 * compared with and whose validation phase it shares): `drafter` is a second context holding a
 * smaller model with the same vocabulary, run with single-row calls (k = 0, or "lookahead_rows" 0);
 * target slot t_slots[i] and drafter slot d_slots[i] hold the same sequence (both prefilled with the
 * same prompt and the same seq_id).  L = the target's look-ahead rows.  Per slot pair: L sequential
 * calls of the drafter, each drawing draft t from its row with the random stream of draft row t of
 * the target's iteration; then the target's one call on (last token, drafts) and the accept / reject
 * chain, residual draw and extra token exactly as in pass_verify (row t-1 of the call is the target
 * distribution for draft t).  Afterwards the target slot has kv_len += 1 + a and a + 1 new tokens,
 * and the drafter slot holds the same sequence again (cache rows of rejected drafts are dead; when all
 * L drafts were accepted one more drafter call makes the missing row).  The drafter's logits rows are
 * kept as the target slot's drafting logits (rows 1 .. L of pass_get_logits(.., 0, ..)).
 * out_drafts: host [n_slots * k] or NULL; out_n_accepted: host [n_slots]; out_tokens: host
 * [n_slots * (k+1)], per slot the a accepted drafts followed by the final token, the rest -1.
 * Errors as pass_verify, plus PASS_EINVAL (same context twice, vocabularies differ, drafter not in
 * single-row mode) and PASS_ESTATE (a slot pair does not hold the same sequence); a failure of the
 * drafter is reported on the target context with the drafter's message. */
int pass_sps_iteration(pass_ctx *target, pass_ctx *drafter, const int32_t *t_slots, const int32_t *d_slots,
                       int n_slots, const pass_sampling *sp, int32_t *out_drafts, int32_t *out_n_accepted,
                       int32_t *out_tokens);

/* Algorithm 1's while loop for a batch of prefilled slots: draft + verify until every slot has
 * produced at least max_new tokens; out_tokens: host [n_slots * max_new], the first max_new
 * tokens of each.  out_stats may be NULL.  Slots that finish early keep stepping with the
 * batch (their extra tokens are dropped) so the launch shape stays fixed. */
int pass_generate(pass_ctx *ctx, const int32_t *slots, int n_slots, int max_new,
                  const pass_sampling *sp, int32_t *out_tokens, pass_stats *out_stats);

/* The body of Algorithm 1's loop exactly n_iters times for a batch of slots (no length target):
 * the serving-loop primitive.  Tokens accumulate in the per-slot token buffer; out_stats (may be
 * NULL) counts them.  Iteration i + 1 is issued before the report of iteration i has been read (the
 * device never waits for the host; K/V pages are provided for an upper bound of the lengths
 * meanwhile); on return, also with an error, the host's view of the slots is exact again.
 * Errors: PASS_ECAPACITY when a slot cannot take another iteration (every iteration that fits has
 * been run). */
int pass_run_iterations(pass_ctx *ctx, const int32_t *slots, int n_slots, int n_iters,
                        const pass_sampling *sp, pass_stats *out_stats);

/* Training of the look-ahead embeddings (Training details of the paper; Section 2.2.1): every
 * parameter of the model is frozen, only the k x d_model look-ahead embeddings learn.  One step takes
 * a batch of prefilled slots (slot b holds the prefix w_1 .. w_T of a training sequence, cut at a
 * position the caller draws at random: K/V of w_1 .. w_{T-1} cached, w_T pending), runs the block
 * (w_T, [LA]_1 .. [LA]_k) through the model, takes the mean cross-entropy of the look-ahead rows
 * (row [LA]_i predicts targets[b * k + i - 1] = w_{T+1+i}; the row of w_T carries no loss), carries
 * its gradient back through the frozen model to the look-ahead rows, and applies AdamW (decoupled
 * weight decay; the paper: learning rate 0.01 after a linear warm-up, cosine schedule, batches of
 * 8 sequences -- the schedule is the caller's: it passes each step's learning rate).  The trained
 * values are fp32 ("master") and enter the forward pass unrounded; after every step the model's
 * own look-ahead tensor is refreshed from them in its storage type, so pass_draft uses what was
 * learned.  Slots are left as they were (the block's K/V rows lie beyond kv_len: dead).
 * Both kernel paths train.  On the matrix-core path (bf16 models, the default) the forward pass is
 * the drafting call's and every backward product runs on a packed transpose of its weight matrix,
 * which pass_train_begin builds inside the workspace: the workspace then holds a second copy of
 * the model's matrices, and d_model, n_heads * head_dim and d_ffn must be multiples of 64, the
 * vocabulary a multiple of 32 (else PASS_ESTATE: load such a model with option "path" = 1).
 *   pass_train_bytes   device bytes pass_train_begin needs for this context, after pass_load_weights
 *                      (0: no context, no weights, or k = 0)
 *   pass_train_begin   device_workspace: caller's device memory (256-byte aligned, kept alive while
 *                      training); the embeddings start from the embedding of init_token (the paper:
 *                      [UNK]) or, with init_token < 0, from the model's own look-ahead tensor;
 *                      AdamW's moments and step count start at zero; pass_load_weights ends the set-up
 *   pass_train_step    slots: host, n_slots prefilled slots, (1+k) * n_slots <= PASS_MAX_ROWS, at most
 *                      8192 keys each; targets: host [n_slots * k]; *out_loss: the batch loss before
 *                      the update (may be NULL).  Returns when the step is done.
 *   pass_train_read    what = 0: the master values, 1: the gradient of the last step, 2 / 3: AdamW's first /
 *                      second moment; out: host [k * d_model]
 *   pass_train_resume  restores a saved training state: master values, moments (host [k * d_model] each; a
 *                      NULL pointer leaves that part as it is) and the number of optimiser steps taken so
 *                      far (it enters AdamW's bias correction); the model's own look-ahead tensor follows
 *                      the master values
 * Errors: PASS_ESTATE (no pass_train_begin, look-ahead options not at their defaults, a shape the
 * path cannot train, d_model above 8192), PASS_EINVAL, PASS_ECAPACITY. */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
} pass_adamw;
size_t pass_train_bytes(pass_ctx *ctx);
int pass_train_begin(pass_ctx *ctx, void *device_workspace, size_t bytes, int32_t init_token);
int pass_train_step(pass_ctx *ctx, const int32_t *slots, int n_slots, const int32_t *targets, const pass_adamw *opt,
                    float *out_loss);
int pass_train_read(pass_ctx *ctx, int what, float *out);
int pass_train_resume(pass_ctx *ctx, const float *master, const float *m1, const float *m2, int64_t steps);

/* Parity hook: fp32 logits [(1+k) * vocab] of the slot's last drafting (which = 0) or
 * validation (which = 1) call, copied to host memory. */
int pass_get_logits(pass_ctx *ctx, int slot, int which, float *out);

/* Parity hook for the random numbers of Algorithm 1 ("sample", "r ~ U[0,1]"): the uniform variates
 * the device epilogues attach to vocabulary indices first .. first + n - 1 of one (seed, sequence id,
 * iteration, row, purpose), computed by the epilogues' own generator (Philox4x32-10, key = seed,
 * counter = (index / 4, iteration, row | purpose << 8, sequence id), word index % 4; top 23 bits ->
 * (bits + 0.5) * 2^-23) and copied to the host array out[n].  purpose: 0 drafting draw, 1 accept test
 * (index 0 only is used by the method), 2 residual draw, 3 bonus draw.  The values pass through the
 * buffer of the validation call's logits: pass_get_logits(.., 1, ..) is stale afterwards until the
 * next validation call; sequence state is untouched.  PASS_EINVAL: row > 255, purpose > 3, first not
 * a multiple of 4, first + n beyond 2^32, out NULL. */
int pass_rng_uniforms(pass_ctx *ctx, uint64_t seed, uint32_t seq_id, uint32_t iteration, uint32_t row,
                      uint32_t purpose, uint32_t first, size_t n, float *out);

/* Tokens first .. first + n - 1 of everything the slot's sequence has generated since its prefill
 * (by pass_draft / pass_verify, pass_generate or pass_run_iterations), copied to the host array
 * out[n].  An iteration of Algorithm 1 adds 2 .. k + 2 tokens, so pass_generate may commit up to
 * k + 1 tokens beyond max_new to the sequence (and to the cache): they are part of the sequence,
 * the next call continues after them, and this call is how the caller reads them.
 * PASS_EINVAL: bad slot, first < 0, n < 0, out NULL; PASS_ESTATE: empty slot; PASS_ECAPACITY:
 * first + n exceeds the number of generated tokens (pass_seq_len). */
int pass_get_tokens(pass_ctx *ctx, int slot, int first, int n, int32_t *out);

/* Introspection hook for the split-KV attention of the matrix-core path (no context, no GPU): how a
 * group of query rows that sees n_keys cached positions of a model with n_heads heads is cut into
 * splits (*n_splits workgroups of *chunk_keys keys each; a function of the sequence's own length
 * only, so its arithmetic cannot depend on what else is batched), and *grid_splits, the grid width
 * the host launches for calls whose longest group has at most n_keys keys (never less than any
 * shorter group's split count).  Any output pointer may be NULL.  PASS_EINVAL: n_keys or n_heads < 1. */
int pass_attention_plan(int n_heads, int n_keys, int *n_splits, int *chunk_keys, int *grid_splits);

/* Introspection hook for pass_prefill_batch (no context, no GPU): how prompts of lens[n] tokens are packed into
 * tiled passes of at most rows_per_pass rows (a multiple of 128).  Prompt b has lens[b] - 1 rows to cache.  Writes
 * *n_segs and, for each segment in launch order, five values to out_segs: pass, prompt, first row of the prompt,
 * rows, first row in the pass (a multiple of 128).  PASS_EINVAL: bad arguments; PASS_ECAPACITY: more than max_segs
 * segments (*n_segs is still written; max_segs = 0 just counts). */
int pass_prefill_plan(int rows_per_pass, const int32_t *lens, int n, int max_segs, int32_t *out_segs, int *n_segs);

/* kv_len and number of generated tokens of a slot (either pointer may be NULL). */
int pass_seq_len(pass_ctx *ctx, int slot, int32_t *kv_len, int32_t *n_generated);

/* Options:
 *   "graph"            1 = replay each model call and its epilogue as a captured HIP graph; ignored when the
 *                      context runs on the null stream, which cannot be captured
 *   "path"             0 = auto, 1 = force the generic kernels; before pass_load_weights
 *   "attention"        0 = auto, 1 = never use the matrix-core attention kernel and its transposed V pages;
 *                      before pass_load_weights
 *   "lookahead_rows"   look-ahead rows per call from now on, 0 .. k: the drafting call uses the first that many
 *                      look-ahead embeddings; outputs and logits keep their k-sized layout with unused entries
 *                      -1 / stale (the paper's sweep over the number of look-ahead tokens without reloading)
 *   "lookahead_token"  -1 = trained look-ahead embeddings; a token id = the drafting call appends that token's
 *                      embedding instead (the paper's second baseline with a fixed [UNK] token).  Both only
 *                      between iterations, else PASS_ESTATE
 *   "kernel_timing"    1 = after every model call, launch the dominant kernel, the gate/up GEMM, once per layer
 *                      with that layer's weights on the call's rows, back to back between two HIP events on the
 *                      context's stream, and synchronise; the launches write workspaces only; setting the option
 *                      resets the counters pass_kernel_time reports
 *   "prefill_chunk"    1 .. PASS_MAX_ROWS: prompt rows per pass over the weights when the prompt goes through
 *                      the decode kernels
 *   "prefill_tiled"    -1 = prompts of more than 2 * PASS_MAX_ROWS rows take the tiled, compute-bound prompt pass
 *                      when the model runs on the matrix-core path with the matrix-core attention kernel,
 *                      0 = never, 1 = every prompt does
 * Names that start with "tune." are sweep knobs of the kernels' launch shapes for development; they are not part
 * of this interface and may change (they are listed where pass_set_option is defined).
 * Unknown names: PASS_EINVAL. */
int pass_set_option(pass_ctx *ctx, const char *name, int value);

/* Timed replay of one drafting-shaped step on the given slots without changing any sequence
 * state (no sampling state is committed): returns the mean device milliseconds of `iters`
 * steps after `warmup`.  Used by the benchmark to time the dominant kernels in isolation. */
int pass_time_step(pass_ctx *ctx, const int32_t *slots, int n_slots, int warmup, int iters,
                   double *out_ms);

/* Sum of the event-measured durations (ms) and the number of launches of the dominant kernel
 * since "kernel_timing" was last set. */
int pass_kernel_time(pass_ctx *ctx, double *total_ms, int64_t *launches);

/* Measurement yardstick: a kernel that only reads `bytes` bytes of the loaded model (16-byte
 * non-temporal loads, every workgroup a contiguous segment, nothing computed or written) is launched
 * `iters` times back to back on the context's stream, each launch on the next `bytes` of the weights
 * (wrapping around), between two HIP events; *out_us = mean duration of a launch in microseconds.
 * What a kernel that streams that many bytes once can at best take on this device.
 * PASS_EINVAL: bytes not a multiple of 16, zero, or more than the model holds; iters < 1.
 * PASS_ESTATE: no weights loaded. */
int pass_plain_read(pass_ctx *ctx, size_t bytes, int iters, double *out_us);

/* Message of the last failure on ctx; ctx == NULL: of the last failed pass_create. */
const char *pass_last_error(pass_ctx *ctx);
void pass_destroy(pass_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* PASS_H_ */
