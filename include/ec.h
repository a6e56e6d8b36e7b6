/*
 * ec.h - C ABI of the EntropyCache denoising step for AMD MI355X (gfx950).
 *
 * One context = one model (borrowed device weights) + one generation in flight: prompt, masked
 * generation slots, per-layer KV cache, decode history.  A denoising step is either FULL (every
 * position recomputes Q/K/V and overwrites the cache) or PARTIAL (only the masked positions of
 * the current block plus the recently decoded tokens recompute Q/K/V, scatter their K/V into the
 * cache and attend bidirectionally against the whole cached context).  After the forward pass
 * the step decodes tokens from the block's logits, evaluates the maximum entropy of the newly
 * decoded tokens and sets the flag that chooses the next step's mode.
 *
 * Paper passages: Method section ("Entropy-based skipping", Eq. 1; "Recent token
 * recomputation", Eq. 2, Eq. 3, tau_R, R), Algorithm 1, and the appendix "Full EntropyCache
 * algorithm".
 *
 * Conventions
 *  - Every call returns EC_OK or a negative error code; it never throws or aborts (a failed host
 *    allocation inside a call comes back as EC_ERR_HOST_MEMORY).  Outputs are
 *    written only on success.  ec_last_error() gives a message for the last failure of a context
 *    (or of ec_init when passed NULL).
 *  - Pointers marked DEVICE are device addresses on the current HIP device; HOST are host
 *    addresses.  Weights and workspace are BORROWED: the caller allocates them (e.g. through
 *    PyTorch), keeps them alive and unchanged while the context lives, and frees them afterwards.
 *    The context owns only small host-side state and one pinned host buffer.
 *  - All device work is enqueued on the HIP stream given to ec_init.  ec_step synchronises that
 *    stream once, for the read-back of its small result.
 *  - A context is not thread-safe.
 *  - batch sequences generate side by side and independently (own prompt, mask set, history,
 *    flag, block, cache): a step concatenates the rows each sequence recomputes, so the weights
 *    stream once for all of them; the results equal those of running each sequence alone.
 *    batch > 1 needs the bfloat16 path (EC_BF16 or EC_FP8W).  Per-sequence arguments and results are arrays of
 *    batch entries in sequence order.
 *  - All matrices are row-major [out_features, in_features] in the model's storage type
 *    (float32, bfloat16, or under EC_FP8W one e4m3 byte per element plus a float32 scale per
 *    row).  Norm gains and the embedding are float32 (EC_F32) or bfloat16.
 */
#ifndef EC_H
#define EC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EC_MAX_N 32        /* most tokens one step may unmask (tokens_per_step <= EC_MAX_N)   */
#define EC_MAX_BLOCK 128   /* largest block (window) size                                     */
#define EC_MAX_BATCH 64    /* most sequences of one context                                   */

typedef struct ec_ctx ec_ctx; /* opaque */

/* Storage type of the model.  EC_FP8W: the matrices (q, k, v, o, gate, up, down, LM head) are
 * 8-bit e4m3 codes (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities) with one
 * float32 scale per output row - value = scale[row] * e4m3(code) - while the embedding, the norm
 * gains, the activations fed to GEMMs and the KV cache are bfloat16 as under EC_BF16.  It halves
 * the bytes a PARTIAL step streams; the arithmetic (bf16 MFMA on the exactly widened codes, fp32
 * accumulation, scales applied to the sums) is otherwise that of EC_BF16. */
enum { EC_F32 = 0, EC_BF16 = 1, EC_FP8W = 2 };
/* EC_AUTO: follow the flag set by the previous step; the first step is always FULL. */
enum { EC_FULL = 0, EC_PARTIAL = 1, EC_AUTO = 2 };
enum {
  EC_OK = 0,
  EC_ERR_ARG = -1,       /* null pointer, bad enum value, bad size                              */
  EC_ERR_CONFIG = -2,    /* model / decode configuration outside what the kernels support       */
  EC_ERR_WORKSPACE = -3, /* workspace missing, misaligned or smaller than ec_workspace_bytes()  */
  EC_ERR_STATE = -4,     /* PARTIAL before any FULL step; step after the generation is done     */
  EC_ERR_HIP = -5,       /* a HIP runtime call failed                                           */
  EC_ERR_HOST_MEMORY = -6, /* the host ran out of memory inside the call; the context is unusable */
  EC_ERR_NONFINITE = -7  /* a block row's logits had no finite maximum (NaN weights, overflow):
                            the step ran to its end and stayed inside its buffers - such a row
                            reports token 0, confidence 0 and infinite entropy - but what it
                            computed is meaningless; ec_reset() before going on               */
};

/* Model shape.  "Bidirectional Llama-style": pre-norm blocks, RMSNorm, rotate-half RoPE on
 * absolute positions, grouped-query attention without mask, SwiGLU MLP, no biases, untied
 * embedding and LM head.  logit_scale multiplies the LM-head output (1.0 = the model as is).
 * Supported (EC_ERR_CONFIG otherwise): head_dim 64 or 128; n_heads a multiple of n_kv_heads;
 * d_model and d_ffn multiples of 8 (bfloat16: of 32, EC_FP8W: of 64, and vocab a multiple of 16);
 * vocab at most 163840; prompt + generation at most 15000 positions per sequence.
 * bfloat16 path: the sum of squares of a row of the residual stream is kept in 44.20 fixed point
 * (exact to 5e-7 per 16 features, which is all a row needs down to sums of squares of ~1e-3); it
 * saturates at about 4e12 (|h| of ~3e4 at d_model 4096) instead of overflowing - such a row's
 * RMSNorm output is then too large rather than garbage. */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, mask_id;
  float rms_eps, rope_base, logit_scale;
  int32_t dtype; /* EC_F32 | EC_BF16 | EC_FP8W */
} ec_model_cfg;

/* DEVICE pointers, BORROWED.  Per-layer entries are HOST arrays of n_layers DEVICE pointers. */
typedef struct {
  const void *tok_emb;          /* [vocab, d_model]                 */
  const void *lm_head;          /* [vocab, d_model]                 */
  const void *final_norm;       /* [d_model]                        */
  const void *const *attn_norm; /* [L] of [d_model]                 */
  const void *const *wq;        /* [L] of [n_heads*head_dim, d_model]    */
  const void *const *wk;        /* [L] of [n_kv_heads*head_dim, d_model] */
  const void *const *wv;        /* [L] of [n_kv_heads*head_dim, d_model] */
  const void *const *wo;        /* [L] of [d_model, n_heads*head_dim]    */
  const void *const *mlp_norm;  /* [L] of [d_model]                 */
  const void *const *w_gate;    /* [L] of [d_ffn, d_model]          */
  const void *const *w_up;      /* [L] of [d_ffn, d_model]          */
  const void *const *w_down;    /* [L] of [d_model, d_ffn]          */
  /* EC_FP8W only (ignored otherwise, may be NULL): float32 scales, one per output row of the
   * matrix of the same name */
  const float *lm_head_scale;         /* [vocab]                    */
  const float *const *wq_scale;       /* [L] of [n_heads*head_dim]  */
  const float *const *wk_scale;       /* [L] of [n_kv_heads*head_dim] */
  const float *const *wv_scale;
  const float *const *wo_scale;       /* [L] of [d_model]           */
  const float *const *w_gate_scale;   /* [L] of [d_ffn]             */
  const float *const *w_up_scale;
  const float *const *w_down_scale;   /* [L] of [d_model]           */
} ec_weights;

/* Decoding parameters: generation length N, block (window) size w, recent-token budget k,
 * tokens unmasked per step n, entropy threshold tau in nats (Algorithm 1 inputs).
 *  conf_threshold  0: a step unmasks the n most confident rows of the block.  > 0: confidence-
 *                  based parallel decoding (the paper's experimental setup uses 0.9): every row
 *                  whose confidence (maximum probability) exceeds it is unmasked, the n most
 *                  confident ones in any case, at most EC_MAX_N.
 *  gate_metric     what is compared with tau over the newly decoded tokens (the paper's
 *                  ablation "Choice of thresholding variable"): EC_GATE_MAX_ENTROPY (Eq. 1, the
 *                  method) and EC_GATE_ENTROPY_SUM skip the recomputation when the value is at
 *                  most tau, EC_GATE_MAX_CONFIDENCE when it is at least tau.
 *  schedule        EC_SCHED_BLOCKS: M^t = the masked positions of the current fixed block of
 *                  `block` generation slots; the next block starts when it is empty.
 *                  EC_SCHED_SLIDING: sliding-window decoding (the paper's experiments; it gives no
 *                  advance rule): M^t = the leftmost `block` still-masked generation slots. */
enum { EC_GATE_MAX_ENTROPY = 0, EC_GATE_ENTROPY_SUM = 1, EC_GATE_MAX_CONFIDENCE = 2 };
enum { EC_SCHED_BLOCKS = 0, EC_SCHED_SLIDING = 1 };
typedef struct {
  int32_t batch, gen_len, block, k_recent, tokens_per_step;
  float tau;
  float conf_threshold;
  int32_t gate_metric;
  int32_t schedule;
} ec_decode_cfg;

/* What one step did.  positions / tokens / entropy / confidence list the step's OWN decode()
 * choice (n_unmasked entries, most confident first).  max_entropy is the gate value of that
 * choice: the maximum entropy E of Eq. 1, or what gate_metric selects instead.  next_mode is
 * EC_PARTIAL iff that value passes the threshold (max entropy: E <= tau).
 * Under ec_step_forced the caller's tokens are committed instead and the context's flag follows
 * THEIR gate value: these fields still describe the step's own choice, so next_mode is then what
 * the step would have chosen, not necessarily what EC_AUTO runs next. */
typedef struct {
  int32_t n_unmasked;
  int32_t done;         /* 1 when no masked position is left after this step                   */
  int32_t mode_run;     /* EC_FULL | EC_PARTIAL: what this step executed                        */
  int32_t next_mode;    /* EC_AUTO's next mode (forced steps: what the own choice would give)   */
  int32_t n_query_rows; /* |S|: rows that recomputed Q/K/V in this step                         */
  int32_t step_index;   /* t of this step, starting at 1                                        */
  int32_t n_block_rows; /* |M^t|: masked rows of the current block = rows that got logits       */
  int32_t n_recent_next;/* |R^{t+1}|                                                            */
  float max_entropy;
  int32_t positions[EC_MAX_N];
  int32_t tokens[EC_MAX_N];
  float entropy[EC_MAX_N];
  float confidence[EC_MAX_N];
} ec_step_result;

typedef struct {
  int32_t steps, full_steps, partial_steps, tokens;
  int64_t rows_recomputed; /* sum of |S| over steps; recompute ratio = rows / (steps * T)       */
  double ms_total;         /* host wall-clock of the whole generation                           */
} ec_gen_stats;

/* Kernel classes for ec_profile_*: names follow the paper's wall-clock breakdown (attention
 * with rotary embeddings, feed-forward, KV-cache update, decision, remaining operations). */
enum {
  EC_K_EMBED = 0, EC_K_NORM, EC_K_QKV, EC_K_ROPE_KV, EC_K_ATTN, EC_K_OPROJ, EC_K_GATEUP,
  EC_K_SWIGLU, EC_K_DOWN, EC_K_LMHEAD, EC_K_VOCAB_REDUCE, EC_K_DECIDE, EC_K_COUNT
};
typedef struct {
  double ms[EC_K_COUNT];        /* accumulated device time per kernel class, from HIP events    */
  int64_t launches[EC_K_COUNT]; /* accumulated launch count per class                           */
  int64_t steps;
} ec_profile;

/* What ec_debug_read copies to the host. */
enum {
  EC_DBG_LOGITS = 0, /* float32 [n_block_rows, vocab] of the last step (already scaled); needs
                        ec_debug_keep_logits to have been on during that step                 */
  EC_DBG_KCACHE,     /* layer's keys, post-RoPE, storage type, [T, n_kv_heads, head_dim]       */
  EC_DBG_VCACHE,     /* layer's values, same layout                                            */
  EC_DBG_X,          /* int32 [T] current token ids                                            */
  EC_DBG_MASKED,     /* uint8 [T] 1 = still masked                                             */
  EC_DBG_HIST,       /* int32 [gen_len] decode step per slot, INT32_MIN = never                */
  EC_DBG_ROWS,       /* int32 [n]: row set the NEXT partial step would use (M u R), ascending  */
  EC_DBG_ROW_STATS   /* float32 [n_block_rows, 4]: token id (as float), confidence, entropy, max logit of the last step's rows */
};

/* Bytes of DEVICE workspace ec_init needs for this model, decode setup and prompt lengths
 * (every sequence's KV cache - the cached K, V of the appendix algorithm - activations, state,
 * and for bfloat16 a re-tiled copy of the matrices).  Pure host computation.
 * Returns 0 on NULL arguments or a configuration ec_init would reject. */
size_t ec_workspace_bytes(const ec_model_cfg *model, const ec_decode_cfg *decode,
                          const int32_t *prompt_lens /*HOST [batch]*/);

/* Creates a context (initialisation lines of Algorithm 1 and of the appendix algorithm):
 * validates the configuration, carves the workspace, uploads the prompts, fills the generation
 * slots with mask_id, clears the history (t = 1, flag = recompute), re-tiles bfloat16 matrices.
 * No forward pass runs here; the first step is FULL (appendix algorithm, t == 1 branch).
 *  out         receives the context (NULL on failure); destroy it with ec_destroy
 *  model, weights, decode   HOST structs, copied; the weight tensors they point to are DEVICE
 *              memory, BORROWED for the life of the context and never written
 *  prompt_ids  HOST, the batch's prompts one after the other, prompt_lens[b] ids each; any id
 *              in [0, vocab) is accepted
 *  workspace   DEVICE, 256-byte aligned, >= ec_workspace_bytes(); BORROWED
 *  hip_stream  hipStream_t to enqueue on (NULL = the default stream)
 * Errors: EC_ERR_ARG (NULL pointer, prompt id outside the vocabulary), EC_ERR_CONFIG (shape or
 * decode setting the kernels do not support; ec_last_error(NULL) names it), EC_ERR_WORKSPACE,
 * EC_ERR_HIP.  Synchronises the stream once. */
int ec_init(ec_ctx **out, const ec_model_cfg *model, const ec_weights *weights,
            const ec_decode_cfg *decode, const int32_t *prompt_ids, const int32_t *prompt_lens,
            void *workspace, size_t workspace_bytes, void *hip_stream);

/* Restarts the generation of an existing context with new prompts of the SAME lengths (state
 * as after ec_init; the cache contents become meaningless until the next FULL step).
 * Errors: EC_ERR_ARG, EC_ERR_HIP. */
int ec_reset(ec_ctx *ctx, const int32_t *prompt_ids /*HOST*/);

/* One denoising step (Algorithm 1 loop body; appendix algorithm: full branch or partial branch,
 * decode, history update, Eq. 1 - 3, flag) of every unfinished sequence.  mode = EC_AUTO follows
 * each sequence's entropy flag; EC_FULL / EC_PARTIAL override it for all of them.
 * out: HOST, batch ec_step_result, written on success only; a sequence that had finished earlier
 * reports done = 1 and zeros.
 * Errors: EC_ERR_ARG (NULL, bad mode), EC_ERR_STATE (every sequence finished; EC_PARTIAL for a
 * sequence that has not run a FULL step yet) - the state is untouched then - EC_ERR_HIP, and
 * EC_ERR_NONFINITE: some block row's logits had no finite maximum.  That step has run and the
 * state has advanced (no access left its buffers: the row took token 0), out is written, but
 * nothing computed from then on means anything; ec_reset() the context.
 * Waits once, for the results (which the decision kernel leaves in pinned host memory). */
int ec_step(ec_ctx *ctx, int mode, ec_step_result *out);

/* Teacher forcing: runs the forward pass and the vocabulary reduction in `mode`, reports the
 * step's own choice in `out`, but commits the caller's n (position, token) pairs (HOST arrays;
 * n may be 0) to x, the mask set and the history; the flag follows the committed tokens.
 * Batch 1 only.  Errors as ec_step, plus EC_ERR_ARG for a position that is not a masked
 * generation slot, a token outside the vocabulary, a repeated position, n > EC_MAX_N. */
int ec_step_forced(ec_ctx *ctx, int mode, int32_t n, const int32_t *positions,
                   const int32_t *tokens, ec_step_result *out);
/* The same for a batch: modes[b] and n[b] per sequence (entries of finished sequences are
 * ignored), the pairs of all sequences one after the other in positions / tokens. */
int ec_step_forced_batch(ec_ctx *ctx, const int32_t *modes, const int32_t *n,
                         const int32_t *positions, const int32_t *tokens, ec_step_result *out);

/* Runs EC_AUTO steps until no masked position is left in any sequence (Algorithm 1, whole
 * loop; returns the generated part of x).  out_tokens: HOST [batch, gen_len] final ids of the
 * generation slots.  stats may be NULL; its full_steps / partial_steps count sequence-steps.
 * Errors: those of ec_step; on failure out_tokens is not written. */
int ec_generate(ec_ctx *ctx, int32_t *out_tokens, ec_gen_stats *stats);

/* Per-kernel-class device timing with HIP events on the context's stream.  While enabled every
 * launch is bracketed by two events (this slows the step slightly; keep it off when timing
 * whole steps).  ec_profile_read accumulates since the last enable. */
int ec_profile_enable(ec_ctx *ctx, int on);
int ec_profile_read(ec_ctx *ctx, ec_profile *out);

/* The bfloat16 path reduces the vocabulary (Eq. 1: argmax, confidence, entropy) inside the
 * LM-head kernel and never writes the logits to memory.  on != 0 makes the following steps store
 * them as well (16 MB per step at a 126464-token vocabulary) so that EC_DBG_LOGITS can read them;
 * the step's results are bit-identical either way.  Off by default.  (Float32 models and steps with
 * more than 64 block rows over the batch materialise their logits anyway.)  Errors: EC_ERR_ARG. */
int ec_debug_keep_logits(ec_ctx *ctx, int on);

/* Copies internal state of one sequence to the host (synchronises the stream; test and
 * diagnosis aid, not part of the method).  bytes must not exceed the size of the item
 * (EC_ERR_ARG otherwise); the copy is truncated to bytes.  EC_DBG_LOGITS of a step that did not
 * store its logits is EC_ERR_STATE. */
int ec_debug_read(ec_ctx *ctx, int what, int layer, void *host_dst, size_t bytes); /* sequence 0 */
int ec_debug_read_seq(ec_ctx *ctx, int seq, int what, int layer, void *host_dst, size_t bytes);

/* The O(V) reduction behind the method's decision (Eq. 1 and the complexity discussion of the
 * Method section) as a call of its own, for logits that already sit on the device: for each row
 * of a float32 matrix, stats[row] = (argmax token id as a float, lowest id on ties; confidence =
 * maximum softmax probability; entropy -sum p ln p in nats; maximum logit).  One pass over the
 * logits; partial (max, argmax, sum e, sum e*(z-max)) tuples per 2048 columns are merged in a
 * fixed order, so the result is bit-reproducible.  A logit of -inf has probability 0.  A row
 * that holds a NaN reports NaN statistics, and a token id outside [0, vocab) if it has no
 * finite maximum at all: check before using it as an index.
 *  logits     DEVICE float32 [rows, vocab], row stride ld elements (ld >= vocab); read only
 *  rows       0 .. EC_MAX_BLOCK; vocab 2 .. 163840
 *  stats      DEVICE float32 [rows, 4], 16-byte aligned; written
 *  workspace  DEVICE, 256-byte aligned, >= ec_row_entropy_workspace_bytes(rows, vocab) (0 for
 *             arguments outside the limits); holds the partial tuples; BORROWED for the call
 * Enqueues on hip_stream (NULL = default stream) and returns without synchronising.
 * Errors: EC_ERR_ARG, EC_ERR_WORKSPACE, EC_ERR_HIP; ec_last_error(NULL) names the cause. */
size_t ec_row_entropy_workspace_bytes(int32_t rows, int32_t vocab);
int ec_row_entropy(const float *logits, int32_t rows, int32_t vocab, size_t ld, float *stats,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/* ec_row_entropy for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels
 * and results (bit for bit) as ec_row_entropy, but the partial tuples live in a 160 KiB array
 * that is part of the library's device image (one copy per GPU, held until the process ends):
 * the call allocates nothing, on the device or through any library.  Limits as ec_row_entropy
 * (rows <= EC_MAX_BLOCK, vocab <= 163840; anything beyond is EC_ERR_ARG).  The array keeps the
 * last call's contents and every entry a call reads it has written before, so nothing needs
 * clearing; all calls on one GPU share it, so two calls that overlap in time on the same GPU
 * (different streams, different threads) race - serialise them.  The first call on a device
 * looks up the array's device address (hipGetSymbolAddress); do that call outside a capture.
 * Errors: EC_ERR_ARG, EC_ERR_HIP. */
int ec_row_entropy_noalloc(const float *logits, int32_t rows, int32_t vocab, size_t ld,
                           float *stats, void *hip_stream);

/* Frees host-side state only; never frees weights or workspace.  NULL is allowed. */
void ec_destroy(ec_ctx *ctx);

const char *ec_strerror(int code);
const char *ec_last_error(const ec_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* EC_H */
