/*
 * ngg -- one batched, learning-free speculative verify step for greedy decoding
 * of a decoder-only transformer on AMD MI355X (gfx950).
 *
 * Plain C ABI.  No call throws or aborts; every call returns an ngg_status and
 * leaves a message readable through ngg_last_error().  Argument errors are
 * detected on the host before anything is launched.  A context is used from
 * one host thread at a time.  All work of a context is enqueued on the HIP
 * stream given to ngg_create; calls that fill host buffers synchronise that
 * stream before returning.
 *
 * State of a context (Section 3, "Assumptions on parallelism for
 * verification"): the context holds n tokens (prompt + generated); every token
 * except the final one has its keys and values cached (positions 0 .. n-2).
 */
#ifndef NGG_H
#define NGG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ngg_ctx ngg_ctx; /* opaque; owns KV caches, activations, token history, bigram table */

typedef enum {
  NGG_OK = 0,
  NGG_EINVAL = -1,    /* null pointer, bad shape, token id out of range, unsupported model shape */
  NGG_ECAPACITY = -2, /* sequence would exceed max_seq, or k / w exceed max_k / max_w */
  NGG_ESTATE = -3,    /* call out of order: verify before prefill, commit without a verify */
  NGG_EHIP = -4,      /* a HIP runtime call failed; the message holds hipGetErrorString */
  NGG_ENOMEM = -5     /* device or host allocation failed */
} ngg_status;

typedef enum { NGG_F32 = 0, NGG_BF16 = 1 } ngg_dtype;

/* Decoder shape.  The base model M of Section 4.1 is a pre-norm decoder with
 * RMSNorm, rotary multi-head attention (rotate-half pairing: element i pairs
 * with i + head_dim/2), SwiGLU feed-forward, no biases, a final RMSNorm and an
 * untied output embedding.  Constraints checked by ngg_create: head_dim in
 * {32, 64, 128}; d_model, d_ffn, n_heads*head_dim and vocab multiples of 32;
 * d_model <= 16384 and d_ffn <= 65536 (what the norm and sweep kernels hold
 * per workgroup); n_heads a multiple of n_kv_heads. */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t dtype;      /* ngg_dtype of weights, KV cache and GEMM inputs; accumulation is always fp32 */
  float rms_eps, rope_theta;
  int32_t max_seq;    /* capacity of the token history and of the KV cache */
  int32_t max_k;      /* largest number of draft rows k */
  int32_t max_w;      /* largest draft width w */
} ngg_model_desc;

/* DEVICE pointers, row-major [out][in], element type desc.dtype.  BORROWED:
 * the caller keeps them alive and unchanged for the life of the context.
 * (ngg_create copies every matrix into an MFMA-operand-order layout of its own,
 * which costs a second copy of the weights in HBM; tok_emb and the norm gains
 * are read in place on every step.) */
typedef struct {
  const void *attn_norm; /* [d_model] */
  const void *wq;        /* [n_heads*head_dim][d_model] */
  const void *wk;        /* [n_kv_heads*head_dim][d_model] */
  const void *wv;        /* [n_kv_heads*head_dim][d_model] */
  const void *wo;        /* [d_model][n_heads*head_dim] */
  const void *mlp_norm;  /* [d_model] */
  const void *w_gate;    /* [d_ffn][d_model] */
  const void *w_up;      /* [d_ffn][d_model] */
  const void *w_down;    /* [d_model][d_ffn] */
} ngg_layer_weights;

typedef struct {
  const void *tok_emb;    /* input embedding,  [vocab][d_model] (device) */
  const void *unemb;      /* output embedding, [vocab][d_model] (device) */
  const void *final_norm; /* [d_model] (device) */
  const ngg_layer_weights *layers; /* HOST array of n_layers entries (read during ngg_create only) */
} ngg_weights;

/* Draft batch shape (glossary of the paper): k rows, w speculated tokens per
 * row; context N-gram queries use the last q tokens, q tried from q_max down
 * to q_min (q_min == q_max is the matcher of Section 4.2); at most k_ctx_max
 * rows come from the context (k_ctx_max == k is the rule of Section 4.3). */
typedef struct {
  int32_t k, w, k_ctx_max, q_min, q_max;
} ngg_draft_cfg;

/* Result of one verify call.  All pointers are HOST buffers owned by the
 * caller; any of them may be NULL to skip that output. */
typedef struct {
  int32_t k, w;        /* filled by the call */
  int32_t winner;      /* row with the longest accepted prefix (lowest row on ties) */
  int32_t n_accept;    /* accepted drafted tokens of the winner, 0 .. w */
  int32_t n_new;       /* n_accept + 1: tokens a commit would append (before budget truncation) */
  int32_t *greedy;     /* [k][w+1] greedy token after every block position */
  int32_t *accept_len; /* [k] */
  int32_t *new_tokens; /* [w+1], first n_new valid */
  float *logits;       /* [k][w+1][vocab] fp32, or NULL (costs a k*(w+1)*vocab*4-byte device->host copy) */
} ngg_verify_out;

typedef struct {
  int64_t calls;          /* verify calls */
  int64_t tokens;         /* generated tokens (including the one produced by prefill) */
  int64_t new_hist[34];   /* new_hist[i] = calls that appended i tokens (i <= max_w+1 <= 33) */
  int64_t winner_src[2];  /* calls won by a context row / by a bigram row */
  int64_t ctx_rows;       /* context rows found, summed over calls */
  double ms_prefill, ms_drafts, ms_verify, ms_commit; /* host wall time per phase; the drafts are not waited for,
                                                         so ms_verify (which ends with the step's one
                                                         synchronisation) holds their device time too */
  /* the quantities of the paper's ablation on strategies (Section 5.2), index 0 = context rows, 1 = bigram rows */
  int64_t accept_hist[2][34];  /* [s][a]: calls whose winning row came from strategy s and had a drafted tokens accepted */
  int64_t rank_hist[2][32];    /* [s][r]: calls with an accepted draft whose winning row was the r-th row of strategy s */
  int64_t alloc_hist[33];      /* [c]: calls whose batch held c context rows (and k - c bigram rows) */
} ngg_stats;

/* Creates a context: allocates caches and activations on the current device,
 * builds the rotary table and the bigram's top-1 table next1[x] = argmax_v
 * <unemb[v], tok_emb[x]> (the O(1) lookup of Section 4.1, "Extensions").
 * hip_stream is a hipStream_t (NULL = the default stream), borrowed. */
ngg_status ngg_create(const ngg_model_desc *desc, const ngg_weights *weights, void *hip_stream, ngg_ctx **out);
ngg_status ngg_destroy(ngg_ctx *ctx);

/* Resets the context to `prompt` (HOST, n_prompt >= 1 tokens), caches keys and
 * values of every prompt token and appends the model's first greedy token:
 * afterwards n = n_prompt + 1.  Runs the verify kernels on chunks of the
 * prompt; it is plumbing, not part of the timed step. */
ngg_status ngg_prefill(ngg_ctx *ctx, const int32_t *prompt, int32_t n_prompt);

/* Draft construction (Section 4): context N-gram rows first (Section 4.2:
 * earlier occurrences of the last q tokens, the w tokens that follow, ranked by
 * count, ties to the later match), then rows of the model bigram (Section 4.1:
 * top-k of <unemb[v], tok_emb[x_last]>, ties to the lower id, each extended to
 * w tokens by chaining next1).  The drafts stay on the device for
 * ngg_verify_step(drafts = NULL); the host copies are optional:
 * drafts [k][w], row_src [k] (0 = context, 1 = bigram), n_ctx_rows. */
ngg_status ngg_build_drafts(ngg_ctx *ctx, const ngg_draft_cfg *cfg, int32_t *drafts, int8_t *row_src,
                            int32_t *n_ctx_rows);

/* One model call on the block of shape (k, w+1) of Section 3: row r =
 * [x_last, drafts[r][0..w)] at positions n-1 .. n-1+w, all rows sharing the
 * cached context (read once).  Then the per-position greedy argmax (lowest id
 * on ties), the accepted length of every row and the winner.  drafts: HOST
 * [k][w], or NULL to use what ngg_build_drafts left on the device (same k, w).
 * Does not change the committed state.  NGG_ECAPACITY if n + w > max_seq. */
ngg_status ngg_verify_step(ngg_ctx *ctx, const int32_t *drafts, int32_t k, int32_t w, ngg_verify_out *out);

/* Commits the last verify call (Appendix D: the cache becomes that of the
 * longest accepted speculation): appends min(n_new, max_new) tokens and the
 * winner row's keys/values for the block columns they came from.  max_new <= 0
 * is NGG_EINVAL; NGG_ESTATE without a preceding verify.  The count is also cut
 * to the room left in the context (a fully accepted block at n + w == max_seq
 * appends w tokens, not w + 1); NGG_ECAPACITY only when n == max_seq already.
 * n_committed may be NULL. */
ngg_status ngg_commit(ngg_ctx *ctx, int32_t max_new, int32_t *n_committed);

/* Prefill + repeated (build_drafts, verify_step, commit) until n_gen tokens
 * were generated (the first comes from the prefill).  cfg == NULL, or k = 1 and
 * w = 0, is plain greedy decoding, one token per model call.  out_tokens: HOST
 * [n_gen]; stats may be NULL. */
ngg_status ngg_greedy_decode(ngg_ctx *ctx, const int32_t *prompt, int32_t n_prompt, int32_t n_gen,
                             const ngg_draft_cfg *cfg, int32_t *out_tokens, ngg_stats *stats);

/* Continues from the committed state: (build_drafts, verify_step, commit) until
 * n_gen more tokens were appended or max_calls verify calls were made, whichever
 * comes first, without returning to the caller in between (a serving loop with
 * no per-call host overhead).  cfg as in ngg_greedy_decode.  out_tokens: HOST
 * [n_gen] or NULL; *n_out = tokens appended; stats cover these calls only
 * (stats->tokens = tokens appended).  NGG_ESTATE before ngg_prefill. */
ngg_status ngg_decode_more(ngg_ctx *ctx, int32_t n_gen, int32_t max_calls, const ngg_draft_cfg *cfg,
                           int32_t *out_tokens, int32_t *n_out, ngg_stats *stats);

/* The paper's own model bigram as a precomputed table (Section 4.1, "Model
 * bigram"; Appendix A builds the same lookup): p_M(. | x) is the next-token
 * distribution of the WHOLE model on the one-token context x.  For every
 * vocabulary entry x the library runs the decoder on [x] (Mcap contexts per
 * pass, each attending to itself only, position 0) and keeps the top_k token
 * ids by (logit desc, id asc) in a device table [vocab][top_k]; column 0 is
 * the lookup the chained extension to w > 1 tokens uses (Section 4.1,
 * "Extensions").  Costs vocab / Mcap model calls, once.  Requires
 * max_k <= top_k <= min(64, vocab).  Leaves the committed state as it was; a
 * pending verify call can no longer be committed (NGG_ESTATE from ngg_commit). */
ngg_status ngg_bigram_table_build(ngg_ctx *ctx, int32_t top_k);

/* The model unigram (Section 4.1, "Unigram"): p(x) ~ exp(-d(x)) with d(x) the
 * distance of x's output embedding from the mean output embedding in the norm
 * induced by the input embeddings, d(x)^2 = sum over tokens y of
 * ((unemb[x] - mean) . tok_emb[y])^2.  Computes d for the whole vocabulary on
 * the device (vocab / Mcap GEMM passes, once) and keeps the top_k nearest
 * tokens (ties to the lower id).  Requires max_k <= top_k <= min(64, vocab). */
ngg_status ngg_unigram_build(ngg_ctx *ctx, int32_t top_k);

/* Where the model rows of ngg_build_drafts come from: NGG_BIGRAM_DIRECT (the
 * default: one sweep of <unemb[v], tok_emb[x_last]> per step, chained through
 * next1), NGG_BIGRAM_TABLE (two lookups in the full-model table; NGG_ESTATE if
 * it was not built) or NGG_UNIGRAM (q = 0: row i starts with the i-th nearest
 * unigram token whatever the context, then chains through next1; NGG_ESTATE if
 * it was not built).  The choice changes the drafts, never the committed tokens. */
enum { NGG_BIGRAM_DIRECT = 0, NGG_BIGRAM_TABLE = 1, NGG_UNIGRAM = 2 };
ngg_status ngg_bigram_source(ngg_ctx *ctx, int32_t source);

/* Row allocation between the two strategies inside ngg_greedy_decode / ngg_decode_more (Section 5.2 closes on
 * the remark that the context strategy is often handed the whole batch although its wins come from its first
 * rows, and that a better allocation could gain more).  NGG_ALLOC_FIXED (default): every call may take up to
 * cfg.k_ctx_max context rows, the rule of Section 4.3.  NGG_ALLOC_ADAPTIVE: once warmup_wins calls since the
 * last prefill were won by a context row with at least one accepted token, a call may take at most c context
 * rows, c being the smallest count of leading context rows that held coverage_percent of those wins (never
 * more than cfg.k_ctx_max, never fewer than 1); the bigram fills the rest.  The choice changes the drafts,
 * never the committed tokens.  ngg_build_drafts called directly is not affected. */
enum { NGG_ALLOC_FIXED = 0, NGG_ALLOC_ADAPTIVE = 1 };
ngg_status ngg_allocation(ngg_ctx *ctx, int32_t mode, int32_t coverage_percent, int32_t warmup_wins);

/* Replay of captured steps inside ngg_greedy_decode / ngg_decode_more (the method's loop of Section 3: drafts, one
 * model call on the (k, w+1) block, acceptance, commit).  A step whose launch shapes equal the previous step's can be
 * replayed from a HIP graph (recorded on a stream of the library's own, launched on the context's stream); its
 * kernels read the context length from device memory, which the graph's last node advances, so the same graph serves
 * step after step and is captured again only when k, w, the draft settings or the number of attention slices change.
 * Steps that the generation budget clamps (the last ones), steps with profiling brackets enabled and the first step
 * of every shape are always launched on the stream.  mode 0: never replay.  mode 1: replay every step that qualifies.
 * mode 2 (default): per step shape, time three steps launched on the stream and, unless those took more than 6 us
 * per kernel launch (a step bound by the device: replay cannot win and the capture is not paid), three replayed; keep the
 * faster way (replay pays where a step is bound by its launches: small models; at the 7B shapes it measured no
 * gain).  In every
 * mode the same kernels run in the same shapes: the committed tokens and the statistics are identical.
 * ngg_build_drafts, ngg_verify_step and ngg_commit called directly always launch on the stream. */
ngg_status ngg_step_graphs(ngg_ctx *ctx, int32_t mode);

/* Committed token history: copies min(n, cap) tokens to dst (HOST), n to *n. */
ngg_status ngg_get_tokens(const ngg_ctx *ctx, int32_t *dst, int32_t cap, int32_t *n);

/* Message of the last failing call on this context (ctx == NULL: of the last
 * failing ngg_create on this thread).  Never NULL. */
const char *ngg_last_error(const ngg_ctx *ctx);

/* Per-kernel-class device time, taken with HIP events recorded on the context's
 * stream around every launch of the classes whose bit is set in class_mask
 * (bit i = class i, -1 = all, 0 = off).  Events between launches cost a little
 * time: enable few classes while timing whole steps.  ngg_profile_read sums the
 * milliseconds and launch counts per class since the last ngg_profile_reset. */
enum {
  NGG_PROF_GEMM_QKV = 0, NGG_PROF_GEMM_O, NGG_PROF_GEMM_GATEUP, NGG_PROF_GEMM_DOWN, NGG_PROF_GEMM_UNEMBED,
  NGG_PROF_ATTENTION, NGG_PROF_NORM, NGG_PROF_DRAFTS, NGG_PROF_ACCEPT_COMMIT, NGG_PROF_OTHER, NGG_PROF_COUNT
};
ngg_status ngg_profile_enable(ngg_ctx *ctx, int32_t class_mask);
ngg_status ngg_profile_reset(ngg_ctx *ctx);
/* Brackets only one launch in every `every` of each enabled class (default 1 = all): a bracket costs
 * about 5 us of stream time, so a whole step is timed with a sparse sample (an `every` coprime to the
 * launches of the class per step walks through the layers). */
ngg_status ngg_profile_sample(ngg_ctx *ctx, int32_t every);
ngg_status ngg_profile_read(ngg_ctx *ctx, double *ms /*[NGG_PROF_COUNT]*/, int64_t *launches /*[NGG_PROF_COUNT]*/);
/* What a bracket of two events reads around an EMPTY kernel on the context's
 * stream, in microseconds (mean of 64 brackets queued back to back): the part of every ngg_profile_read time
 * that is the dispatch of the launch and the events themselves, not the kernel. */
ngg_status ngg_profile_bracket_overhead(ngg_ctx *ctx, double *us);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the context N-gram rows of ngg_build_drafts without a context
 * object and without any allocation.  tokens: DEVICE [n], the whole context, its last q tokens being
 * the query; rows: DEVICE [k_ctx_max][w], the continuations found, in rank order (count descending,
 * ties to the later match; query lengths q_max down to q_min, a continuation already taken is skipped);
 * *n_rows: DEVICE, how many rows were found (rows beyond it are left untouched).  The matcher's working
 * memory (match list, group table: 1.125 MiB) is a static device array inside the library, so
 * n <= NGG_STATIC_MAX_TOKENS (NGG_ECAPACITY beyond); 1 <= w, k_ctx_max <= 32; 1 <= q_min <= q_max <= 64.
 * The launch is queued on hip_stream (a hipStream_t, NULL = the default stream) and the call returns
 * without synchronising; it calls no hipMalloc / hipFree / memset.  All calls on one GPU share the
 * one array: calls that overlap in time on a GPU (different streams or threads) race; calls queued
 * on one stream do not.  Errors are reported through ngg_last_error(NULL). */
#define NGG_STATIC_MAX_TOKENS 32768
ngg_status ngg_context_drafts_static(const int32_t *tokens, int32_t n, int32_t w, int32_t k_ctx_max, int32_t q_min,
                                     int32_t q_max, int32_t *rows, int32_t *n_rows, void *hip_stream);

/* What a plain streaming read reaches on this GPU, in GB/s: every CU reads its share of the library's copy of
 * the weights once with 16-byte loads (2048 workgroups, best of 4 sweeps, timed with events on the context's
 * stream).  Context for the roofline fractions, which are quoted against the published 8 TB/s. */
ngg_status ngg_profile_read_bandwidth(ngg_ctx *ctx, double *gbps);

/* Debug aid for parity tests: copies an internal device buffer to dst (HOST), at most cap bytes,
 * and reports its full size in *bytes.  Names: "h" (residual stream, fp32 [M][d_model]), "z"
 * (bigram scores of the last ngg_build_drafts, fp32 [vocab]), "next1" (int32 [vocab]), "hist"
 * (int32 token history), "block_tok" (int32 block tokens of the last forward), "kcache" /
 * "vcache" (whole caches, [layer][kv head][*stride / 32 tiles]: a tile holds 32 positions x head_dim
 * elements in MFMA operand order, i.e. blocks of 16 rows x 32 contraction elements of 512 elements
 * each; a key tile is the [32 positions][head_dim] matrix with position 8a + 4f + b stored as row
 * 16f + 4a + b, a value tile the transposed [head_dim][32 positions] matrix; element (row n, column
 * k) of a tile matrix with K columns sits at ((n/16)*(K/32) + k/32)*512 + (((k%32)/8)*16 + n%16)*8
 * + k%8 for 2-byte elements), "attn" (attention output of the last layer, model dtype, in
 * chunks of 256 (bf16) or 128 (fp32) features: [feature chunk][Mcap rows][chunk]).
 * "attn_layout" (int32[4], host-side record of the last model call: slices of the key list per head,
 * workgroups of the attention kernel, block rows, cached positions).  "step_graphs" (int32[4], host-side record:
 * replay mode, a capture failed, captures so far, replayed steps so far).  Synchronises the stream. */
ngg_status ngg_debug_peek(ngg_ctx *ctx, const char *name, void *dst, int64_t cap, int64_t *bytes, int32_t *stride);

#ifdef __cplusplus
}
#endif
#endif /* NGG_H */
