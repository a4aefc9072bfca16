/*
 * dart.h -- C ABI of the MI355X (gfx950) implementation of DART's drafting step.
 *
 * The drafting step (paper Sec. 3.2, Sec. 4, Alg. 1, App. C/D) is
 *   1. one forward pass of the single-layer draft model over
 *      [z_1..z_n, MASK x (K-1)] -> K rows of vocabulary logits
 *      (row 0 from the last prefix position, rows 1..K-1 from the mask positions);
 *   2. per-position top-k of each row with s_logit = log(softmax(l) + eps);
 *   3. continuity-aware tree pruning: K levels of beam expansion scored by
 *      Combine(s_logit, s_ng), every expansion kept in the global tree, the
 *      theta best nodes returned as a token tree for tree-attention verification.
 *
 * Conventions
 *   - All matrices are row-major [out_features][in_features]; vectors are dense.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers
 *     are ordinary host memory.  The library never frees caller memory.
 *   - The three hot calls (dart_draft_forward*, dart_topk, dart_tree_prune) only
 *     enqueue kernels on the given HIP stream (hipStream_t passed as void*, NULL =
 *     default stream).  They do not synchronise and do not allocate: every
 *     workspace is sized at dart_create / dart_ngram_create.
 *   - Every call returns a status; nothing aborts or throws across the ABI.  On
 *     DART_ERR_ARG / DART_ERR_SHAPE / DART_ERR_STATE nothing has been launched and
 *     the outputs are untouched.
 *   - A dart_ctx must not be used from two streams at once (calls share its
 *     workspaces and K/V buffers).
 *   - Numeric range (bf16 contexts).  Weights are used as the exact bf16 values by the
 *     single-sequence calls.  Intermediates that the library stores in 16 bits are fp16:
 *     the rotated queries, the draft K/V buffers and the soft-max probabilities, and, in the
 *     batched calls, every projection input and an fp16 copy of every weight matrix.  fp16
 *     stores saturate at +-65504 instead of overflowing, and weights below 2^-14 in magnitude
 *     become fp16 subnormals in that copy (absolute error <= 2^-25).  Results are within the
 *     stated logit tolerance while |k|, |v|, |q| (after the optional q/k norm and the rotation),
 *     the normed rows, the attention output and the SwiGLU products stay below 65504; with
 *     qk_norm = 0 this bounds |Wk RMSNorm(z)| and |Wv RMSNorm(z)|, i.e. the weights' scale, not
 *     the scale of the hidden states (every projection input is RMS-normalised).  Values beyond
 *     the range saturate silently: finite, but wrong.
 */
#ifndef DART_H
#define DART_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dart_ctx dart_ctx;       /* device weights, draft K/V buffers, workspaces */
typedef struct dart_ngram dart_ngram;   /* device-resident N-gram successor table */

typedef enum {
  DART_OK = 0,
  DART_ERR_ARG = 1,    /* NULL pointer or value out of its documented range */
  DART_ERR_SHAPE = 2,  /* sizes inconsistent with the context's configuration */
  DART_ERR_OOM = 3,    /* host or device allocation failed (create calls only) */
  DART_ERR_HIP = 4,    /* a HIP runtime call failed */
  DART_ERR_STATE = 5   /* call sequence invalid (e.g. n_cached beyond what is cached) */
} dart_status;

enum { DART_F32 = 0, DART_BF16 = 1 };

/* Hard limits of this build (kernels keep per-level state in LDS / registers). */
enum {
  DART_MAX_K = 16,          /* draft length (logit rows per sequence) */
  DART_MAX_TOPK = 64,       /* candidates per position */
  DART_MAX_BEAM = 64,       /* beam width w */
  DART_MAX_BUDGET = 128,    /* tree nodes including the root */
  DART_MAX_LEVEL_NODES = 4096, /* beam_w * k, the expansions of one level */
  DART_TOPK_STATIC_CELLS = 4864 /* dart_topk_static: rows * ceil(vocab / 4096) at most (128 rows of a
                                   151936-token vocabulary) */
};

/* Shapes of the draft layer: one pre-norm decoder layer "aligned with the target
 * model" (App. B): RMSNorm, grouped-query attention with rotary positions
 * (half-split pairing), optional per-head RMSNorm of q and k, SwiGLU, final
 * RMSNorm, LM head.  dtype is the storage type of weights, hidden states and the
 * K/V buffers; accumulation is always fp32 and logits are fp32. */
typedef struct {
  int32_t d, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  int32_t max_ctx;     /* longest prefix n */
  int32_t max_K;       /* <= DART_MAX_K; mask_emb has max_K-1 rows */
  int32_t max_batch;   /* number of independent sequences (K/V buffer slots); > 1 also keeps an
                          fp16 copy of the bf16 matrices for the batched calls */
  int32_t dtype;       /* DART_F32 | DART_BF16 */
  int32_t qk_norm;     /* 0/1 */
  float rms_eps;
  float rope_base;
  /* Front end (Sec. 3.2 "Draft model architecture", App. B): 0 = the calls take the fused
   * prefix representation z [n][d]; 1 = the context also holds the FC layer and the target's
   * embedding table, dart_draft_forward_features takes the target's raw outputs, and the layer's
   * attention input is the 2d-wide z = [g ; e] (see dart_draft_forward_features). */
  int32_t front_end;
  int32_t feat_dim;    /* front_end: width of the concatenated target hidden states (3 d) */
} dart_config;

/* HOST pointers, element type per dart_config.dtype (bf16 = raw 16-bit patterns).
 * wq [Hq*hd][d], wk/wv [Hkv*hd][d], wo [d][Hq*hd], w_gate/w_up [ffn][d],
 * w_down [d][ffn], w_lm [vocab][d], norm gains [d] (q_norm/k_norm [hd], may be
 * NULL when qk_norm == 0), mask_emb [max_K-1][d] (the trainable <MASK>
 * representation, App. B; may be NULL when max_K == 1).
 * dart_create copies (and re-tiles) everything; the caller keeps its arrays.
 * With front_end = 1: wq/wk/wv are [..][2d] (columns 0..d-1 act on the g half, d..2d-1 on
 * the embedding half), mask_emb is [max_K-1][2d], and three more tensors are read: w_fc
 * [d][feat_dim] (the FC layer, no bias), embed [vocab][d] (the target's frozen embedding
 * table), w_emb_norm [d] (RMSNorm gain of the embedding half; w_in_norm is the g half's). */
typedef struct {
  const void *w_in_norm, *wq, *wk, *wv, *q_norm, *k_norm, *wo, *w_post_norm;
  const void *w_gate, *w_up, *w_down, *w_final_norm, *w_lm, *mask_emb;
  const void *w_fc, *embed, *w_emb_norm;
} dart_weights;

/* Pruning hyper-parameters (App. D): k candidates per level, beam width w,
 * budget = theta + 1 nodes (the root, i.e. the already sampled token t_{n+1}, is
 * node 0), w_ng (0.5), logit_decay (0.9, w_logit = decay^level) and level_pow (0.7,
 * w_level = (level+1)^-pow), level 0-based. */
typedef struct {
  int32_t k, beam_w, budget;
  float w_ng, logit_decay, level_pow;
} dart_prune_params;

const char *dart_status_str(dart_status s);

/* Build a context on the current HIP device.  Errors: ARG (NULL, non-positive
 * sizes, max_K > DART_MAX_K, head_dim not 64 or 128, n_q_heads not a multiple of
 * n_kv_heads, bf16 with d, Hq*hd or ffn not a multiple of 32; fp32 with d not a
 * multiple of 8 or ffn not a multiple of 4; d > 16384; max_ctx + max_K > 32768; more than 8 query heads per K/V head), OOM, HIP. */
dart_status dart_create(const dart_config *cfg, const dart_weights *w, dart_ctx **out);
void dart_destroy(dart_ctx *ctx);

/* Forget the cached draft K/V rows of sequence slot `seq`. */
dart_status dart_reset(dart_ctx *ctx, int seq);

/* Draft forward for one sequence (Sec. 3.2).
 *   hidden      device [ctx_len][d], prefix representation z_1..z_n in cfg.dtype;
 *               only rows [n_cached, ctx_len) are read.
 *   n_cached    number of leading prefix rows whose draft K/V are already in slot
 *               `seq` from earlier calls with the same rows (0 = stateless call).
 *               The draft is a single layer, so K/V of a row depend on that row
 *               alone and results do not depend on n_cached.
 *   K           1..max_K logit rows.
 *   logits_out  device [K][vocab] fp32.
 * Row j of logits_out is the draft distribution of the (j+1)-th future token:
 * row 0 is read at the last prefix position, rows 1..K-1 at the mask positions.
 * Errors: ARG (NULL, K, seq out of range, ctx_len < 1), SHAPE (ctx_len > max_ctx),
 * STATE (n_cached > ctx_len-1 or > rows cached in the slot), HIP. */
dart_status dart_draft_forward(dart_ctx *ctx, int seq, const void *hidden, int ctx_len,
                               int n_cached, int K, float *logits_out, void *stream);

/* dart_draft_forward followed by dart_topk on its K rows, as one call: on bf16 contexts with
 * K <= 8 the LM-head workgroups select the k best logits and the (max, sum exp) of the vocabulary
 * strips they compute while those are still on chip, and only the short row merge runs afterwards
 * -- the candidate extraction of Alg. 1 ("Top-k_i tokens from l_i", App. D "s_logit") without a
 * second pass over the K x vocab logits.  Other contexts run the two steps one after the other.
 *   logits_out  device [K][vocab] fp32, or NULL when the caller only needs the candidates
 *   ids_out     device [K][k] int32, scores_out device [K][k] fp32: exactly what
 *               dart_topk(logits, K, vocab, k, eps) returns for the logits this call computes
 *               (ids and order identical; scores to the rounding of the row's log-sum-exp)
 * Errors: as dart_draft_forward and dart_topk (ARG also for NULL ids_out / scores_out). */
dart_status dart_draft_forward_topk(dart_ctx *ctx, int seq, const void *hidden, int ctx_len,
                                    int n_cached, int K, int k, float eps, float *logits_out,
                                    int32_t *ids_out, float *scores_out, void *stream);

/* dart_draft_forward_batched followed by dart_topk on its batch*K rows (Sec. 3.2, then Alg. 1
 * "Top-k_i tokens from l_i", App. D "s_logit"), as one call that needs no logits buffer from the
 * caller: without one, the logits of each group of up to 16 sequences pass through a buffer of
 * the context.  The two steps run one after the other (the multi-row LM head does not select
 * candidates itself: measured no faster than the separate top-k).
 *   hidden, ctx_len, n_cached, K   as dart_draft_forward_batched
 *   logits_out  device [batch][K][vocab] fp32, or NULL when only the candidates are needed
 *   ids_out     device [batch][K][k] int32, scores_out device [batch][K][k] fp32: exactly what
 *               dart_topk returns for the logits this call computes (ids and order identical)
 * Errors: as dart_draft_forward_batched and dart_topk; STATE on contexts with the front end. */
dart_status dart_draft_forward_topk_batched(dart_ctx *ctx, int batch, const void *const *hidden,
                                            const int32_t *ctx_len, const int32_t *n_cached, int K,
                                            int k, float eps, float *logits_out, int32_t *ids_out,
                                            float *scores_out, void *stream);

/* Draft forward from the target model's raw outputs (contexts created with front_end = 1;
 * Sec. 3.2, Fig. 3): for every new prefix position, g = FC(features) and e = embedding of the
 * token that follows it (the shifted embeddings e_{2:n+1}); z = [g ; e] is the layer's 2d-wide
 * attention input, each half under its own RMSNorm, and g is the layer's residual stream.
 *   features     device [ctx_len][feat_dim] in cfg.dtype: the three target hidden states of
 *                each position, concatenated; only rows [n_cached, ctx_len) are read
 *   next_tokens  device [ctx_len] int32: token following each position (the last entry is the
 *                freshly sampled t_{n+1}); only entries [n_cached, ctx_len) are read; values
 *                must lie in [0, vocab)
 * Everything else as dart_draft_forward.  Errors: additionally STATE when the context has no
 * front end (and dart_draft_forward* return STATE on a context that has one). */
dart_status dart_draft_forward_features(dart_ctx *ctx, int seq, const void *features,
                                        const int32_t *next_tokens, int ctx_len, int n_cached,
                                        int K, float *logits_out, void *stream);

/* dart_draft_forward_features followed by dart_topk on its K rows, as one call: what
 * dart_draft_forward_topk is to dart_draft_forward (same selection inside the LM head on bf16
 * contexts with K <= 8, same outputs; Sec. 3.2 + Alg. 1 "Top-k_i tokens from l_i").
 * Errors: as dart_draft_forward_features and dart_topk (ARG also for NULL ids_out / scores_out). */
dart_status dart_draft_forward_features_topk(dart_ctx *ctx, int seq, const void *features,
                                             const int32_t *next_tokens, int ctx_len, int n_cached,
                                             int K, int k, float eps, float *logits_out,
                                             int32_t *ids_out, float *scores_out, void *stream);

/* Same for `batch` sequences in slots 0..batch-1 (ragged lengths).
 *   hidden      HOST array of `batch` device pointers, each [ctx_len[b]][d]
 *   ctx_len, n_cached   HOST arrays [batch]
 *   logits_out  device [batch][K][vocab] fp32
 * All rows of all sequences share every launch.  On bf16 weights the projections of this call
 * multiply an fp16 copy of the weights (made by dart_create when max_batch > 1) by fp16
 * activations, where the single-sequence call feeds two-term bf16 activations: the two calls
 * agree to rounding (both within the logit tolerance of the fp64 definition), not bit for
 * bit, and a K/V slot filled by one is reused by the other to rounding only.  Each call
 * reproduces its own cold result in a warm call bit for bit. */
dart_status dart_draft_forward_batched(dart_ctx *ctx, int batch, const void *const *hidden,
                                       const int32_t *ctx_len, const int32_t *n_cached, int K,
                                       float *logits_out, void *stream);

/* dart_draft_forward_features for `batch` sequences in slots 0..batch-1 (ragged lengths;
 * contexts created with front_end = 1; Sec. 3.2, Fig. 3).
 *   features     HOST array of `batch` device pointers, each [ctx_len[b]][feat_dim]
 *   next_tokens  HOST array of `batch` device pointers, each [ctx_len[b]] int32
 *   ctx_len, n_cached   HOST arrays [batch]
 *   logits_out   device [batch][K][vocab] fp32
 * Errors as dart_draft_forward_batched; STATE on a context without the front end. */
dart_status dart_draft_forward_features_batched(dart_ctx *ctx, int batch,
                                                const void *const *features,
                                                const int32_t *const *next_tokens,
                                                const int32_t *ctx_len, const int32_t *n_cached,
                                                int K, float *logits_out, void *stream);

/* Per-row top-k with log-softmax scores (Alg. 1, App. D "s_logit").
 *   logits      device [rows][vocab] fp32 (finite values), rows <= max_batch*max_K
 *   ids_out     device [rows][k] int32, by (logit descending, token id ascending)
 *   scores_out  device [rows][k] fp32 = min(0, log(softmax(l)_t + eps))
 * Errors: ARG (NULL, k < 1, k > min(vocab, DART_MAX_TOPK), rows < 1),
 * SHAPE (vocab > cfg.vocab, rows too large), HIP. */
dart_status dart_topk(dart_ctx *ctx, const float *logits, int rows, int vocab, int k, float eps,
                      int32_t *ids_out, float *scores_out, void *stream);

/* dart_topk without a context and without any allocation, for callers that cannot allocate
 * device memory (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): same arguments, kernels and results as dart_topk, but the workspace of the chunk
 * kernel is a fixed array inside the library image (2.5 MiB per GPU, resident until the process
 * ends) instead of a buffer owned by a dart_ctx.  The call enqueues two kernels on `stream` and
 * calls no allocating routine; the array's device address is looked up once per device, on the
 * first call made with that device current.
 *   rows * ceil(vocab / 4096) <= DART_TOPK_STATIC_CELLS, else SHAPE (nothing launched).
 * All calls on one GPU share the array: calls that overlap on one GPU (different streams or
 * threads) race; calls on one stream, or otherwise ordered, are safe.  Nothing needs clearing
 * between calls (every cell read is written first by the same call).
 * Errors: ARG (NULL, k < 1, k > min(vocab, DART_MAX_TOPK), rows < 1), SHAPE, HIP. */
dart_status dart_topk_static(const float *logits, int rows, int vocab, int k, float eps,
                             int32_t *ids_out, float *scores_out, void *stream);

/* Build the device N-gram table from raw counts (App. C): context = previous
 * n_gram-1 tokens -> up to succ_per_key successors.  HOST inputs:
 *   keys        [n_keys][n_gram-1] int32, oldest token first, rows distinct
 *   succ_ids    [n_keys][succ_per_key] int32, >= 0 and distinct within a row wherever the
 *               count is positive (ids of unused slots are ignored)
 *   succ_counts [n_keys][succ_per_key] int32 >= 0, 0 marks an unused slot
 * Stored score of a successor: min(0, log(count / sum(row counts) + eps)) rounded
 * to fp32; an absent context or successor scores log(eps).  No back-off unless
 * dart_ngram_set_backoff attaches a lower-order table.
 * Errors: ARG (NULL, n_gram not 2 or 3, succ_per_key not in 1..64, a negative context token,
 * a duplicate context, a negative count, a used successor with a negative id or repeated
 * within its row, n_keys > 2^30), OOM, HIP. */
dart_status dart_ngram_create(int n_gram, int64_t n_keys, int succ_per_key, const int32_t *keys,
                              const int32_t *succ_ids, const int32_t *succ_counts, float eps,
                              dart_ngram **out);
void dart_ngram_destroy(dart_ngram *t);

/* Optional one-level back-off (the paper's N-gram store is a trie, App. C.2, and is silent on
 * contexts it has not seen; without this call they score log(eps)).  Attaches to a trigram
 * table a bigram table of the same succ_per_key, built from HOST arrays laid out as for
 * dart_ngram_create (keys [n_keys][1]): when dart_tree_prune finds no row for a context
 * (t_-2, t_-1) it looks up (t_-1) here, and a successor found scores
 * min(0, log(alpha * count / sum(row counts) + eps)), eps being the table's.  A stored context
 * never backs off (its unseen successors keep log(eps)).  0 < alpha <= 1 is the discount of
 * the shorter context.  A table attached earlier is replaced and freed; the call must not
 * overlap with a dart_tree_prune that uses `table`.
 * Errors: ARG (NULL table, table not a trigram table, alpha out of range, bad rows as in
 * dart_ngram_create), OOM, HIP. */
dart_status dart_ngram_set_backoff(dart_ngram *table, int64_t n_keys, const int32_t *keys,
                                   const int32_t *succ_ids, const int32_t *succ_counts, float alpha);

/* Continuity-aware tree pruning (Alg. 1, App. D) for `batch` independent
 * sequences, one workgroup each.
 *   ids, scores  device [batch][K][k]: candidates per level, best first
 *                (dart_topk output with the same k); ids distinct within a level and
 *                scores <= 0 (log-probabilities), neither is checked on the device
 *   ctx_tail     device [batch][n_gram-1] int32: last real tokens, the root
 *                t_{n+1} last
 *   tokens_out   device [batch][budget] int32; node 0 = root, then level-major,
 *                within a level by (score desc, creation order); -1 beyond n_nodes
 *   parents_out  device [batch][budget] int32 index of the parent node (-1: root
 *                and unused slots); parents precede children.  With scores <= 0 and the
 *                parameter ranges below, increments are <= 0 and the theta best nodes are
 *                closed under "parent of"; a caller that passes positive scores may find
 *                -2 here for a kept node whose parent was not kept
 *   mask_out     device [batch][budget][budget] uint8, mask[i][j] = 1 iff j == i
 *                or j is an ancestor of i (tree-attention mask); 0 elsewhere
 *   n_nodes_out  device [batch] int32 = 1 + min(budget-1, total expansions)
 * Scoring arithmetic is fp32 with one rounding per operation in the order
 * ((w_logit*s_logit) + (w_ng*s_ng)) * w_level, then parent + increment, so trees
 * are reproducible bit for bit.  Ties: beam cut by (score desc, creation asc),
 * global cut by (score desc, level asc, creation asc).
 * Errors: ARG (NULL, K not in 1..DART_MAX_K, k, beam_w, budget out of range,
 * beam_w*k > DART_MAX_LEVEL_NODES, batch < 1, w_ng < 0, logit_decay <= 0, or a non-finite
 * w_ng, logit_decay or level_pow), HIP. */
dart_status dart_tree_prune(int batch, const int32_t *ids, const float *scores, int K,
                            const int32_t *ctx_tail, const dart_ngram *table,
                            const dart_prune_params *params, int32_t *tokens_out,
                            int32_t *parents_out, uint8_t *mask_out, int32_t *n_nodes_out,
                            void *stream);

/* Hand-over to the target model's verification pass (Sec. 2.1; Fig. 3 "Tree Attention") for
 * `batch` trees as dart_tree_prune emits them (tokens, parents, n_nodes; `budget` = row
 * length of those arrays).  All pointers are device memory; one wavefront per tree.
 *   ctx_len       [batch] int32 prefix lengths n, or NULL (= 0)
 *   position_ids  [batch][budget] int32 out, or NULL: ctx_len + depth of the node below the
 *                 root (the root, t_{n+1}, sits at sequence position n); -1 beyond n_nodes.
 *                 Together with the ancestor mask this is what tree attention needs.
 *   target_next   [batch][budget] int32, or NULL to skip the acceptance walk: the token the
 *                 target model itself produces after each tree node (its arg-max at
 *                 temperature 0), as read from the verification pass
 *   accept_path   [batch][path_cap] int32 out: node indices of the accepted path, root
 *                 first, -1 padded.  A child is accepted iff its token equals target_next
 *                 of its parent; the walk stops at the first node without such a child.
 *   n_accepted    [batch] int32 out: accepted draft tokens = path length - 1 (tau of the step)
 *   next_token    [batch] int32 out: target_next at the last accepted node, i.e. the root of
 *                 the next draft step
 * path_cap >= 1 bounds the path (DART_MAX_K + 1 always suffices).
 * Errors: ARG (NULL tokens/parents/n_nodes; target_next without the three outputs; batch < 1;
 * budget not in 1..DART_MAX_BUDGET; path_cap < 1), HIP. */
dart_status dart_tree_verify_greedy(int batch, const int32_t *tokens, const int32_t *parents,
                                    const int32_t *n_nodes, int budget, const int32_t *ctx_len,
                                    int32_t *position_ids, const int32_t *target_next,
                                    int path_cap, int32_t *accept_path, int32_t *n_accepted,
                                    int32_t *next_token, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DART_H */
