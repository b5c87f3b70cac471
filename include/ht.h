/*
 * ht.h — C ABI of the Hidden Transfer tree-verify decoding library for AMD MI355X (gfx950).
 *
 * The library computes, at batch 1 on one GPU, the decode step of "Parallel Decoding via Hidden
 * Transfer for Lossless Large Language Model Acceleration" (arXiv 2404.12022):
 *
 *   transfer  : pseudo hidden states p_i = W_i h  for the next k positions        (Sec. 3.2, eq. of Sec. 3.3)
 *   draft     : the pseudo rows run through the remaining blocks and the original
 *               LM head; their top candidates fill a static tree                   (Sec. 1, 3.2, 3.4)
 *   verify    : one forward of the flattened tree with ancestor-only attention and
 *               original positional indices over the KV cache                      (Sec. 3.4, 3.4.1)
 *   accept    : last accepted position under greedy decoding, next token, and the
 *               KV cache keeps only the accepted rows                              (Fig. 2, Sec. 3.4, 4.1)
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless marked "host".  The library
 *     allocates no device memory: all of its device state lives in the caller's `workspace`, including,
 *     for bf16 models, a repacked copy of every projection matrix (streaming layout).
 *   - Matrices are row-major [out_features, in_features]; y = x W^T.  No biases.
 *   - `stream` is a hipStream_t passed as void*.  Calls enqueue on it and return without waiting unless
 *     stated otherwise.  One model is used from one stream at a time; calls are not re-entrant.
 *   - Positions are 0-based: the cache holds positions 0..n-1, the tree root sits at position n and a
 *     node of depth e at n+e.  "Layer t" is the residual stream after t complete blocks.
 *   - Return value: HT_OK (0) or a negative error.  Arguments and state are checked before anything is
 *     enqueued: HT_EINVAL, HT_ECAPACITY, HT_ETREE, HT_ESTATE and HT_EUNSUPPORTED leave the model and the
 *     stream as they were.  HT_EHIP reports a failed HIP call, which may come after part of the work was
 *     enqueued: the model is then in an undefined state and needs a new ht_prefill (ht_decode_steps also
 *     returns it when the device's own step log is inconsistent).  `ht_last_error()` gives a thread-local
 *     message.  No exception crosses this boundary.
 */
#ifndef HT_H_
#define HT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ht_model ht_model; /* opaque, host side, owned by the library */

enum { HT_OK = 0, HT_EINVAL = -1, HT_ECAPACITY = -2, HT_ETREE = -3, HT_ESTATE = -4, HT_EHIP = -5,
       HT_EUNSUPPORTED = -6 };
enum { HT_F32 = 0, HT_BF16 = 1 };
enum { HT_MAX_TRANSFER = 8, HT_MAX_TREE = 128 /* nodes of a tree */, HT_MAX_ROWS = 256 /* rows of a pass */,
       HT_MAX_TOPK = 64 };

/* Llama-style decoder shape plus the hidden-transfer hyper-parameters (Sec. 3.3: the number of
 * transfer steps k and the transfer layers t_i; Sec. 4.1 uses a different layer for every step).  The layers must
 * not decrease, t_1 <= t_2 <= .. <= t_k; steps that share a layer share one saved hidden state ("slot": slot 0
 * is the lowest distinct layer). */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_base;
  int32_t dtype;                             /* HT_F32 or HT_BF16: storage type of weights, activations, KV */
  int32_t k;                                 /* 1..HT_MAX_TRANSFER */
  int32_t transfer_layer[HT_MAX_TRANSFER];   /* 1 <= t_1 <= .. <= t_k < n_layers: residual after t_i blocks */
  int32_t max_cache;                         /* KV slots per layer (multiple of 8) */
  int32_t max_tree;                          /* most rows of a pass: tree nodes (root included) plus pseudo
                                                rows riding in the verify pass; <= HT_MAX_ROWS (a tree itself has
                                                at most HT_MAX_TREE nodes).  Projections run 128 rows per launch:
                                                a pass of more rows streams the weights twice. */
} ht_config;

/* Borrowed weight pointers (device).  They must outlive the model.  Per-layer arrays are host arrays
 * of n_layers device pointers; w_transfer is a host array of k device pointers. */
typedef struct {
  const void *tok_emb;                       /* [vocab, d] */
  const void *final_norm;                    /* [d] */
  const void *lm_head;                       /* [vocab, d] */
  const void *const *attn_norm;              /* [d] */
  const void *const *wq;                     /* [n_heads*head_dim, d] */
  const void *const *wk, *const *wv;         /* [n_kv_heads*head_dim, d] */
  const void *const *wo;                     /* [d, n_heads*head_dim] */
  const void *const *ffn_norm;               /* [d] */
  const void *const *w_gate, *const *w_up;   /* [d_ffn, d] */
  const void *const *w_down;                 /* [d, d_ffn] */
  const void *const *w_transfer;             /* k x [d, d] */
} ht_weights;

/* Loading a model that is larger than half of the GPU memory (bf16 only).  Every bf16 projection is copied
 * into the workspace in the library's streaming layout, so the original wq/wk/wv/wo/w_gate/w_up/w_down
 * matrices and lm_head are only read while they are packed.  A caller that cannot hold both copies leaves those
 * ht_weights entries NULL in ht_init_model (per layer, all seven together) and supplies them afterwards, one
 * layer at a time; the source tensors may be released as soon as `stream` has passed the call.  Every layer and
 * the head must have been supplied before ht_prefill (HT_ESTATE otherwise).  Norm gains, the embedding table
 * and the transfer maps are always borrowed. */
int ht_load_layer(ht_model *m, int32_t layer, const void *wq, const void *wk, const void *wv, const void *wo,
                  const void *w_gate, const void *w_up, const void *w_down, void *stream);
int ht_load_lm_head(ht_model *m, const void *lm_head, void *stream);

/* Bytes of device workspace `ht_init_model` needs for this configuration (KV cache, activations,
 * tree tables, decoder state). */
int ht_workspace_bytes(const ht_config *cfg, size_t *out_bytes);

/* Validates cfg, carves `workspace` (device, 256-byte aligned, >= ht_workspace_bytes) and clears it on
 * `stream`.  The returned model starts with an empty cache and no tree. */
int ht_init_model(const ht_config *cfg, const ht_weights *weights, void *workspace, size_t workspace_bytes,
                  void *stream, ht_model **out);
int ht_free_model(ht_model *m);

/* Static candidate tree (Sec. 3.4.1 "pre-defined tree structure"): T nodes, root included.
 * T <= min(max_tree, HT_MAX_TREE); parent[0] = -1, 0 <= parent[v] < v, depth <= k; rank[v] (v >= 1) selects the rank-th best candidate
 * of pseudo position depth[v], 0 <= rank < HT_MAX_TOPK, distinct among siblings.  Host arrays, copied
 * before return.  HT_ETREE if malformed. */
int ht_set_tree(ht_model *m, int32_t T, const int32_t *parent /*host*/, const int32_t *rank /*host*/, void *stream);

/* A tree chosen anew at every step instead of a fixed one.  The paper decodes with a pre-defined tree (Sec. 3.4.1)
 * and names the tree's structure as what the speed hangs on (Limitation section); this rule is the library's own.
 * After every draft the b best candidates of each of the k pseudo positions get their log-probability (log-softmax
 * over the whole vocabulary, float32).  A node that picks ranks r_1 .. r_e along its path scores
 * lp[1][r_1] + .. + lp[e][r_e], added in float32 from the root down (NaN counts as -inf): the draws of the k
 * positions do not depend on one another (Sec. 3.2), so exp(score) is how likely a greedy verification reaches the
 * node if the drafts were exact.  The tree is the root plus the T - 1 nodes that come first in the order (score
 * descending, depth ascending, rank path ascending), numbered in that order; it is closed under taking parents.
 * From this call on `ht_tree_verify_step(tree_tokens = NULL)` and `ht_decode_steps` build it on the device before
 * each verify pass (views HT_BUF_TREE_PARENT, HT_BUF_TREE_RANK, HT_BUF_CANDIDATE_LOGPROBS show the last one);
 * forced tree tokens and `ht_set_fused_nodes` are HT_ESTATE in this mode; `ht_set_tree` returns to a fixed tree.
 * HT_ETREE unless 1 <= T <= min(max_tree, HT_MAX_TREE), 1 <= b <= HT_MAX_TOPK and T - 1 <= b + b^2 + .. + b^k. */
int ht_set_dynamic_tree(ht_model *m, int32_t T, int32_t b, void *stream);

/* Draft inside the verify pass (Fig. 2 caption and the end of Sec. 3.4: one forward verifies the current
 * candidates and produces the next ones; Sec. 5 names the price, a longer input sequence).  Every listed
 * tree node v gets k pseudo rows: when the pass reaches the transfer layer, row (v, i) = W_i applied to v's
 * layer-t residual joins at position n + depth[v] + i and sees the cache, v's ancestors-or-self, the pseudo
 * rows (v, j < i) and itself; the LM head turns it into the distribution of the token i places after v.  If
 * the next acceptance ends on a listed node, the following `ht_tree_verify_step(tree_tokens = NULL)` builds its
 * tree from those rows and needs no `ht_transfer` and no draft pass (an `ht_transfer(m, NULL, NULL, ..)` in
 * between returns at once); if it ends elsewhere the step drafts after acceptance as without this call.
 * Either way the tokens are the same (the two schedules compute the same distributions).
 * nodes: host array of `count` distinct node ids of the current tree, count = 0 switches the feature off (always
 * allowed, also after ht_set_dynamic_tree, where any other count is HT_ESTATE); `ht_set_tree` also switches it off.  The pass then has T + count * k rows, which must fit max_tree (and
 * n + T + count * k must fit max_cache at every step): HT_ECAPACITY otherwise; HT_ETREE for bad ids;
 * HT_ESTATE without a tree. */
int ht_set_fused_nodes(ht_model *m, int32_t count, const int32_t *nodes /*host*/, void *stream);

/* Runs the prompt (host array of n token ids, n >= 1) through the model in chunks with plain causal
 * attention, fills the KV cache, sets the pending root token to the greedy next token and keeps the
 * layer-t residual of the last prompt token as the transfer source.  Resets any previous cache. */
int ht_prefill(ht_model *m, const int32_t *tokens /*host*/, int32_t n, void *stream);

/* Forward pass of the training stage for transfer step `step` (1-based i of Sec. 3.3) and its distillation loss.
 * The n tokens (HOST array) run causally; at layer t_i every hidden state h_j becomes a pseudo state W_i h_j that
 * goes on through blocks t_i+1..L at position id j + i, attending to the hidden states of positions 0 .. j+i-1 and
 * to itself (no other pseudo state); all rows pass the LM head.  The loss is the sum over j = 0 .. n-i-2 (the index
 * range of the loss equation, 0-based) of KL(P~_j || P_{j+i}), the pseudo state's distribution against that of the
 * hidden state it stands for, the first argument weighting the log ratio; float32 per term, summed in double in
 * index order on the host.  Forward only: the maps are not updated.
 * The sequence is processed in chunks of C = (max_tree - step) / 2 positions: blocks t_i+1..L and the LM head run a
 * chunk's hidden rows, `step` hidden rows of lookahead and its pseudo rows in one pass; blocks 1..t_i, which see
 * hidden rows only, run two chunks per pass.
 * kl_out: HOST [n - step - 1] or NULL; loss_out: HOST or NULL; logits_hidden_out: DEVICE [n, vocab] float32 or NULL
 * (a lookahead row is computed by two passes, which in bf16 may round it differently: the row returned is the one
 * the loss used);
 * logits_pseudo_out: DEVICE [n - step + 1, vocab] float32 or NULL (pseudo states exist for j <= n - step, the
 * positions whose visible hidden states all lie inside the sequence).  Waits for `stream`.
 * The KV cache afterwards holds the n tokens, but no pending root: decoding needs a new ht_prefill.  The tree set
 * by ht_set_tree / ht_set_dynamic_tree is kept.
 * HT_EINVAL unless 1 <= step <= k, n >= step + 2 and all tokens lie in the vocabulary; HT_ECAPACITY unless
 * max_tree >= step + 2 and n + (max_tree - step) / 2 <= max_cache; HT_ESTATE while deferred weights are missing. */
int ht_training_forward(ht_model *m, int32_t step, const int32_t *tokens /*host*/, int32_t n, float *kl_out /*host*/,
                        double *loss_out /*host*/, float *logits_hidden_out, float *logits_pseudo_out, void *stream);

/* The same forward pass and loss with all positions in one pass per block (Sec. 3.3: the doubled sequence of hidden
 * and pseudo hidden states), for sequences of hundreds or thousands of tokens: every projection runs once over all n
 * (above the transfer layer n + n - step + 1) rows on a kernel tiled over tokens and features, so the matrix cores
 * and not the weight stream set the pace; attention runs as one launch per block for the hidden rows (causal over
 * the KV cache) and one for the pseudo rows (pseudo row j over the hidden keys 0 .. j + step - 1, merged with its own
 * key and value, which live in the workspace, not in the cache).  The pseudo
 * states come from a matrix product with bf16-rounded hidden states (ht_training_forward and the decode step feed
 * the transfer map float32 states).  Same outputs and argument meaning as ht_training_forward.
 * train_ws: DEVICE, 256-byte aligned, >= ht_training_workspace_bytes(cfg, n) (activations of all 2 n rows, their
 * logits, the pseudo rows' keys and values, the packed transfer map).  Waits for `stream`.  The KV cache afterwards
 * holds the n tokens, but no pending root: decoding needs a new ht_prefill; the tree set before is kept.
 * HT_EUNSUPPORTED unless the model is bf16 on packed weights (widths and vocabulary multiples of 16, heads of 64 or
 * 128); HT_ECAPACITY unless n <= max_cache; HT_EINVAL / HT_ESTATE as for ht_training_forward. */
int ht_training_workspace_bytes(const ht_config *cfg, int32_t n, size_t *out_bytes);
int ht_training_forward_batched(ht_model *m, int32_t step, const int32_t *tokens /*host*/, int32_t n, float *kl_out /*host*/,
                                double *loss_out /*host*/, float *logits_hidden_out, float *logits_pseudo_out,
                                void *train_ws, size_t train_ws_bytes, void *stream);

/* Hidden transfer (Sec. 3.2; equation of Sec. 3.3): pseudo[i] = W_i h, i = 0..k-1, a bare matrix
 * product of the layer-t_i hidden state.  h_src: [slots, d] in the model dtype (one vector per distinct transfer
 * layer, lowest first), or NULL to use the saved residuals of the last
 * accepted token.  pseudo_out: [k, d] float32, or NULL; the result is also kept inside the model for
 * the next `ht_tree_verify_step`. */
int ht_transfer(ht_model *m, const void *h_src, float *pseudo_out, void *stream);

/* One tree-verify step (Sec. 3.4).
 *   tree_tokens == NULL: draft first — the pseudo rows of the last `ht_transfer` run through blocks
 *     t+1..L at positions n, n+1, .. seeing the cache, earlier pseudo rows and themselves, the LM head
 *     gives D[k, vocab], top candidates by (logit desc, id asc) fill the tree under the pending root.
 *   tree_tokens != NULL: device [T] token ids used as the tree (external drafter / forced trees);
 *     tree_tokens[0] should be the pending root for the result to be a greedy continuation.
 * Then the T rows are verified in one forward: row v at position n + depth[v] attends to cache[0, n)
 * and its ancestors-or-self; K/V go to cache slot n+v; the layer-t residuals are saved.
 * argmax_out: device [T] int32 or NULL, greedy token after each node (ties -> lowest id).
 * logits_out: device [T, vocab] float32 or NULL.
 * HT_ESTATE without a tree / prefill / (for drafting) transfer or in-pass drafts of the accepted node;
 * HT_ECAPACITY if n + max(T + fused rows, k) > max_cache. */
int ht_tree_verify_step(ht_model *m, const int32_t *tree_tokens, int32_t *argmax_out, float *logits_out,
                        void *stream);

/* Greedy acceptance and cache compaction (Fig. 2; Sec. 3.4, 4.1).  From the root, repeatedly follows the
 * first child (lowest node index) whose token equals the greedy token after the current node.  The m >= 1
 * nodes on that path are accepted: their K/V rows move to cache slots n..n+m-1, n += m, the pending root
 * becomes the greedy token after the last accepted node and its layer-t residual becomes the transfer
 * source.  All outputs are HOST pointers (may be NULL) filled before return: this call waits for `stream`.
 * accepted_tokens, path_out: [k+1]. HT_ESTATE unless it follows a verify step. */
int ht_accept_and_compact(ht_model *m, int32_t *n_accepted, int32_t *accepted_tokens, int32_t *next_root,
                          int32_t *path_out, void *stream);

/* `steps` whole decode steps without a host round trip in between: each step is ht_transfer, the draft pass,
 * ht_tree_verify_step on the drafted tree and ht_accept_and_compact (Sec. 3.2 - 3.4, drafting after acceptance),
 * but the cache length lives on the device: every kernel reads it there, the acceptance advances it, and this
 * call waits for `stream` once, after the last step.  Same tokens as the same number of single steps.
 * n_accepted: HOST [steps] or NULL; accepted_tokens: HOST [steps * (k + 1)] or NULL, the emitted tokens of all
 * steps back to back (sum of n_accepted entries are written); next_root: HOST or NULL.
 * HT_EINVAL unless 1 <= steps <= HT_MAX_LOOP_STEPS; HT_ESTATE without tree or prefill, between a verify step and
 * its ht_accept_and_compact, or while ht_set_fused_nodes lists nodes (the loop cannot take the data-dependent
 * branch that skips the draft pass); HT_ECAPACITY unless n + steps * (k + 1) + max(T, k) <= max_cache (the worst
 * case is checked up front: nothing on the device can report an overflow mid-loop). */
enum { HT_MAX_LOOP_STEPS = 64 };
int ht_decode_steps(ht_model *m, int32_t steps, int32_t *n_accepted, int32_t *accepted_tokens, int32_t *next_root,
                    void *stream);

int32_t ht_cache_len(const ht_model *m);      /* n */
const char *ht_last_error(void);

/* Read-only views of the model's device buffers, for tests and tools.  `which` is one of HT_BUF_*;
 * `layer` selects the decoder layer of the cache views and the transfer-layer slot of the saved residuals and
 * transfer sources.  The pointer stays valid until ht_free_model. */
enum { HT_BUF_DRAFT_LOGITS = 0 /* float [k, vocab] */, HT_BUF_CANDIDATES = 1 /* int32 [k, HT_MAX_TOPK] */,
       HT_BUF_TREE_TOKENS = 2 /* int32 [T] */,
       HT_BUF_SAVED_HIDDEN = 3 /* float [T, d] residuals at the transfer layer of slot `layer` */,
       HT_BUF_TRANSFER_SRC = 4 /* float [d] transfer source of slot `layer` */,
       HT_BUF_K_CACHE = 5 /* dtype [max_cache, n_kv_heads, head_dim] */,
       HT_BUF_V_CACHE = 6 /* dtype [n_kv_heads, head_dim, max_cache]: key index contiguous */,
       HT_BUF_PSEUDO = 7 /* float [k, d] */, HT_BUF_ROOT = 8 /* int32 [1] pending root token */,
       HT_BUF_FUSED_DRAFT_LOGITS = 9 /* float [fused nodes * k, vocab] of the last verify pass, rows in the order
                                        they joined it: slot by slot, node by node, step by step */,
       HT_BUF_FUSED_CANDIDATES = 10 /* int32 [fused nodes, k, HT_MAX_TOPK] */,
       HT_BUF_CANDIDATE_LOGPROBS = 11 /* float [k, HT_MAX_TOPK], dynamic tree only: entries 0..b-1 of every row */,
       HT_BUF_TREE_PARENT = 12 /* int32 [T] */, HT_BUF_TREE_RANK = 13 /* int32 [T] */ };
int ht_get_buffer(const ht_model *m, int32_t which, int32_t layer, void **dev_ptr, size_t *bytes);

/* ---- op-level entry points (same kernels as the model path) -------------------------------------- */

/* Tree-masked attention over a KV cache (Sec. 3.4.1): rotary at original positional indices, append,
 * ancestor-only softmax attention.
 *   q      [T, Hq, hd]  queries of the tree rows (pre-rotary if k_new != NULL)
 *   k_new, v_new [T, Hkv, hd] or both NULL.  If given, q and k_new are rotated at position n + depth[v]
 *          (pairs (j, j+hd/2), angle pos * rope_base^(-2j/hd)) and row v is stored at cache slot n+v
 *          before attending; if NULL, slots n..n+T-1 already hold the tree rows and q is used as is.
 *   k_cache [cap, Hkv, hd], v_cache [Hkv, hd, cap] (key index contiguous); cap multiple of 8, n + T <= cap
 *   out    [T, Hq*hd]: row v = softmax over {cache 0..n-1} U {n+u : u ancestor-or-self of v} of q.k/sqrt(hd), times V
 *   scratch: device bytes >= ht_tree_attention_scratch_bytes(...)
 * parent is a host array; this call turns it into depth and ancestor tables and uploads them into `scratch` from
 * pageable memory (the call may wait for the copy, and such a call cannot be captured into a HIP graph).
 * parent == NULL skips both: the tables an earlier call with the same T left in the same `scratch` are used again (a
 * serving loop uploads a tree once; that form is capturable and keeps no state outside its arguments, so calls from
 * several threads on their own scratch buffers and streams do not interfere).  T <= HT_MAX_ROWS.  dtype selects HT_F32 or HT_BF16 for q/k/v/out (softmax and sums in fp32). */
size_t ht_tree_attention_scratch_bytes(int32_t T, int32_t Hq, int32_t hd);
int ht_tree_attention(const void *q, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                      int32_t cap, int32_t n, int32_t T, const int32_t *parent /*host*/, int32_t Hq, int32_t Hkv,
                      int32_t hd, int32_t dtype, float rope_base, void *out, void *scratch, size_t scratch_bytes,
                      void *stream);

/* Skinny weight-streaming product out[M, N] (float32) = a[M, K] . w[N, K]^T with M <= HT_MAX_ROWS rows,
 * the contraction every projection of the verify step uses (Sec. 1: decoding time goes to loading the
 * parameters).  a must be readable up to ht_padded_rows(M) rows.
 *   ht_weight_pack        : bf16 w[N, K] (N % 16 == 0, K % 8 == 0) -> the library's streaming layout
 *                           (16-row x 32-column tiles in matrix-core operand order, contiguous along K);
 *                           `packed` needs ht_weight_pack_bytes(N, K) bytes (0 = shape not packable).
 *                           ht_init_model does the same for every projection of a bf16 model.
 *   ht_skinny_gemm_packed : the product on packed bf16 weights; scratch (may be NULL) holds split-K partials.
 *   ht_skinny_gemm        : convenience for either dtype: packs into scratch when it can, then multiplies.
 *                           scratch >= ht_skinny_gemm_scratch_bytes(M, N, K), 256-byte aligned.
 *   ht_gate_up_pack       : bf16 w_gate[f, K], w_up[f, K] (f % 16 == 0, K % 8 == 0) -> one packed matrix of 2 f
 *                           rows with gate and up row blocks alternating; `packed` needs
 *                           ht_weight_pack_bytes(2 f, K) bytes.
 *   ht_gate_up_silu_packed: the feed-forward block's first half as the verify pass runs it, one kernel:
 *                           act_out[M, f] (bf16) = silu(a . w_gate^T) * (a . w_up^T), a bf16 [M, K], fp32 sums.
 *                           The largest projection of a decoder block, hence the kernel bench.py takes the
 *                           roofline of.  HT_EINVAL on NULL pointers, M outside 1..HT_MAX_ROWS or bad f, K. */
/* The two steps of `ht_set_dynamic_tree`'s rule on their own (all pointers DEVICE).
 * ht_candidate_logprobs: d [rows, V] float32 logits, cand [rows, HT_MAX_TOPK] token ids of which the first b per row
 *   are read; lp [rows, HT_MAX_TOPK]: lp[i][r] = d[i][cand[i][r]] - log(sum_v exp d[i][v]) for r < b.
 *   HT_EINVAL unless 1 <= rows <= HT_MAX_ROWS, 1 <= b <= HT_MAX_TOPK, V >= 1.
 * ht_dynamic_tree: lp, cand [k, HT_MAX_TOPK] (first b per row read), root [1]; writes parent, depth, rank [T],
 *   anc [T, HT_MAX_ROWS / 64] (bit u of row v: u is v or an ancestor of v) and tokens [T] (the root token, then
 *   cand[depth - 1][rank] of every node).  HT_EINVAL / HT_ETREE as for `ht_set_dynamic_tree`. */
/* The loss term of `ht_training_forward` on its own (all pointers DEVICE): z holds rows of V float32 logits;
 * kl[p] = KL(softmax(z[row_a + p]) || softmax(z[row_b + p])) for p < pairs, the first argument weighting the log
 * ratio (Sec. 3.3).  HT_EINVAL unless 1 <= pairs <= 65535, V >= 1 and the row indices are >= 0. */
int ht_kl_divergence_rows(const float *z, int32_t row_a, int32_t row_b, int32_t pairs, int32_t V, float *kl,
                          void *stream);
int ht_candidate_logprobs(const float *d, const int32_t *cand, int32_t rows, int32_t b, int32_t V, float *lp,
                          void *stream);
int ht_dynamic_tree(const float *lp, const int32_t *cand, const int32_t *root, int32_t k, int32_t b, int32_t T,
                    int32_t *parent, int32_t *depth, int32_t *rank, uint64_t *anc, int32_t *tokens, void *stream);

int32_t ht_padded_rows(int32_t M);
size_t ht_weight_pack_bytes(int32_t N, int32_t K);
int ht_weight_pack(const void *w, int32_t N, int32_t K, void *packed, void *stream);
size_t ht_skinny_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K);
int ht_gate_up_pack(const void *w_gate, const void *w_up, int32_t f, int32_t K, void *packed, void *stream);
int ht_gate_up_silu_packed(const void *a, const void *packed, int32_t M, int32_t f, int32_t K, void *act_out,
                           void *stream);
int ht_skinny_gemm_packed(const void *a, const void *packed, int32_t M, int32_t N, int32_t K, float *out,
                          void *scratch, size_t scratch_bytes, void *stream);
int ht_skinny_gemm(const void *a, const void *w, int32_t M, int32_t N, int32_t K, int32_t dtype, float *out,
                   void *scratch, size_t scratch_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP-graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): `ht_skinny_gemm_packed` without a scratch argument.  The split-K partial sums go to a
 * device array of HT_NOALLOC_SCRATCH_BYTES that is part of the library image (every GPU the library runs on holds
 * its own copy until the process ends); the call allocates and frees nothing.  Same kernels, same K split and
 * therefore the same bits as `ht_skinny_gemm_packed` given enough scratch.  HT_ECAPACITY when the partial sums
 * (K splits x M x N x 4 bytes; shapes that need no split always fit) exceed the array; HT_EINVAL as for
 * `ht_skinny_gemm_packed`.  All calls on one GPU share that GPU's array, which keeps the last call's contents
 * (every element is written before it is read, so nothing is cleared): calls that overlap in time on one GPU,
 * from two streams or two threads, race; calls on one stream are safe back to back. */
#define HT_NOALLOC_SCRATCH_BYTES (16u << 20)
int ht_skinny_gemm_packed_noalloc(const void *a, const void *packed, int32_t M, int32_t N, int32_t K, float *out,
                                  void *stream);

/* Measurement aid for the roofline (Sec. 1: decoding time is the time to load the parameters): reads `buf`
 * (device, 16-byte aligned) once with the access pattern of the packed weight stream (256 workgroups, each
 * walking its own contiguous region in nontemporal 1 KiB wavefront loads) and does nothing else, so its time is
 * the floor for streaming that many bytes on this machine.  The largest multiple of 8 MiB not above `bytes` is
 * read and stored in *bytes_read (host, may be NULL); `sink` is a device word the kernel may write.
 * HT_EINVAL for NULL / misaligned / too small buffers. */
int ht_stream_read_probe(const void *buf, size_t bytes, void *sink, size_t *bytes_read, void *stream);

/* Measurement aid for the matrix-core roofline of the token-tiled products (the forward pass of the training stage,
 * Sec. 3.3): 512 workgroups of four wavefronts issue `iters` rounds of independent bf16 matrix-core instructions on
 * register operands and nothing else: form 0 = 32 accumulators of v_mfma_f32_16x16x32_bf16 per wavefront (the
 * instruction of the product kernels), form 1 = 8 accumulators of v_mfma_f32_32x32x16_bf16, both on small whole
 * numbers; forms 2 and 3 = the same two with operands in +-[1, 2) whose sign and mantissa bits are hashed (the
 * sustained rate depends on the operand bits).  *flops (host, may be NULL) receives the floating-point operations
 * of the launch; the caller times it.  `sink` is a device word the kernel may write.  HT_EINVAL for a NULL sink,
 * another form, or iters outside 1 .. 2^20. */
int ht_mfma_rate_probe(int32_t form, int32_t iters, void *sink, double *flops, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HT_H_ */
