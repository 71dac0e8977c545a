/*
 * ded_verify.h — C ABI of the MI355X (gfx950) draft-tree verification library.
 *
 * The library implements the verification stage of adaptive draft-verification decoding
 * (Sec. 2.4, "Draft Construction and Verification"): the target decoder runs ONE forward pass over a
 * pseudo-sequence that holds every draft token once, under a tree-attention mask that lets a draft
 * token see the context and its own ancestors only; then the model's own token at every node is
 * compared with the draft tokens below it and the longest approved path is kept.  The target models
 * are Llama-2 / Vicuna style decoders (Sec. 4.1): pre-norm, RMSNorm, rotary positions, (grouped-query)
 * soft-max attention, SwiGLU feed-forward, untied LM head.  Sampling is greedy (Sec. 4.1 default).
 *
 * Conventions
 *   - One GPU, one HIP stream per context.  A context is not re-entrant.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory.  The library allocates no device memory: everything it needs lives in the
 *     caller's workspace (ded_workspace_bytes) and KV buffers (ded_kv_layer_bytes).
 *   - Every call returns DED_OK (0) or a negative DED_E* code; nothing throws or aborts.
 *     All argument validation happens on the host before the first kernel launch.
 *   - Same inputs give bit-identical argmax, accepted tokens and compaction indices (fixed
 *     reduction orders, no floating-point atomics).
 *   - Tree encoding: node 0 is the root = the last committed token, whose K/V is not in the cache
 *     yet (parent[0] = -1, depth 0, position prefix_len).  Nodes 1..n-1 are draft tokens with
 *     0 <= parent[i] < i.  Node i sits at position prefix_len + depth(i).
 */
#ifndef DED_VERIFY_H
#define DED_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DED_OK = 0,
  DED_EINVAL = -1, /* null pointer, bad shape or unsupported configuration */
  DED_ETREE = -2,  /* malformed parent array */
  DED_ETOKEN = -3, /* token id outside [0, vocab) */
  DED_ECAP = -4,   /* prefix_len + n_nodes exceeds kv_capacity, or a size exceeds its maximum */
  DED_ESTATE = -5, /* call out of order (e.g. ded_accept without a pending step) */
  DED_EHIP = -6,   /* a HIP runtime call failed */
  DED_ENOMEM = -7, /* workspace too small / host allocation failed */
  DED_ENONFINITE = -8 /* the logits of a tree node hold a NaN or an infinity (see ded_accept) */
};

enum { DED_F32 = 0, DED_BF16 = 1 };

typedef struct ded_ctx ded_ctx; /* opaque */

/* Model and capacity description.  dtype is the type of the weight matrices, K/V rows and q / o
 * tensors that cross this interface (accumulation, residual stream, norms and soft-max statistics
 * are always fp32).  With DED_BF16 the library keeps 2-byte storage but computes with IEEE half
 * matrix-core operands: bf16 weights are widened exactly, K/V produced by the model are kept as
 * half, GEMM inputs and queries as hi + lo half pairs.  DED_BF16 needs head_dim == 128,
 * d_model % 128 == 0, d_ffn % 128 == 0, vocab % 16 == 0 and kv_capacity % 64 == 0;
 * max_nodes <= 256. */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_base; /* rotary base; pairing is (i, i + head_dim/2), angle pos * base^(-2i/head_dim) */
  float rms_eps;
  int32_t dtype; /* DED_F32 or DED_BF16 */
  int32_t max_batch;
  int32_t kv_capacity; /* cache slots per sequence */
  int32_t max_nodes;   /* largest tree (root included) per sequence */
} ded_config;

/* Weights, device memory, row-major, every linear map stored [out_features][in_features] (y = W x),
 * in the config's dtype; norm gains are fp32.  The per-layer members are HOST arrays of n_layers
 * device pointers.  ded_verify_init re-lays the matrices out inside the workspace; after it returns
 * the caller may release or overwrite these buffers.
 *   wqkv[l]     [(H + 2 Hkv) * hd][d]  rows: all query heads, then all key heads, then all value heads
 *   wo[l]       [d][H * hd]
 *   wgate_up[l] [2 F][d]               rows: gate projection, then up projection
 *   wdown[l]    [d][F]                                                                    */
typedef struct {
  const void *emb;         /* [vocab][d] */
  const void *lm_head;     /* [vocab][d] */
  const float *final_norm; /* [d] */
  const void *const *wqkv;
  const void *const *wo;
  const void *const *wgate_up;
  const void *const *wdown;
  const float *const *norm_attn; /* [n_layers] -> [d] */
  const float *const *norm_ffn;  /* [n_layers] -> [d] */
} ded_weights;

/* KV cache: HOST arrays of n_layers device buffers, each ded_kv_layer_bytes(cfg) bytes, holding
 * max_batch sequences of kv_capacity slots.  The element layout inside a buffer belongs to the
 * library (bf16 caches are stored as matrix-core operand fragments); use ded_kv_store / ded_kv_load
 * to move plain [Hkv][n][hd] rows in and out.  Keys are stored after the rotary embedding. */
typedef struct {
  void *const *k;
  void *const *v;
} ded_kv;

/* Sizes the caller must allocate (bytes of device memory). 0 on an invalid config. */
size_t ded_workspace_bytes(const ded_config *cfg);
size_t ded_kv_layer_bytes(const ded_config *cfg);

/* Host-only check of a step's arguments (the same check ded_verify_step performs before it launches
 * anything): DED_OK, DED_EINVAL, DED_ETREE, DED_ETOKEN or DED_ECAP.  Touches no device. */
int ded_validate_tree(const ded_config *cfg, int32_t batch, const int32_t *prefix_len,
                      const int32_t *n_nodes, const int32_t *parent, const int32_t *token);

/* Pseudo-sequence of Sec. 2.4 (Draft Construction and Verification): merges ranked candidate
 * continuations of the last committed token into one tree in which every candidate is a root-to-node
 * path and every common prefix appears once - the input ded_verify_step takes.  Host only, touches
 * no device.
 *   root_token   the last committed token (node 0)
 *   n_cand       number of candidates, in rank order; cand_len [n_cand] their lengths (0..max_len)
 *   cand_tokens  host [n_cand][max_len] token ids (entries past cand_len are ignored)
 *   max_nodes    node budget (>= 1, root included): a candidate is cut where the budget runs out,
 *                later candidates still follow nodes that exist
 *   parent, token  host outputs [max_nodes]; nodes are numbered in order of first appearance, so
 *                  parent[0] = -1 and 0 <= parent[i] < i
 *   cand_end     host output [n_cand] or NULL: the node where candidate c ends (or was cut)
 *   n_nodes      host output: nodes written
 * Errors: DED_EINVAL (null output, negative sizes, a length above max_len). */
int ded_build_tree(int32_t root_token, int32_t n_cand, const int32_t *cand_len, const int32_t *cand_tokens,
                   int32_t max_len, int32_t max_nodes, int32_t *parent, int32_t *token,
                   int32_t *cand_end, int32_t *n_nodes);

/* ---- Draft maker (host only, touches no device; the paper runs it on the CPU beside the verification step) ----
 *
 * ded_trigram is the LLM representative of Sec. 2.2: for a context (w_{i-2}, w_{i-1}) the words that may follow and
 * their probabilities.  The successors of a context keep their order of first appearance (corpus order, then the
 * insertions of ded_trigram_adjust); that order fixes expansion order, tie breaks and the inverse CDF below.
 * All probabilities and scores are double precision.  A ded_trigram is not thread safe. */
typedef struct ded_trigram ded_trigram;

/* NULL if the host is out of memory.  ded_trigram_free accepts NULL. */
ded_trigram *ded_trigram_create(void);
void ded_trigram_free(ded_trigram *m);

/* Adds the tri-grams of one document (host [n] token ids; n < 3 adds nothing) to the counts C(w_{i-2}, w_{i-1}, w_i)
 * and C(w_{i-2}, w_{i-1}) of Eq. (1); the bi-gram count is the number of tri-grams that start with the pair.
 * `times` >= 0 counts the document as if it occurred that often in the corpus.
 * Errors: DED_EINVAL, DED_ENOMEM. */
int ded_trigram_count(ded_trigram *m, const int32_t *tokens, int64_t n, int64_t times);

/* (Re)builds the matrix from the counts: P = C(w_{i-2}, w_{i-1}, w_i) / C(w_{i-2}, w_{i-1}) (Eq. (1)) for every
 * tri-gram counted at least t times (the elimination threshold of Appendix F.1, t = 12 there; survivors are not
 * re-normalised, contexts left without successors disappear).  Discards earlier ded_trigram_adjust updates. */
int ded_trigram_finalize(ded_trigram *m, int32_t t);

/* Adjust3Gram (Appendix G, Alg. 2): for every tri-gram inside the last max_length tokens of `tokens` (host [n]):
 * p <- min(p + increment, max_prob), or p <- increment for a tri-gram that is new (appended to its context, which
 * is created if needed).  The paper gives no values for increment, max_prob and max_length. */
int ded_trigram_adjust(ded_trigram *m, const int32_t *tokens, int64_t n, int64_t max_length, double increment,
                       double max_prob);

/* Successors of (w0, w1): *n_out = how many there are; the first min(cap, *n_out) go to words / probs (host). */
int ded_trigram_lookup(const ded_trigram *m, int32_t w0, int32_t w1, int32_t cap, int32_t *words, double *probs,
                       int32_t *n_out);

/* Number of tri-grams in the matrix (negative: DED_EINVAL). */
int64_t ded_trigram_size(const ded_trigram *m);

/* The draft search of Sec. 2.3 / Appendix G, Alg. 1 from the last two tokens (w0, w1) of the sequence:
 * `iterations` rounds of selection by the score of Eq. (2), (3)
 *     PUCT(s,a) = Q(s,a) + E P(s,a) sqrt(sum_b N(s,b)) / (1 + N(s,a)),  E = c1 + log((sum_b N(s,b) + c2 + 1) / c2)
 * (Q = accumulated score / visits of the child, 0 if unvisited; P = its tri-gram probability; first child wins a
 * tie), expansion (all successors at once, the search goes on with the one created last), simulation up to l words
 * (inverse CDF over the successors in stored order, weights relative to their sum, with
 * uniform[iteration * l + words already in the sentence]) and back-propagation of 1 + the sum of the sentence's
 * tri-gram probabilities.  The root-to-leaf paths of the search tree, ranked by the leaf's accumulated score
 * (depth-first order among equals), are the candidates; the best n are returned.
 *   uniform      host [n_uniform] numbers in [0, 1), n_uniform >= iterations * l; the caller owns the randomness
 *   cand_tokens  host output [n][l]; cand_len [n] words of each candidate (1..l); cand_score [n] or NULL
 *   n_cand       host output: candidates written (0 if the context (w0, w1) is unknown)
 * Appendix F.1 uses iterations = 150, l = 4, n = 24, c1 = 32, c2 = 8.
 * Errors: DED_EINVAL (null, l < 1, c2 <= 0, too few uniforms), DED_ENOMEM. */
int ded_draft_mcts(const ded_trigram *m, int32_t w0, int32_t w1, int32_t iterations, int32_t l, int32_t n,
                   double c1, double c2, const double *uniform, int64_t n_uniform, int32_t *cand_tokens,
                   int32_t *cand_len, double *cand_score, int32_t *n_cand);

/* Creates a context: validates cfg, re-lays out the weights into `workspace` (device, 256-byte
 * aligned, >= ded_workspace_bytes) on `hip_stream` (a hipStream_t; NULL = the default stream) and
 * waits for that to finish.  The workspace and KV buffers must outlive the context; their contents
 * are the library's while the context lives.  Errors: DED_EINVAL, DED_ENOMEM, DED_EHIP. */
int ded_verify_init(const ded_config *cfg, const ded_weights *weights, const ded_kv *kv,
                    void *workspace, size_t workspace_bytes, void *hip_stream, ded_ctx **out);
void ded_verify_free(ded_ctx *ctx);

/* The verification forward of Sec. 2.4, enqueued on the context's stream (asynchronous).
 *   batch       number of sequences, 1..max_batch; sequence b uses cache slot range b
 *   prefix_len  host [batch]: tokens already in the cache of sequence b
 *   n_nodes     host [batch]: tree rows of sequence b, 1..max_nodes (root included)
 *   parent      host [batch][max_nodes]: parent[0] = -1, 0 <= parent[i] < i
 *   token       host [batch][max_nodes]: token ids, token[0] = the root token
 *   logits_out  device fp32 [batch][max_nodes][vocab] or NULL; when given, the rows of the real
 *               nodes are written there (rows of absent nodes are left untouched)
 * Effects: K/V of node i of sequence b are written to cache slot prefix_len[b] + i (scratch until
 * accepted); the per-node argmax and top-1/top-2 margin are kept in the workspace.  With DED_BF16 the
 * [rows][vocab] logits themselves reach memory only when logits_out is given or the context has been
 * used with ded_sample before: otherwise the LM-head GEMM hands the argmax its per-tile candidates
 * directly (same tokens and margins, bit for bit).
 * Errors: DED_EINVAL, DED_ETREE, DED_ETOKEN, DED_ECAP, DED_EHIP.  On error nothing was launched. */
int ded_verify_step(ded_ctx *ctx, int32_t batch, const int32_t *prefix_len, const int32_t *n_nodes,
                    const int32_t *parent, const int32_t *token, float *logits_out);

/* Stochastic approval (Sec. 2.4: at each position a token is sampled from the model's distribution and
 * compared with the draft token; Sec. 4.4 varies temperature and top-p).  Optional call between
 * ded_verify_step and ded_accept: replaces the model's token at every node of the pending step - the
 * argmax - by a sample; ded_accept then walks with the sampled tokens.
 *   p_i = softmax(logits / temperature); the nucleus is the smallest set of most probable tokens whose
 *   probabilities reach top_p (ties with its last member included); the token is the smallest id j of
 *   the nucleus with  sum_{i in nucleus, i <= j} p_i > u * sum_{nucleus} p.
 *   temperature > 0, 0 < top_p <= 1
 *   uniform  host [batch][max_nodes], one number in [0, 1) per node, drawn by the caller
 * Synchronises the stream.  ded_get_argmax afterwards returns the sampled tokens (margins unchanged).
 * The first sampled step of a DED_BF16 context runs the LM head once more to obtain the logits that the
 * step did not keep; later steps of that context keep them.
 * Errors: DED_EINVAL (range of an argument, null), DED_ESTATE (no pending step), DED_ENONFINITE, DED_EHIP. */
int ded_sample(ded_ctx *ctx, float temperature, float top_p, const float *uniform);

/* Approval walk + cache compaction for the pending step (Sec. 2.4: a draft token is approved when
 * it equals the model's token at its parent; the draft is discarded from the first mismatch on).
 *   mode 0  greedy walk: end node = the deepest approved node (lowest index among equally deep);
 *   mode 1  force-accept: the tree must be a chain and all of it is kept (chunked prefill).
 * Outputs (host; stride = max_nodes + 1 per sequence):
 *   accepted_tokens [batch][max_nodes+1]  draft tokens on the kept path below the root, then the
 *                                         model's own token at the end node (the next root)
 *   n_accepted      [batch]               number of tokens written (path length)
 *   compaction_idx  [batch][max_nodes+1]  node indices of the kept path, root first
 *   new_prefix_len  [batch]               prefix_len + path length
 * The K/V of path node j move to slot prefix_len + j; slots beyond new_prefix_len are dead.
 * Non-finite values: if the logits of any real node of a sequence hold a NaN or an infinity (weights that
 * are not finite, or activations beyond the half-precision range of the DED_BF16 matrix-core operands,
 * |x * gain| > 65504), there is no meaningful model token: the call returns DED_ENONFINITE, writes no
 * output, keeps nothing of ANY sequence of the batch (every cache is as it was before the step; the
 * slots the step appended are zeroed) and the step is consumed.
 * Synchronises the stream.  Errors: DED_EINVAL, DED_ESTATE, DED_ETREE (mode 1, not a chain),
 * DED_ENONFINITE, DED_EHIP. */
int ded_accept(ded_ctx *ctx, int32_t mode, int32_t *accepted_tokens, int32_t *n_accepted,
               int32_t *compaction_idx, int32_t *new_prefix_len);

/* Per-node model tokens of the last step: argmax host [batch][max_nodes] (lowest id on exact ties),
 * margin host [batch][max_nodes] or NULL (top-1 minus top-2 logit).  Synchronises the stream.
 * DED_ENONFINITE (nothing written) if the logits of a real node hold a NaN or an infinity. */
int ded_get_argmax(ded_ctx *ctx, int32_t *argmax, float *margin);

/* Plain <-> library layout for `n` cache slots starting at `first_slot` of sequence `seq`, layer
 * `layer`.  k_plain / v_plain: device [Hkv][n][hd] in the config's dtype (either may be NULL).
 * Asynchronous on the context's stream.  Errors: DED_EINVAL, DED_ECAP, DED_EHIP. */
int ded_kv_store(ded_ctx *ctx, int32_t layer, int32_t seq, int32_t first_slot, int32_t n,
                 const void *k_plain, const void *v_plain);
int ded_kv_load(ded_ctx *ctx, int32_t layer, int32_t seq, int32_t first_slot, int32_t n,
                void *k_plain, void *v_plain);

/* Tree-masked attention of ONE layer on its own (Sec. 2.4, the tree-attention mask), for queries
 * and tree K/V supplied by the caller: q device [batch][max_nodes][H][hd], k_tree / v_tree device
 * [batch][Hkv][max_nodes][hd] (already rotated), all in the config's dtype; the prefix K/V are
 * whatever the cache of `layer` holds in slots [0, prefix_len).  The tree K/V are first written to
 * slots prefix_len + i.  out device [batch][max_nodes][H][hd], config dtype.  Asynchronous.
 * Errors as ded_verify_step. */
int ded_tree_attention(ded_ctx *ctx, int32_t layer, int32_t batch, const int32_t *prefix_len,
                       const int32_t *n_nodes, const int32_t *parent, const void *q,
                       const void *k_tree, const void *v_tree, void *out);

/* ded_tree_attention for callers that cannot allocate device memory and have no workspace region to spare for
 * it: code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments,
 * same kernels and bit-identical output, but every transient device buffer of the call (the uploaded tree
 * description, the re-laid-out queries and output, the split-KV partial results) lives in an array that is
 * part of the library's own device image: ded_static_scratch_bytes() bytes (32 MiB) per GPU, held from the
 * first ded_verify_init on that GPU until the process ends.  The call allocates nothing and frees nothing.
 * The context's device must be current.  A call whose buffers would not fit the array (roughly
 * batch * n_heads * key ranges * padded nodes * 520 bytes + 8 * rows * n_heads * head_dim bytes) is refused
 * with DED_ECAP before anything is enqueued; DED_BF16 contexts only (DED_EINVAL otherwise).  All calls on
 * one GPU share the array and it keeps the last call's contents (every element that is read is written first
 * by the same call, nothing has to start at zero); calls that overlap in time on one GPU - from different
 * contexts or streams - race.  Asynchronous.  Other errors as ded_tree_attention. */
int ded_tree_attention_static(ded_ctx *ctx, int32_t layer, int32_t batch, const int32_t *prefix_len,
                              const int32_t *n_nodes, const int32_t *parent, const void *q,
                              const void *k_tree, const void *v_tree, void *out);
size_t ded_static_scratch_bytes(void);

/* Kernel timing.  While enabled, every kernel launch of the forward is bracketed by HIP events on
 * the context's stream (this serialises nothing but adds event overhead, so use a separate pass).
 * ded_profile_read synchronises, then fills up to `cap` entries: names[i] points to a static string,
 * total_ms[i] is the summed duration and launches[i] the launch count since ded_profile_enable.
 * Returns the number of kernel classes (>= 0) or a negative error. */
int ded_profile_enable(ded_ctx *ctx, int32_t on);
int ded_profile_read(ded_ctx *ctx, int32_t cap, const char **names, double *total_ms, int64_t *launches);

/* Measurement aid, not part of the method: one pass of plain 16-byte-per-lane reads over `bytes` of device
 * memory (device_buffer 16-byte aligned; sink4: 4 bytes of device memory that the kernel may write),
 * enqueued on hip_stream.  bytes / kernel time is the streaming-read rate this chip sustains, the
 * ceiling that the weight- and cache-streaming kernels of the library are reported against.
 * Errors: DED_EINVAL, DED_EHIP. */
int ded_probe_stream_read(const void *device_buffer, size_t bytes, void *sink4, void *hip_stream);

const char *ded_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DED_VERIFY_H */
