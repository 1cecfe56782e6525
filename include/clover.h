/*
 * clover.h -- C ABI of the MI355X (gfx950) Clover-2 speculative-step library.
 *
 * One speculative step (paper Sec. 2.1 and Sec. 3):
 *   draft_tree          the Clover-2 draft head proposes a token tree,
 *   verify_tree         the target LLM scores every tree node in one pass (tree attention),
 *   accept_and_compact  greedy verification keeps the longest correct root path.
 *
 * Conventions
 *  - Every function returns CLOVER_OK (0) or a negative CLOVER_E_* code; nothing throws.
 *  - Arguments are validated on the host before anything is launched.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host memory.
 *  - The library allocates no device memory: KV caches, lengths and all scratch live in the
 *    caller's workspace; weights are borrowed for the lifetime of the context.  For bf16 models the
 *    workspace also holds the library's own copy of every linear weight in MFMA-fragment order
 *    (+1x the weight bytes); the originals are then read only by the embedding gathers.
 *  - Calls enqueue work on the stream given at init and return without synchronising, unless
 *    stated otherwise.  A HIP error found while launching is returned as CLOVER_E_HIP.
 *  - Model tensors (weights, norm gains, biases) are in the model dtype (fp32 or bf16 bit
 *    patterns); hidden states and logits cross the boundary as fp32; ids are int32.
 *  - Linear weights are row-major [out_features, in_features].
 *  - Rows are laid out [batch, max-nodes stride]: row (b, i) of a [B, R, ...] buffer is at
 *    index b*R + i where R is the stride named for that argument.
 */
#ifndef CLOVER_H_
#define CLOVER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CLOVER_OK = 0,
  CLOVER_E_NULL = -1,      /* a required pointer is null */
  CLOVER_E_CONFIG = -2,    /* inconsistent model configuration */
  CLOVER_E_TREE = -3,      /* tree is not a breadth-first rooted tree / rank or depth out of range */
  CLOVER_E_CAPACITY = -4,  /* workspace too small, or a sequence would outgrow max_seq */
  CLOVER_E_SHAPE = -5,     /* batch / row counts outside what the context was sized for */
  CLOVER_E_HIP = -6,       /* HIP runtime error (see clover_last_error) */
  CLOVER_E_STATE = -7      /* device-side guard tripped (reported by clover_seq_len) */
};

enum { CLOVER_DTYPE_F32 = 0, CLOVER_DTYPE_BF16 = 1 };
enum {
  CLOVER_FLAG_GENERIC = 1,       /* use the plain fp32-ALU kernels everywhere (no MFMA path) */
  CLOVER_FLAG_INTERVAL_MASK = 2  /* tree attention decides "is key w on the root path of query u" from two integers per
                                    node instead of a bit set per node: the linear-size tree mask of Appendix A.1, read
                                    as the interval labels of a depth-first numbering (w is u or an ancestor of u iff
                                    enter[w] <= enter[u] <= exit[w]).  Same results; lifts max_nodes to 256. */
};
#define CLOVER_MAX_NODES 128 /* upper bound on max_nodes with the bit-set mask (2 x 64 bit per node) */
#define CLOVER_MAX_NODES_INTERVAL 256 /* upper bound on max_nodes with CLOVER_FLAG_INTERVAL_MASK (static trees; a
                                         dynamic tree still has at most 128 nodes) */
#define CLOVER_MAX_DEPTH 8   /* upper bound on draft_depths */
#define CLOVER_MAX_RANK 16   /* ranks are < 16 */
#define CLOVER_MAX_PREFILL_ROWS 256 /* upper bound on prefill_rows: one weight pass of the many-row GEMM */

/* Model + capacity description.  Plain data, copied at init. */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float rope_base, rms_eps;
  int32_t dtype;         /* CLOVER_DTYPE_*: type of every model tensor.  KV caches: fp32 elements for fp32 models;
                            for bf16 models each cached value is a pair of bf16 numbers (hi + lo, 16 mantissa bits,
                            4 bytes): twice the bytes of a plain bf16 cache, the price of the 3e-2 logit bound */
  int32_t aug_layers;    /* decoder layers in the Augmenting Block (Sec. 3.3) */
  int32_t ad_heads;      /* heads of the Attention Decoder's cosine gate (Appendix A.3) */
  int32_t draft_depths;  /* D: deepest tree level the draft head can fill (FC_0 .. FC_{D-1}) */
  int32_t max_batch, max_seq, max_nodes;   /* max_seq: a multiple of 32 (the page size of the caches) */
  int32_t flags;         /* CLOVER_FLAG_* */
  int32_t prefill_rows;  /* prompt rows clover_prefill processes per pass (0: max_batch * max_nodes); the row buffers
                            of the workspace are sized for max(max_batch * max_nodes, prefill_rows).  At most 256. */
} clover_config;

/* Static tree topology (Sec. 2.1: candidates merged on common prefixes form a tree).
 * HOST arrays, copied.  Nodes in breadth-first order: parent[0] = -1, 0 <= parent[u] < u,
 * depth non-decreasing in u.  rank[u] says node u carries the rank[u]-th best continuation
 * of its parent (0 = best); siblings have distinct ranks. */
typedef struct {
  int32_t n_nodes;
  const int32_t *parent;
  const int32_t *rank;
} clover_tree;

/* One LLaMA-style decoder layer.  dev pointers, model dtype. */
typedef struct {
  const void *attn_norm; /* [H] */
  const void *wq;        /* [n_q*d, H] */
  const void *wk;        /* [n_kv*d, H] */
  const void *wv;        /* [n_kv*d, H] */
  const void *wo;        /* [H, n_q*d] */
  const void *ffn_norm;  /* [H] */
  const void *w_gate;    /* [F, H] */
  const void *w_up;      /* [F, H] */
  const void *w_down;    /* [H, F] */
} clover_layer_weights;

/* Attention Decoder (Appendix A.3): norm on x, q from x, k and v from y, all with bias. */
typedef struct {
  const void *norm;          /* [H] */
  const void *wq, *bq;       /* [H,H], [H] */
  const void *wk, *bk;
  const void *wv, *bv;
} clover_ad_weights;

/* All weights.  The struct and the `layers`/`aug`/`fc_w`/`fc_b` arrays are HOST memory (copied
 * at init); every tensor pointer inside is a dev pointer borrowed until clover_destroy. */
typedef struct {
  const void *embed;                     /* [V,H] target input embedding */
  const clover_layer_weights *layers;    /* host array [n_layers] */
  const void *final_norm;                /* [H] */
  const void *lm_head;                   /* [V,H]; its rows are also the draft's token embeddings */
  clover_ad_weights ad1, ad2;            /* before the Augmenting Block / in the regressive loop */
  const clover_layer_weights *aug;       /* host array [aug_layers] */
  const void *fc0_w, *fc0_b;             /* head 0: [H,H], [H] */
  const void *const *fc_w;               /* host array [draft_depths]: fc_w[j] = [H,2H] for j>=1, fc_w[0] unused */
  const void *const *fc_b;               /* host array [draft_depths]: [H] */
  const void *head_norm;                 /* [H] norm before the shared LM head */
} clover_weights;

typedef struct clover_ctx clover_ctx;    /* opaque; owned by the library */

/* Bytes of device workspace a context of this configuration needs (256-byte aligned base). */
int clover_workspace_bytes(const clover_config *cfg, size_t *bytes_out);

/* Create a context.  `workspace` is a dev pointer to >= clover_workspace_bytes bytes that the
 * caller keeps alive; `hip_stream` is a hipStream_t (NULL = default stream).  Sequence lengths
 * start at zero.  Synchronises the stream once (uploads the tree tables). */
int clover_init(const clover_config *cfg, const clover_weights *weights, const clover_tree *tree,
                void *workspace, size_t workspace_bytes, void *hip_stream, clover_ctx **ctx_out);
int clover_destroy(clover_ctx *ctx);

/* Forget all sequences: target and augmenting-block cache lengths become zero. */
int clover_reset(clover_ctx *ctx);

/* Replace the static tree (e.g. a chain for prompt chunks, one node for plain decoding).
 * n_nodes <= max_nodes.  Synchronises the stream. */
int clover_set_tree(clover_ctx *ctx, const clover_tree *tree);

/* Dynamic (score-pruned) tree (Sec. 4.1: the tree is constructed from the draft's own probabilities).  After this
 * call draft_tree chooses a new topology for every sequence and call, and verify_tree / accept_and_compact use
 * it: a candidate's score is the sum of the draft log-probabilities along its root path; the root expands into
 * its `topk` most probable tokens; at every depth 1 .. draft_depths-1 the `frontier` best candidates are expanded
 * the same way; the n_nodes - 1 best of all candidates (score descending, shallower first, older first) and the
 * root form the tree, numbered breadth-first.  Ties go to the lower token id / older candidate.  At most 256
 * candidates (1 + topk + (draft_depths-1) * frontier * topk), topk <= 16, frontier <= 64.  clover_set_tree returns
 * to a static tree.  Synchronises the stream. */
int clover_set_dynamic_tree(clover_ctx *ctx, int32_t n_nodes, int32_t topk, int32_t frontier);

/* Test helper (synchronises): the dynamic tree of sequence b as the last draft_tree left it.  HOST arrays:
 * parent, rank, keep [n_nodes] (keep = candidate number of every tree node); cand_token, cand_score, cand_parent
 * [256] (candidates in creation order: 0 = root, depth-1 candidates by rank, then per depth the children of the
 * expanded candidates in (expansion order, rank) order); frontier [CLOVER_MAX_DEPTH * 64]: the candidates
 * expanded at depth j, best first, at [j * 64 ...). */
int clover_read_dynamic_tree(clover_ctx *ctx, int32_t b, int32_t *parent_out, int32_t *rank_out, int32_t *keep_out,
                             int32_t *cand_token_out, float *cand_score_out, int32_t *cand_parent_out,
                             int32_t *frontier_out);

/* Draft head (Sec. 3; Sec. 3.1-3.3; Appendix A.3).  For every sequence b < batch with
 * m[b] >= 1: rows i < m[b] pair hid_acc[b,i] (target hidden state before the final norm) with
 * next_tok[b,i] (the token that followed it; the last is the new root).  AD1 and the Augmenting
 * Block run on those rows and append m[b] rows to the block's own KV cache; then head 0 and the
 * regressive AD2/FC updates fill the tree level by level through the shared LM head.
 *   hid_acc     dev in  fp32 [batch, max_nodes, H]
 *   next_tok    dev in  int32 [batch, max_nodes]
 *   m           dev in  int32 [batch], 0 <= m[b] <= max_nodes; m[b] = 0 skips sequence b
 *   tree_tokens dev out int32 [batch, max_nodes]: node u of sequence b at [b, u]; [b,0] = root
 * Ranking ties go to the lower token id. */
int draft_tree(clover_ctx *ctx, int32_t batch, const float *hid_acc, const int32_t *next_tok,
               const int32_t *m, int32_t *tree_tokens);

/* Verification pass (Sec. 2.1, tree attention).  Node u of sequence b is embedded, rotated to
 * position len[b] + depth(u), its K/V stored at cache slot len[b] + u, and it attends to all
 * cached slots and to the tree nodes on its own root path.  Lengths are not changed.
 *   tree_tokens dev in  int32 [batch, max_nodes]
 *   logits      dev out fp32 [batch, max_nodes, V]  (rows >= n_nodes untouched)
 *   hidden      dev out fp32 [batch, max_nodes, H]  last block's output, before the final norm
 * Fails with CLOVER_E_CAPACITY if a sequence could exceed max_seq. */
int verify_tree(clover_ctx *ctx, int32_t batch, const int32_t *tree_tokens, float *logits, float *hidden);

/* Greedy verification and cache compaction (Sec. 2.1; temperature 0).  Per sequence: start at
 * the root; while a child of the current node carries argmax(logits[node]) move to it.  The
 * visited nodes are accepted, the argmax at the last one is the bonus token.  K/V rows of the
 * accepted nodes are moved to slots len..len+m-1 in every target layer and len += m.
 *   m          dev out int32 [batch]              accepted rows (>= 1)
 *   acc_idx    dev out int32 [batch, max_nodes]   accepted node indices, first m valid
 *   new_tokens dev out int32 [batch, max_nodes]   tokens of accepted nodes 1..m-1, then the bonus
 *   hid_acc    dev out fp32  [batch, max_nodes, H] hidden rows of the accepted nodes
 *   next_tok   dev out int32 [batch, max_nodes]   = new_tokens (input of the next draft_tree)
 * argmax ties go to the lower token id. */
int accept_and_compact(clover_ctx *ctx, int32_t batch, const int32_t *tree_tokens, const float *logits,
                       const float *hidden, int32_t *m, int32_t *acc_idx, int32_t *new_tokens,
                       float *hid_acc, int32_t *next_tok);

/* Verification at a temperature > 0 (Table 1, temperature 1 rows) and cache compaction.  Per sequence, starting
 * at the root: with p = softmax(logits[node] / temperature) the children of the node are tried in index order and
 * child i is accepted when uniforms[b, node, i] < p(its token) / (1 - p-mass of the children already refused); the
 * walk then moves to it.  When none is accepted (or the node is a leaf) the next token is drawn from what is left
 * of p (the refused tokens removed) by inverting its cumulative sum in token-id order with uniforms[b, node, 16],
 * and the walk ends.  Every emitted token is then distributed exactly as the target model's own sample.
 *   temperature dev-independent scalar > 0
 *   uniforms    dev in fp32 [batch, max_nodes, 17], values in [0, 1): the caller's random numbers
 * Everything else as accept_and_compact. */
int accept_and_compact_sampled(clover_ctx *ctx, int32_t batch, const int32_t *tree_tokens, const float *logits,
                               const float *hidden, float temperature, const float *uniforms, int32_t *m,
                               int32_t *acc_idx, int32_t *new_tokens, float *hid_acc, int32_t *next_tok);

/* Prompt hand-off for a chain-shaped tree (the prefill phase of Sec. 1 run as chunks of plain
 * decoding): accept nodes 0..n_rows[b]-1 of sequence b unconditionally (n_rows[b] = 0 leaves
 * the sequence untouched).  The token after the last row is forced_next[b], or the target's
 * argmax there when forced_next[b] < 0.  Outputs as accept_and_compact.  The current tree must
 * be a chain.
 *   n_rows, forced_next  dev in int32 [batch] */
int clover_accept_forced(clover_ctx *ctx, int32_t batch, const int32_t *tree_tokens, const float *logits,
                         const float *hidden, const int32_t *n_rows, const int32_t *forced_next,
                         int32_t *m, int32_t *acc_idx, int32_t *new_tokens, float *hid_acc, int32_t *next_tok);

/* Prefill of one sequence (Sec. 1: the prefill phase that precedes the decode phase; Sec. 3.1, 3.3: the
 * Augmenting Block sees every earlier position paired with its follow-up token).  The n prompt tokens run through
 * the target in passes of up to prefill_rows rows -- every GEMM one weight pass over all rows of the pass, causal
 * attention over the cache and the pass's own rows, K/V written in place at slots len .. len+n-1 -- and the
 * LM head runs on the LAST row only.  The draft side pairs position i with token i+1 for i < n-1 (Attention
 * Decoder 1, then the Augmenting Block, causal over its own cache): n-1 rows appended there.  Afterwards
 * len[b] += n; the caller picks the first generated token g from logits_last (next_tok_out holds the
 * argmax, ties to the lower id), and a draft_tree call with m[b] = 1, hid_acc[b,0] = hid_last,
 * next_tok[b,0] = g completes the hand-off exactly as after accept_and_compact.
 *   b            sequence index, 0 <= b < max_batch
 *   tokens       dev in  int32 [n]
 *   n            number of prompt tokens, >= 1; len[b] + n <= max_seq
 *   logits_last  dev out fp32 [vocab]: target logits after the last prompt token
 *   hid_last     dev out fp32 [hidden]: its pre-final-norm hidden state
 *   next_tok_out dev out int32 [1], may be null
 * Enqueues on the context's stream; does not synchronise.  Errors: CLOVER_E_NULL, CLOVER_E_SHAPE (b, n),
 * CLOVER_E_CAPACITY (max_seq). */
int clover_prefill(clover_ctx *ctx, int32_t b, const int32_t *tokens, int32_t n, float *logits_last,
                   float *hid_last, int32_t *next_tok_out);

/* Paged KV caches (Sec. 1 names the large-batch serving regime; the paper does not describe a cache).  Both caches of
 * every layer are pools of max_batch * max_seq / 32 pages of 32 positions; position p of sequence b lives in page
 * table[b * (max_seq / 32) + p / 32].  The default is the identity table.  table_host: HOST int32
 * [max_batch * max_seq / 32], a permutation of the page numbers (CLOVER_E_SHAPE otherwise); NULL restores the identity.
 * Rows already cached are not moved: call it on empty sequences (after init or clover_reset).  Synchronises. */
int clover_set_page_table(clover_ctx *ctx, const int32_t *table_host);

/* Synchronise and read the target cache lengths into out_host[max_batch]; refreshes the
 * host-side bound used by the capacity check.  Returns CLOVER_E_STATE if a device guard fired. */
int clover_seq_len(clover_ctx *ctx, int32_t *out_host);

/* Test helper (synchronises): copy cache rows [slot0, slot0+n_slots) of one layer and sequence
 * to host as fp32 [n_slots, n_kv, d].  stack 0 = target, 1 = augmenting block. */
int clover_read_kv(clover_ctx *ctx, int32_t stack, int32_t layer, int32_t b, int32_t slot0, int32_t n_slots,
                   float *k_out_host, float *v_out_host);

/* Test helper (synchronises): the mirror of clover_read_kv.  Writes n_slots cache rows of one layer and sequence
 * from host fp32 [n_slots, n_kv, d] (stored in the cache's own format).  Lengths are not changed. */
int clover_write_kv(clover_ctx *ctx, int32_t stack, int32_t layer, int32_t b, int32_t slot0, int32_t n_slots,
                    const float *k_in_host, const float *v_in_host);

/* Test helper (synchronises): declare the first len_host[b] slots of the target cache and the first
 * aug_len_host[b] slots of the augmenting block's cache of every sequence valid (after a prompt of L tokens the
 * target holds L rows and the block L - 1: its last row arrives with the next draft_tree).  HOST int32 [max_batch]. */
int clover_set_seq_len(clover_ctx *ctx, const int32_t *len_host, const int32_t *aug_len_host);

/* Test helper: while dev_out is non-null every draft_tree also copies the draft logits it ranks (Sec. 3.2: the
 * shared LM head after FC_j) to dev_out, fp32: the rows of depth j start at batch * (number of internal nodes
 * shallower than j) * V, row (b, r) of that depth at ((b * n_j) + r) * V, r-th internal node of the depth in
 * index order (dynamic tree: r-th expanded candidate of the depth, best first).  Depths that would not fit
 * capacity_floats are skipped.  null switches it off. */
int clover_capture_draft_logits(clover_ctx *ctx, float *dev_out, size_t capacity_floats);

/* Per-kernel-class timing with HIP events on the library's stream.  While enabled, every launch
 * is bracketed by two events.  collect synchronises, adds up the
 * elapsed milliseconds and launch counts per class since the last collect, and clears them.
 * Class names: clover_kernel_class_name(i), i < clover_kernel_class_count(). */
int clover_profile_enable(clover_ctx *ctx, int32_t on);
int clover_profile_collect(clover_ctx *ctx, double *ms_by_class, int64_t *launches_by_class, int32_t n_classes);
int clover_kernel_class_count(void);
const char *clover_kernel_class_name(int32_t cls);

/* Which kernels this context runs: bit 0 = MFMA path (bf16 model), bit 1 = MFMA tree attention.
 * Negative: error code. */
int clover_path_info(clover_ctx *ctx);

/* Message of the last error on this context ("" if none); valid until the next call. */
const char *clover_last_error(clover_ctx *ctx);
/* Message of the last error of a call that had no context (init, workspace_bytes). */
const char *clover_last_global_error(void);

/* ---- single operators, exported for unit tests and kernel benchmarks -------------------- */

/* Y[M,N] (fp32, leading dimension ldy) = X[M,K] (fp32, ld = K) * W[N,K]^T, W in `dtype`.
 * path 0 = generic fp32-ALU kernel, 1 = MFMA weight-streaming kernels (bf16 only; W is first copied
 * into `scratch` in the library's fragment-major layout), 2 = as 1 but reusing the copy a previous
 * path-1 call with the same W and scratch left behind (times the GEMM alone); 3 = full-K panel
 * kernel (bf16, M <= 64, K % 256 == 0, N % 16 == 0, ldy % 4 == 0), 4 = as 3 reusing the copy;
 * 5 = the panel kernel over ranges of K (narrow N with long K, e.g. 4096 x 14336; CLOVER_E_SHAPE
 * where the launcher would not pick it) followed by the sum of the ranges, 6 = as 5 reusing the copy;
 * 7 = the tiled kernel for many rows (M <= 256, K % 64 == 0, N % 16 == 0) over ranges of K, then their sum.
 * `scratch` dev, >= clover_op_gemm_scratch_bytes(M,N,K).  Stream as given. */
size_t clover_op_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K);
int clover_op_gemm(int32_t path, int32_t dtype, const float *X, const void *W, float *Y, int32_t ldy,
                   int32_t M, int32_t N, int32_t K, void *scratch, size_t scratch_bytes, void *hip_stream);

/* clover_op_gemm for callers that cannot allocate device memory (code under HIP-graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the scratch is a fixed device array inside the library, one per GPU,
 * CLOVER_STATIC_SCRATCH_BYTES long, held until the process ends.  Same arguments and results as clover_op_gemm
 * for path 0, 1, 3 or 5 (the weight copy is always made: the array keeps only the LAST call's contents).
 * CLOVER_E_CAPACITY when clover_op_gemm_scratch_bytes(M, N, K) exceeds the array; CLOVER_E_SHAPE for the
 * copy-reusing paths.  Allocates nothing.  All calls on one GPU share the array: calls that overlap on one
 * GPU (different streams or threads) race. */
#define CLOVER_STATIC_SCRATCH_BYTES (32u << 20)
int clover_op_gemm_static(int32_t path, int32_t dtype, const float *X, const void *W, float *Y, int32_t ldy,
                          int32_t M, int32_t N, int32_t K, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CLOVER_H_ */
