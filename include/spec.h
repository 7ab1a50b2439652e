/*
 * libspec: batch-1 speculative decoding with a dynamic draft tree on one
 * MI355X (gfx950).  C ABI; no torch types; every pointer says host or device.
 *
 * The calls follow the paper's three-step statement of speculative sampling
 * (Sec. 2, Preliminary): the draft model proposes (spec_draft_tree), the target
 * evaluates all proposals in one parallel forward (spec_verify), and a lossless
 * acceptance rule keeps a prefix (spec_accept).  The draft model is the EAGLE
 * design of Sec. 2: one decoder layer fed the target's last hidden state of the
 * previous position concatenated with the current token's embedding, sharing
 * the target's embedding and LM head.  The tree is the dynamic tree whose two
 * knobs are `depth` (expansion phase) and `number of tokens` (rerank phase)
 * (appendix, Drafting Hyper-Parameters; 60 tokens / depth 6 in Sec. 4.1).
 *
 * Threading: a context is not thread-safe; all work of a context is enqueued on
 * the one HIP stream given at creation.  Calls that return host data wait for
 * the stream.  No call allocates device memory: the caller hands over one
 * workspace of spec_workspace_bytes() bytes at creation.
 *
 * Errors: every int-returning call returns SPEC_OK (0) or a negative code and
 * never aborts or throws; spec_last_error() gives a message for the last
 * failure on that context.
 */
#ifndef SPEC_H_
#define SPEC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPEC_OK      0
#define SPEC_EINVAL -1   /* NULL pointer, bad configuration, malformed tree            */
#define SPEC_ESTATE -2   /* call out of order (see the state machine below)            */
#define SPEC_ECAP   -3   /* KV capacity (max_seq) or workspace too small               */
#define SPEC_EHIP   -4   /* a HIP runtime call failed; message in spec_last_error()    */

#define SPEC_DTYPE_FP32 0
#define SPEC_DTYPE_BF16 1

#define SPEC_MAX_DEPTH  15   /* largest tree depth D accepted                          */
#define SPEC_MAX_TOPK   16   /* largest K accepted                                     */
#define SPEC_MAX_NODES 128   /* largest N (rows of one verify forward, root included)  */

typedef struct spec_ctx spec_ctx;   /* opaque; owned by the library */

/* Plain data, caller-owned, copied at spec_create. */
typedef struct spec_config {
  int32_t  n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float    rope_theta;      /* rotary base (1e4 LLaMA2, 5e5 LLaMA3)                          */
  float    rms_eps;         /* RMSNorm epsilon                                               */
  int32_t  dtype;           /* SPEC_DTYPE_*: storage type of weights, activations, KV cache  */
  int32_t  max_seq;         /* KV capacity in tokens; needs prompt + generated + tree_total  */
  int32_t  tree_depth;      /* D: draft forwards per cycle = longest root-to-leaf path       */
  int32_t  tree_topk;       /* K: children kept per expanded node, nodes expanded per depth  */
  int32_t  tree_total;      /* N: rows verified per cycle, root included (1 = plain decode)  */
  float    temperature;     /* 0: greedy acceptance; > 0: rejection sampling at that T       */
  uint64_t seed;            /* used only when temperature > 0                                */
  int32_t  device;          /* HIP device ordinal                                            */
  void    *stream;          /* hipStream_t, BORROWED; NULL = the default stream              */
  void    *workspace;       /* DEVICE pointer, BORROWED, 256-byte aligned                    */
  uint64_t workspace_bytes; /* >= spec_workspace_bytes(cfg)                                  */
} spec_config;

/* DEVICE pointers, BORROWED for the life of the context, never written.
 * Projection matrices ([out, in], shapes in the comments) are in the library's
 * PACKED layout, produced once at load time by spec_pack_weight() (the gate and
 * up projections of the SwiGLU block together, by spec_pack_gate_up()); the
 * embedding table stays row-major (it is gathered by row); norm weights are
 * [d_model] vectors.  All in the configured dtype. */
typedef struct spec_layer_weights {
  const void *attn_norm;
  const void *wq, *wk, *wv;   /* [n_q_heads*head_dim, d], [n_kv_heads*head_dim, d] x2 */
  const void *wo;             /* [d, n_q_heads*head_dim]                              */
  const void *ffn_norm;
  const void *w_gate_up;      /* gate and up, [d_ffn, d] each, as ONE packed matrix (spec_pack_gate_up) */
  const void *w_down;         /* [d, d_ffn]                                           */
} spec_layer_weights;

typedef struct spec_weights {
  const void *embed;                 /* [vocab, d] row-major; shared by target and draft (Sec. 2) */
  const void *lm_head;               /* [vocab, d] packed; shared by target and draft     */
  const void *final_norm;            /* [d]; its output is the feature given to the draft */
  const spec_layer_weights *layers;  /* HOST array of n_layers entries (device pointers)  */
  const void *draft_fc;              /* [d, 2d] packed: concat(feature, embedding) -> d, no bias */
  spec_layer_weights draft_layer;    /* the draft's single decoder layer                  */
} spec_weights;

/* HOST memory, caller-allocated, each array with room for tree_total entries.
 * Node 0 is the root (the pending token); parents precede their children. */
typedef struct spec_tree {
  int32_t  n_nodes;
  int32_t *token;    /* token id of each node                                    */
  int32_t *parent;   /* node index of the parent; parent[0] = -1                 */
  int32_t *depth;    /* depth[0] = 0; depth[j] = depth[parent[j]] + 1 <= D       */
  float   *score;    /* cumulative draft log-probability; score[0] = 0; may be NULL on input */
} spec_tree;

/* Packed layout.  The weight-streaming kernels read 16-byte pieces in the order
 * the matrix cores consume them, so that one wavefront-wide load covers 1 KiB of
 * consecutive bytes.  A row-major [rows, in] matrix is cut into tiles of 32 rows
 * x 256 bytes of k; tiles of one 32-row block follow each other along k; inside
 * a tile piece (j = 0..7, lane = 0..63) is at byte j*1024 + lane*16 and holds row
 * lane%32, k-bytes (lane/32)*128 + j*16 .. +16 of the tile.  Rows and k are
 * zero-padded to whole tiles.
 *   spec_packed_bytes : size of the packed form (host-only computation; 0 if bad).
 *   spec_pack_weight  : out-of-place repack, DEVICE src (row-major) -> DEVICE dst
 *                       (256-byte aligned, spec_packed_bytes large), enqueued on
 *                       `stream`; src and dst must not overlap. */
uint64_t spec_packed_bytes(int32_t dtype, int32_t rows, int32_t in);
int spec_pack_weight(int32_t dtype, const void *src, int32_t rows, int32_t in, void *dst, void *stream);

/* The gate and up projections of a SwiGLU feed-forward block (the target LLMs of
 * Sec. 4.1 are LLaMA models: act = silu(x . w_gate) * (x . w_up)) as one packed
 * matrix of 32 * ceil(rows / 16) rows: 32-row block b holds the gate rows
 * 16 b .. 16 b + 15 followed by the up rows 16 b .. 16 b + 15 (zero rows past the
 * last one), so that the wavefront that streams a block owns both sums of a
 * column and applies the activation itself.  gate, up: DEVICE, row-major
 * [rows, in]; dst: DEVICE, 256-byte aligned, spec_packed_gate_up_bytes large; no
 * overlap; enqueued on `stream`.  Same argument checks and errors as above. */
uint64_t spec_packed_gate_up_bytes(int32_t dtype, int32_t rows, int32_t in);
int spec_pack_gate_up(int32_t dtype, const void *gate, const void *up, int32_t rows, int32_t in, void *dst, void *stream);

/* Bytes of device workspace a context with this configuration needs (0 if the
 * configuration is invalid).  Host-only computation. */
uint64_t spec_workspace_bytes(const spec_config *cfg);

/* State machine: create -> CREATED; prefill -> READY; draft_tree -> DRAFTED;
 * verify -> VERIFIED; accept -> READY.  Other orders return SPEC_ESTATE. */

/* Sets up the two models the method runs (Sec. 2: a target LLM and a draft
 * model that takes the target's last hidden state together with the token
 * embedding and shares the target's embedding and LM head; Sec. 4.1: LLaMA
 * targets, tree of `tree_depth` / `tree_total`).  Validates the configuration,
 * carves the workspace, keeps copies of cfg and of the weight pointer table.
 * *out receives the context.  Errors: SPEC_EINVAL (bad configuration, NULL
 * weight pointer, workspace NULL or misaligned), SPEC_ECAP (workspace too
 * small), SPEC_EHIP; the message is in spec_last_error(NULL). */
int spec_create(const spec_config *cfg, const spec_weights *w, spec_ctx **out);

/* Produces the state speculation starts from (Sec. 2: drafting begins at a
 * given timestep t and needs the target's hidden state of step t-1 and the
 * token of step t): the target runs over the prompt, which yields its feature
 * at the last position and the first generated token, and the draft model runs
 * over the prompt's (feature of position i-1, token i) pairs so that its own
 * cache covers the context.
 * Runs the target over the prompt (HOST int32 array, 1 <= n_prompt, n_prompt +
 * tree_total <= max_seq), fills both KV caches, and chooses the first token
 * from the last row (argmax at T = 0, a sample at T > 0).  That token is
 * returned in *first_token (HOST) and becomes the pending root. */
int spec_prefill(spec_ctx *ctx, const int32_t *prompt, int32_t n_prompt, int32_t *first_token);

/* Draft phase of one cycle: D draft forwards expand the tree, the pool is
 * reranked by cumulative draft log-probability and the best N-1 nodes plus the
 * root are written to *out (HOST arrays as described at spec_tree).  The
 * caller may edit the tree before spec_verify (tests forge trees this way). */
int spec_draft_tree(spec_ctx *ctx, spec_tree *out);

/* One target forward over all nodes of `tree` with tree attention: row j is at
 * position n + depth[j] and attends to the n cached tokens and to the nodes on
 * its root-to-j path.  Validates the tree (node 0 carries the pending root,
 * parents precede children, depths consistent and <= SPEC_MAX_DEPTH, tokens in
 * range, 1 <= n_nodes <= tree_total).  Keeps logits [n_nodes, vocab] (fp32)
 * and features [n_nodes, d] on the device for spec_accept and the getters. */
int spec_verify(spec_ctx *ctx, const spec_tree *tree);

/* Acceptance, KV compaction and hand-off.  T = 0: follows the child carrying
 * the target's argmax while there is one.  T > 0: multi-round rejection
 * sampling over each node's children in node order, the bonus token drawn from
 * the residual distribution.  Writes the accepted draft tokens followed by the
 * bonus token to out_tokens (HOST, capacity SPEC_MAX_DEPTH + 1) and their
 * count (1 .. D+1) to *n_out.  The bonus token becomes the next pending root.
 * `tree` must be the tree passed to spec_verify. */
int spec_accept(spec_ctx *ctx, const spec_tree *tree, int32_t *out_tokens, int32_t *n_out);

/* Frees host state.  The workspace stays the caller's.  NULL is a no-op. */
void spec_destroy(spec_ctx *ctx);

/* ---- inspection (not on the hot path; each waits for the stream) ---------- */

/* Tokens committed to the target KV cache so far (the pending root excluded). */
int spec_committed(const spec_ctx *ctx);

/* Copies logits [n_nodes, vocab] of the last spec_verify to HOST `dst`
 * (capacity in floats); returns the number of floats written or an error. */
int64_t spec_get_logits(spec_ctx *ctx, float *dst, int64_t cap);

/* Copies features [n_nodes, d_model] of the last spec_verify, widened to fp32. */
int64_t spec_get_features(spec_ctx *ctx, float *dst, int64_t cap);

/* Copies rows [0, n_rows) of one layer's key and value cache, widened to fp32,
 * each [n_rows, n_kv_heads*head_dim].  which = 0: target layer `layer`;
 * which = 1: the draft layer (`layer` ignored; draft row i belongs to token i+1). */
int64_t spec_get_kv(spec_ctx *ctx, int32_t which, int32_t layer, int32_t n_rows, float *k_dst, float *v_dst, int64_t cap);

/* The verify forward, and the draft expansion steps with the rerank, are each
 * captured into a HIP graph and replayed every cycle (their launch arguments
 * are fixed or device-resident), which removes most of the per-kernel launch cost.
 * A graph's attention launches are sized for the context rounded up to a multiple
 * of 256 positions; it is captured again (about a millisecond) when the context
 * outgrows that, so the cycle time does not depend on max_seq.  Graphs need a non-default stream; with stream == NULL
 * or after spec_set_graphs(ctx, 0) every kernel is launched individually.  Both
 * paths run the same kernels on the same data and give identical results. */
int spec_set_graphs(spec_ctx *ctx, int32_t enable);

/* Static draft trees (the tree of the comparison systems of Sec. 4.1: EAGLE's
 * fixed shape, or a chain = conventional speculative sampling, Sec. 2) instead
 * of the dynamic tree of the configuration.  The shape has n_nodes <=
 * cfg.tree_total nodes, node 0 the root, nodes in order of depth, parents
 * before children (HOST arrays parent[], rank[] of n_nodes ints, parent[0] =
 * -1).  rank[i] says which of its parent's proposals node i is: the rank-th
 * best token of the draft distribution at the parent, or, with sampled != 0
 * (needs cfg.temperature > 0), the rank-th of the tokens DRAWN from it without
 * replacement.  The children of a node must be listed in increasing rank; with
 * sampled != 0 they must carry the ranks 0, 1, ..., c-1 without gaps (the ratio
 * rule treats the j-th listed child as the j-th draw: a child whose earlier
 * draws are not in the tree would not follow the distribution the rule
 * divides by, and the output would lose the target distribution); shapes with
 * gaps are for deterministic children only.  A
 * depth may have at most 16 nodes with children; the nodes with children
 * (root excluded) may not exceed cfg.tree_depth * cfg.tree_topk (the draft
 * scratch the workspace was sized for).  spec_draft_tree then drafts this shape
 * (one draft forward per depth over the nodes that have children; scores are
 * cumulative log-probabilities for deterministic children and 0 for sampled
 * ones) and spec_accept uses, for sampled children, the ratio rule min(1, p/q)
 * with residual max(p - q, 0) against the draft rows kept while drafting: the
 * tree must then be passed to spec_verify / spec_accept as drafted.  With
 * deterministic children the acceptance is the one of the dynamic tree.
 * buffer: spec_static_tree_bytes(...) bytes of DEVICE memory, 256-byte aligned,
 * owned by the caller and borrowed until the context is destroyed or another
 * shape is set (0 from spec_static_tree_bytes = shape not accepted).  Call it
 * between cycles (after spec_create / spec_prefill / spec_accept); n_nodes = 0
 * returns to the dynamic tree.  The static path launches its kernels
 * individually (no graph replay).  Errors: SPEC_EINVAL (malformed shape, small
 * buffer), SPEC_ECAP (shape beyond the configured capacity), SPEC_ESTATE. */
uint64_t spec_static_tree_bytes(const spec_config *cfg, int32_t n_nodes, const int32_t *parent, const int32_t *rank, int32_t sampled);
int spec_set_static_tree(spec_ctx *ctx, int32_t n_nodes, const int32_t *parent, const int32_t *rank, int32_t sampled, void *buffer,
                         uint64_t buffer_bytes);

/* Per-phase and per-kernel-class GPU time accounting with HIP events on the
 * context's stream.  level 0: off; 1: one event pair per call (draft, verify,
 * accept); 2: additionally one pair around every weight-streaming GEMM launch
 * (perturbs the pipeline; use in a separate pass).  spec_get_profile fills
 * HOST arrays of 8 doubles / 8 int64 and resets the counters:
 *   [0] draft ms   [1] verify ms   [2] accept ms   [3] prefill ms
 *   [4] GEMM ms inside verify      [5] GEMM ms inside draft
 *   [6] level 2 calibration: one event pair per verify with nothing between its two records, taken
 *       while the stream is busy (what the event mechanism itself adds to every interval of [4], [5])
 *   [7] reserved
 * counts[i] = number of intervals summed into ms[i]. */
int spec_set_profile(spec_ctx *ctx, int32_t level);
int spec_get_profile(spec_ctx *ctx, double *ms, int64_t *counts);

/* Message for the last failure on this context ("" if none); valid until the
 * next call on the context.  With ctx == NULL: the last spec_create failure
 * of the calling thread. */
const char *spec_last_error(const spec_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_H_ */
