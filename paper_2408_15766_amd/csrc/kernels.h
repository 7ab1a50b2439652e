// Host-callable launchers of the gfx950 kernels.  All pointers are device
// pointers unless a comment says otherwise; dtype 0 = fp32, 1 = bf16 storage.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spec {

constexpr int kMaxDepth = 15;          // longest root-to-node path handled by the tail of the attention
constexpr int kAncStride = kMaxDepth + 1;
constexpr int kMaxTopK = 16;
constexpr int kMaxNodes = 128;
#ifndef SPEC_ATTN_PART
#define SPEC_ATTN_PART 128
#endif
constexpr int kAttnPart = SPEC_ATTN_PART;   // key positions per attention partial (fixed absolute boundaries) ...
#ifndef SPEC_ATTN_NEAR
#define SPEC_ATTN_NEAR 1024
#endif
#ifndef SPEC_ATTN_FAR_PART
#define SPEC_ATTN_FAR_PART 256
#endif
constexpr int kAttnNear = SPEC_ATTN_NEAR;         // ... for key positions below this;
constexpr int kAttnFarPart = SPEC_ATTN_FAR_PART;  // beyond it a partial covers this many positions
static_assert(kAttnNear % kAttnPart == 0 && kAttnFarPart % 32 == 0 && kAttnPart % 32 == 0, "parts are whole 32-key blocks");
// First key position of partial t, and the number of partials that intersect [0, keys).  The boundaries are
// absolute (they depend on nothing but t), so a row's partition is the same in every launch.
__host__ __device__ inline int attn_part_begin(int t) {
  return t <= kAttnNear / kAttnPart ? t * kAttnPart : kAttnNear + (t - kAttnNear / kAttnPart) * kAttnFarPart;
}
__host__ __device__ inline int attn_parts_covering(int keys) {
  return keys <= kAttnNear ? (keys + kAttnPart - 1) / kAttnPart : kAttnNear / kAttnPart + (keys - kAttnNear + kAttnFarPart - 1) / kAttnFarPart;
}
constexpr int kTopkSlice = 4096;       // vocabulary entries per first-stage top-k workgroup

// ---- gemm.hip --------------------------------------------------------------------------------
struct GemmArgs {
  const void *x;  int ldx;  int m;      // X [m, in], row stride ldx elements; m > 128 runs as tiles of 128 rows (prefill)
  int in;                               // K, a multiple of 16 bytes / element size
  const void *seg_w[3];                 // up to three PACKED weight matrices ([rows, in] before packing) sharing X (e.g. q, k, v)
  int seg_rows[3];
  int seg_blocks[3];                    // ceil(rows / 32)
  int seg_col0[3];                      // first output column of the segment
  int nseg, total_blocks;
  float *part;  int ldp;  int m_pad;    // partial sums [n_split][m_pad][ldp], fp32
  int n_split;                          // K is cut into n_split ranges of whole slabs, balanced to one slab
  // SwiGLU mode (act != nullptr): one segment, the packed gate/up matrix; seg_rows[0] = columns of act,
  // seg_blocks[0] = ceil(columns / 16), n_split = 1.  The wave that streams a block writes
  // act[i][c] = silu(gate) * up in the storage type instead of partial sums.
  void *act;
  int m_tiles, grid_x;                  // set by launch_gemm: 128-row tiles of X, workgroups per tile and split
  int blk_per_wg, blk_per_wave;         // set by launch_gemm: wave w of workgroup x streams block x * blk_per_wg + w * blk_per_wave
};
hipError_t launch_gemm(int dtype, const GemmArgs &a, hipStream_t st);
hipError_t gemm_init();                 // one-time kernel attributes; call outside any stream capture
int gemm_k_per_slab(int dtype);
int gemm_k_per_iter(int dtype);
// Packed layout of a row-major [rows, in] matrix (see gemm.hip): size in bytes, and the out-of-place repack.
size_t packed_weight_bytes(int dtype, int rows, int in);
hipError_t launch_pack_weight(int dtype, const void *src, int rows, int in, void *dst, hipStream_t st);
// gate and up ([rows, in] each, row-major) as one packed matrix: 16 gate rows, then the 16 up rows of the same columns, per block
size_t packed_gate_up_bytes(int dtype, int rows, int in);
hipError_t launch_pack_gate_up(int dtype, const void *gate, const void *up, int rows, int in, void *dst, hipStream_t st);

// ---- rowops.hip ------------------------------------------------------------------------------
// h[i] = embed[token[i]] (fp32);  x[i] = rmsnorm(h[i]) * w  in the storage type.
// With `table` set, the launch also fills the rotary table of its rows: (cos, sin) of pos[i] * theta^(-2j/hd) for j < hd/2,
// the angles formed in double precision.
hipError_t launch_embed_norm(int dtype, const void *embed, const int *token, int rows, int d, const void *norm_w,
                             float eps, float *h, void *x, hipStream_t st, const int *pos = nullptr, int head_dim = 0,
                             float theta = 0.f, float2 *table = nullptr);
// xcat[i] = [feat[src_row[i]] ; embed[token[i]]]  ([rows, 2d], storage type).  src_row == nullptr: identity.
hipError_t launch_concat_feat_embed(int dtype, const void *feat, const int *src_row, const void *embed,
                                    const int *token, int rows, int d, void *xcat, hipStream_t st, const int *pos = nullptr,
                                    int head_dim = 0, float theta = 0.f, float2 *table = nullptr);
// h[i] = (residual ? h[i] : 0) + sum_s part[s][i][:d];  x[i] = norm_w ? rmsnorm(h[i]) * norm_w : h[i].
hipError_t launch_reduce_add_norm(int dtype, const float *part, int n_split, int m_pad, int ldp, int rows, int d,
                                  int residual, const void *norm_w, float eps, float *h, void *x, hipStream_t st);
// Sums the QKV partials, rotates q and k by the row's position, writes q [rows, hq*hd] (always fp32) and
// the row's key/value (storage type) into cache slot slot[i].  Cache layout [max_seq][hkv*hd].
hipError_t launch_reduce_rope_kv(int dtype, const float *part, int n_split, int m_pad, int ldp, int rows, int hq, int hkv,
                                 int hd, const float2 *rope, const int *slot, void *q, void *kcache, void *vcache,
                                 hipStream_t st);
// act[i][c] = silu(g) * u with g = sum_s part[s][i][c], u = sum_s part[s][i][f + c].
hipError_t launch_reduce_swiglu(int dtype, const float *part, int n_split, int m_pad, int ldp, int rows, int f, void *act,
                                hipStream_t st);

// Row i of a causal chain starting at cache slot `base`: slot = base + i, position = slot + pos_offset,
// depth = i (its tail is the chain itself).
hipError_t launch_chain_rows(int base, int rows, int pos_offset, int *pos, int *slot, int *depth, hipStream_t st);

// ---- attention.hip ---------------------------------------------------------------------------
// Row i sits at key position base + depth[i] and attends to positions 0 .. base + depth[i]:
// position q < base lives in cache slot q; position q >= base lives in slot base + anc[i][q - base]
// (anc == nullptr: slot q, i.e. a causal chain).  Output [rows, hq*hd] in the storage type.
struct AttnArgs {
  const void *q;                        // fp32 [rows, hq*hd]
  const void *kcache; const void *vcache;
  int rows, hq, hkv, hd, base;
  const int *base_ptr;                  // if not null: the base is read from here (device) and `base` is ignored
  const int *depth;                     // [rows]
  const int *anc;                       // [rows][kAncStride] or nullptr
  float scale;
  float *part;                          // scratch: [rows][hq][max_parts][hd + 2]; max_parts >= attn_parts_covering(max_pos + 1) + 1
  int max_parts;
  void *out;
  int tail_only, bulk_keys, bulk_blocks, bulk_parts, q_groups;   // set by launch_attention (hybrid matrix-core / vector split)
};
hipError_t launch_attention(int dtype, const AttnArgs &a, int max_pos, hipStream_t st);

// ---- hca.hip ---------------------------------------------------------------------------------
// Training attention over J = n_streams key/value streams: query t (from the newest stream) uses, for the key
// position t - o, stream J-1-o if o <= J-2 and stream 0 otherwise.  bf16 storage.
// q, out: [batch, seq, hq, hd]; k[m], v[m]: [batch, seq, hkv, hd].
constexpr int kMaxStreams = 8;
struct HcaArgs {
  const void *q;
  const void *k[kMaxStreams];
  const void *v[kMaxStreams];
  void *out;
  int n_streams, batch, seq, hq, hkv, hd;
  float scale_log2e;                    // 1/sqrt(hd) * log2(e)
};
hipError_t launch_hca_attention(const HcaArgs &a, hipStream_t st);

// ---- distill.hip -----------------------------------------------------------------------------
// Per position, from fp32 logit rows zq (target) and zp (draft), row stride ldz:
//   loss_topk = - sum over the k tokens of largest zq of softmax(zq) * log_softmax(zp)   (lower token id on ties)
//   loss_ce   = the same sum over the whole vocabulary.
// scratch: topk_loss_scratch_floats(rows, vocab, k) floats.  rows <= 65535, k <= kLossMaxK, ceil(vocab/4096)*k <= 4096.
constexpr int kLossMaxK = 128;
size_t topk_loss_scratch_floats(int rows, int vocab, int k);
hipError_t launch_topk_loss_rows(const float *zq, const float *zp, int ldz, int rows, int vocab, int k, float *scratch,
                                 float *loss_topk, float *loss_ce, hipStream_t st);
// out[0] = sum of loss_topk[0..rows), out[1] = sum of loss_ce[0..rows), in a fixed order.
hipError_t launch_loss_total(const float *loss_topk, const float *loss_ce, int rows, float *out, hipStream_t st);

// ---- select.hip ------------------------------------------------------------------------------
// argmax over each row of logits [rows, vocab] (ld = vocab), lower index on ties.  Per-slice results go to
// part_val / part_idx [rows][argmax_slices(vocab)]; if `out` is not null a second kernel merges them into
// out[row] (the greedy acceptance merges the slices itself).
int argmax_slices(int vocab);
hipError_t launch_rows_argmax(const float *logits, int rows, int vocab, float *part_val, int *part_idx, int *out,
                              hipStream_t st);
// with x = logit / temp: part[row][slice] = {max x, sum exp(x - max x)} over slices of kTopkSlice entries
// (argmax_slices(vocab) slices per row); the sampling acceptance merges the slices of the rows it visits.
hipError_t launch_rows_softmax_stats(const float *logits, int rows, int vocab, float temp, float2 *part, hipStream_t st);
// per row: top-k (token, log-softmax) pairs, best first, lower token on ties.  Two stages through scratch.
hipError_t launch_rows_topk_logprob(const float *logits, int rows, int vocab, int k, float *sc_val, int *sc_idx,
                                    float2 *sc_stat, int *top_tok, float *top_lp, hipStream_t st);

// Device-resident state of the draft tree expansion.
struct DraftState {
  int *pool_tok, *pool_par, *pool_dep; float *pool_sc;   // candidate pool
  int *n_pool;                                           // [1]
  int *front_pool;                                       // [K] pool index of each frontier row
  int *front_tok;                                        // [K] token of each frontier row
  int *front_src;                                        // [K] row of the previous step's output holding the parent feature
  int *front_depth;                                      // [K] depth argument for the attention (tail length - 1)
  int *front_anc;                                        // [K][kAncStride] scratch-slot offsets of the ancestors and itself
  int *front_slot;                                       // [K] cache slot the row's key/value go to
  int *front_pos;                                        // [K] rotary position
};
// n_draft (device int): committed draft-cache entries = committed tokens; scratch slots start there.
// After the root step: pool <- top-k of the root row; frontier <- those k nodes.
hipError_t launch_pool_init(const DraftState &s, const int *top_tok, const float *top_lp, int k, int root_row,
                            const int *n_draft, hipStream_t st);
// After expansion step t (frontier rows = k nodes of depth t-1): append k*k children; if `select_next`,
// choose the k best children as the next frontier and derive its attention tables.
hipError_t launch_pool_expand(const DraftState &s, const int *top_tok, const float *top_lp, int k, int step,
                              const int *n_draft, int select_next, hipStream_t st);
// Rerank: best (total-1) pool entries by score (ties: lower pool index), kept in pool order.
// tree_* arrays have room for `total` nodes; node 0 = root.
hipError_t launch_rerank(const DraftState &s, int total, const int *root_tok, int *tree_n, int *tree_tok, int *tree_par,
                         int *tree_dep, float *tree_sc, hipStream_t st);

struct AcceptResult {                   // lives on the device; copied to the host after acceptance
  int n_acc;                            // m: accepted draft nodes
  int node[kMaxDepth + 1];              // node[0] = 0 (root), node[d] = accepted node of depth d
  int token[kMaxDepth + 1];             // m accepted tokens then the bonus token
};
hipError_t launch_accept_greedy(const float *amax_val, const int *amax_idx, int n_slices, const int *tree_tok,
                                const int *tree_par, int n_nodes, AcceptResult *res, hipStream_t st);
hipError_t launch_accept_sample(const float *logits, int vocab, const float2 *stat_part, float temp, const int *tree_tok,
                                const int *tree_par, int n_nodes, uint64_t seed, uint32_t cycle, AcceptResult *res,
                                hipStream_t st);
// The ratio rule for sampled children: p_logits[i], q_logits[i] are the target / draft logit rows AT node i (fp32,
// row stride vocab); children are tried in node order; work: vocab floats of scratch.
// qrow_of (nullable): node -> row of q_logits holding the draft's logits at that node (-1: the node has no children).
hipError_t launch_accept_qratio(const float *p_logits, const float *q_logits, const int *qrow_of, int vocab, float temp,
                                const int *tree_tok, const int *tree_par, int n_nodes, uint64_t seed, uint32_t cycle, float *work,
                                AcceptResult *res, hipStream_t st);

// A static tree shape on the device (node 0 = root, nodes in order of depth, parents before children).
struct StaticTables {
  int n_nodes;
  const int *parent, *rank, *depth;     // [n_nodes]; rank = which of the parent's proposals the node is
  const int *erow;                      // [n_nodes] row of the node in its depth's draft forward, -1 if it has no children
  const int *eoff;                      // [n_nodes] draft scratch slot offset of such a node (depth >= 1), -1 otherwise
};
// Fills the tree arrays of the nodes of depth d from the proposals of depth d-1 and prepares the next forward's rows.
hipError_t launch_static_step(const StaticTables &tb, int d, const int *top_tok, const float *top_lp, int root_row,
                              const int *root_tok, const int *n_draft, int with_scores, const DraftState &s, int *t_n, int *t_tok,
                              int *t_par, int *t_dep, float *t_sc, hipStream_t st);
// z[r] = logits[r] / temp + Gumbel noise of stream (seed, cycle, node_stream[r]); rows <= kMaxTopK.
hipError_t launch_perturb_rows(const float *logits, int rows, int vocab, float temp, uint64_t seed, uint32_t cycle,
                               const int *node_stream, float *z, hipStream_t st);
// m <= kMaxTopK tokens drawn without replacement from softmax(logits / temp), in draw order (Gumbel-top-m).
// z: vocab floats; sc_val / sc_idx / sc_stat / top_tok / top_lp: the scratch of launch_rows_topk_logprob for one row.
hipError_t launch_sample_children(const float *logits, int vocab, float temp, int m, uint64_t seed, uint32_t cycle, uint32_t node,
                                  float *z, float *sc_val, int *sc_idx, float2 *sc_stat, int *top_tok, float *top_lp, int *out,
                                  hipStream_t st);
// Sample one token from softmax(logits / temp) by Gumbel-max with stream (seed, cycle, node).
hipError_t launch_sample_row(const float *logits, int vocab, float temp, uint64_t seed, uint32_t cycle, uint32_t node,
                             int *out, hipStream_t st);
// Commit: in every layer move key/value of accepted node d from slot n + node[d] to slot n + d; gather
// the features of root + accepted rows and the tokens for the next draft root step; *root_tok <- bonus;
// *n_committed (device) += 1 + accepted.
hipError_t launch_commit(int dtype, const AcceptResult *res, void *kv_base, size_t layer_stride, size_t kv_stride,
                         int n_layers, int row_elems, int n, const void *feat, int d, void *pend_feat, int *pend_tok,
                         int *root_tok, int *n_committed, hipStream_t st);

}  // namespace spec
