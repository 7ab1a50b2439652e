/*
 * libspec, kernel-level entry points: the individual gfx950 kernels of the
 * decode path (and the acceptance rule for sampled draft tokens, which the
 * decode loop of spec.h does not use), callable on caller-provided DEVICE buffers.  They exist so that
 * each kernel can be checked against the CPU oracle and timed in isolation;
 * the decode loop itself goes through spec.h.  All calls enqueue on `stream`
 * (a hipStream_t, NULL = default stream) and return without waiting.  dtype is
 * SPEC_DTYPE_FP32 (0) or SPEC_DTYPE_BF16 (1) and names the storage type of x,
 * weights and the KV cache.  Return: SPEC_OK or SPEC_EINVAL / SPEC_EHIP.
 */
#ifndef SPEC_KERNELS_H_
#define SPEC_KERNELS_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Weight-streaming projection used for every matrix of the model (QKV, O,
 * gate/up, down, draft fc, LM head; the parallel scoring of all draft tokens
 * by the target, Sec. 2, second step):   part[s][i][c] = sum over the s-th K range of
 * x[i][k] * w[c][k].  Up to three weight matrices (w0, w1, w2; rows0..2 rows
 * each, [rows, in] in the PACKED layout of spec_pack_weight; unused ones
 * NULL / 0) share x and write consecutive column ranges.  x: [m, in] with row stride ldx elements,
 * 1 <= m <= 4096 (more than 128 rows run as tiles of 128 that share the weight
 * rows through L2: the prefill case).  part: fp32 [n_split][m_pad][ldp],
 * ldp >= rows0+rows1+rows2, m_pad >= m.  The K ranges are whole slabs (256 bf16 / 128 fp32 elements),
 * balanced to within one slab; the caller sums the splits in ascending order. */
int spec_k_gemm(int32_t dtype, const void *x, int32_t ldx, int32_t m, int32_t in,
                const void *w0, int32_t rows0, const void *w1, int32_t rows1, const void *w2, int32_t rows2,
                float *part, int32_t ldp, int32_t m_pad, int32_t n_split, void *stream);

/* The gate and up projections of the SwiGLU feed-forward block (the target LLMs of
 * Sec. 4.1 are LLaMA models) in one launch, with the activation applied in the
 * launch's epilogue: act[i][c] = silu(x[i] . w_gate[c]) * (x[i] . w_up[c]), silu(g)
 * = g / (1 + exp(-g)), fp32 accumulation, rounded once to `dtype`.  w_gate_up: the
 * two [rows, in] matrices packed together by spec_pack_gate_up(); x: [m, in] with
 * row stride ldx; act: [m, rows] contiguous in `dtype`, 4-byte aligned; 1 <= m <= 4096.  K is not split (the
 * decode path uses this form whenever the projection has enough 32-row blocks to
 * fill the chip without a split). */
int spec_k_gemm_swiglu(int32_t dtype, const void *x, int32_t ldx, int32_t m, int32_t in, const void *w_gate_up, int32_t rows, void *act,
                       void *stream);

/* Tree attention (verification of several draft sequences in one forward,
 * Sec. 5 related work / Sec. 2 step two).  Row i (of `rows`) has its query in
 * q[i] ([hq*hd], always fp32), sits at key position base + depth[i] and attends to key
 * positions 0 .. base + depth[i]: position p < base is cache row p, position
 * p >= base is cache row base + anc[i*16 + p - base] (anc NULL: row p, a causal
 * chain).  max_depth = the largest depth[i] (host copy); with anc it must not
 * exceed 15.  Every cache row a query attends to must hold data.
 * kcache, vcache: [*, hkv*hd].  out: [rows, hq*hd] in dtype.  scratch: fp32,
 * rows*hq*max_parts*(hd+2) floats with max_parts >= (base+max depth)/128 + 2.
 * hd must be 64 or 128, hq/hkv one of 1, 2, 4, 8. */
int spec_k_attention(int32_t dtype, const void *q, const void *kcache, const void *vcache, int32_t rows, int32_t hq,
                     int32_t hkv, int32_t hd, int32_t base, const int32_t *depth, const int32_t *anc, int32_t max_depth,
                     float *scratch, int32_t max_parts, void *out, void *stream);

/* Per-row top-k log-probabilities over the vocabulary (the draft's confidence
 * scores of the expansion phase, appendix Drafting Hyper-Parameters):
 * logits fp32 [rows, vocab]; outputs top_tok / top_lp with row stride 16,
 * best first, equal values by lower token id; top_lp = log_softmax(logits)[tok].
 * rows <= 16, 1 <= k <= 16.  scratch_f: 16*n_slices*18 floats, scratch_i:
 * 16*n_slices*16 ints, n_slices = ceil(vocab / 4096). */
int spec_k_topk_logprob(const float *logits, int32_t rows, int32_t vocab, int32_t k, float *scratch_f, int32_t *scratch_i,
                        int32_t *top_tok, float *top_lp, void *stream);

/* spec_k_topk_logprob for callers that cannot allocate device memory and have no
 * scratch to pass: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same kernels, inputs, outputs and results as
 * spec_k_topk_logprob; the scratch is a fixed array inside the library (136 KiB
 * per GPU the library runs on, held until the process ends), which bounds the
 * vocabulary: vocab <= SPEC_STATIC_TOPK_MAX_VOCAB, larger ones return SPEC_ECAP.
 * The call allocates nothing and launches on `stream`, which must belong to the
 * CURRENT device (the array's address is looked up per device, on the first
 * call there).  All calls on one GPU share the array: calls that may overlap
 * (different streams, different threads) race; calls on one stream do not.
 * Nothing in the array needs clearing between calls. */
#define SPEC_STATIC_TOPK_MAX_VOCAB 262144
int spec_k_topk_logprob_static(const float *logits, int32_t rows, int32_t vocab, int32_t k, int32_t *top_tok, float *top_lp,
                               void *stream);

/* Acceptance with SAMPLED draft tokens: the ratio rule of speculative sampling
 * (Sec. 2, third step: the modified rejection sampling it names; the rule of the
 * chain and static-tree comparison systems of Sec. 4.1).  The tree has n_nodes
 * <= 128 nodes, node 0 the root, parents before children (tree_tok, tree_par:
 * device int32 arrays).  p_logits[i], q_logits[i] (fp32, [n_nodes, vocab]) are
 * the target's and the draft's logits AT node i; they score node i's children,
 * which must have been drawn from softmax(q_logits[i] / temperature) without
 * replacement and are tried in node order.  A child with token x is accepted
 * with probability min(1, p(x) / q(x)); a rejection replaces p by
 * normalise(max(p - q, 0)) and removes x from q; when all children of the
 * current node are rejected (or it has none, or 15 tokens are accepted) the
 * next token is drawn from the current p.  Random numbers: the library's
 * counter-based generator, stream (seed, cycle, node).
 * work: vocab floats of device scratch.  result: 33 device int32:
 * [0] = m accepted nodes, [1 + d] = accepted node of depth d (d = 0 is the
 * root), [17 + d] = token of depth d+1 for d < m and the next token at d = m. */
int spec_k_accept_qratio(const float *p_logits, const float *q_logits, int32_t n_nodes, int32_t vocab, float temperature,
                         const int32_t *tree_tok, const int32_t *tree_par, uint64_t seed, uint32_t cycle, float *work,
                         int32_t *result, void *stream);

/* The drafting side of the same rule: m (<= 16) distinct tokens drawn from
 * softmax(logits / temperature) without replacement, in draw order, as the m
 * largest of logits / temperature + Gumbel noise of stream (seed, cycle,
 * node_stream).  logits: fp32 [vocab]; out: m device int32.  Use a node_stream
 * that the acceptance does not use for the same cycle (the oracle uses
 * 65536 + node).  scratch_f: vocab + 16*n_slices*18 + 32 floats, scratch_i:
 * 16*n_slices*16 + 16 ints of device memory, n_slices = ceil(vocab / 4096). */
int spec_k_sample_children(const float *logits, int32_t vocab, float temperature, int32_t m, uint64_t seed, uint32_t cycle,
                           uint32_t node_stream, float *scratch_f, int32_t *scratch_i, int32_t *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_KERNELS_H_ */
