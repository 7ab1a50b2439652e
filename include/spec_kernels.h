/*
 * libspec, kernel-level entry points: the individual gfx950 kernels of the
 * decode path, callable on caller-provided DEVICE buffers.  They exist so that
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
 * gate/up, down, draft fc, LM head; target forward of Sec. 2's "evaluates ...
 * in parallel" step):   part[s][i][c] = sum over the s-th K range of
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

#ifdef __cplusplus
}
#endif
#endif /* SPEC_KERNELS_H_ */
