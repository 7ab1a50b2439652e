/*
 * libspec, training-side entry points: kernels of the method's training stage
 * that do not run at decoding time.  Same conventions as spec_kernels.h: all
 * data pointers are DEVICE pointers unless a comment says "host", calls
 * enqueue on `stream` (a hipStream_t, NULL = default stream) and return without
 * waiting; return SPEC_OK or SPEC_EINVAL / SPEC_EHIP (codes in spec.h).
 */
#ifndef SPEC_TRAIN_H_
#define SPEC_TRAIN_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPEC_HCA_MAX_STREAMS 8

/* Attention of harmonized context alignment, training step j = n_streams
 * (Sec. 3.2; appendix A.1, attention).  Stream 0 holds the keys/values derived
 * from the target LLM's features, stream m (1 <= m < j) those derived from the
 * draft features of training step m; the queries derive from the newest
 * stream.  For batch element b, head h, query position t and key position
 * s <= t with offset o = t - s:
 *     key/value = stream j-1-o   if o <= j-2   (one entry per earlier step,
 *                                               the newest at t itself)
 *                 stream 0       otherwise     (target features)
 * and out[b][t][h] = softmax_s(q.k / sqrt(hd)) . v over s = 0 .. t.  With
 * n_streams = 1 this is causal attention (the first step of Sec. 3.2).
 *
 * Layout, all bf16, rotary embedding already applied to q and k:
 *   q, out: [batch, seq, hq, hd];  k[m], v[m]: [batch, seq, hkv, hd].
 * k, v: HOST arrays of n_streams device pointers (read before the call
 * returns).  1 <= n_streams <= SPEC_HCA_MAX_STREAMS, seq >= 1, hd 64 or 128,
 * hq a multiple of hkv, every buffer 16-byte aligned.  Buffers are borrowed
 * for the duration of the kernel; out must not alias an input.  No scratch
 * memory is used. */
int spec_hca_attention(int32_t n_streams, const void *q, const void *const *k, const void *const *v, int32_t batch,
                       int32_t seq, int32_t hq, int32_t hkv, int32_t hd, void *out, void *stream);

#define SPEC_LOSS_MAX_K 128

/* Top-K distillation loss of harmonized objective distillation (Sec. 3.1,
 * Eq. 1), computed from features through the shared LM head, together with the
 * cross-entropy term of the Sec. 3.2 objective.  For each of `rows` positions r
 *     zq = lm_head . feat_target[r],   zp = lm_head . feat_draft[r]     (fp32 accumulation)
 *     q = softmax(zq),  p = softmax(zp),  Omega-hat = the k tokens of largest q
 *                                         (equal q: lower token id)
 *     loss_topk[r] = - sum over Omega-hat of q(x) log p(x)              (Eq. 1)
 *     loss_ce[r]   = - sum over the vocabulary of q(x) log p(x)
 * and loss_sum[0] = sum_r loss_topk[r], loss_sum[1] = sum_r loss_ce[r] (fixed
 * order; the mean over positions and the weight w of Sec. 4.1 are the
 * caller's).  K = 10 in the paper; 1 <= k <= SPEC_LOSS_MAX_K, k <= vocab,
 * ceil(vocab / 4096) * k <= 4096.
 *
 * feat_target, feat_draft: [rows, d] in dtype (SPEC_DTYPE_FP32 / _BF16), row
 * stride d.  lm_head: [vocab, d] in the PACKED layout of spec_pack_weight, same
 * dtype.  Outputs fp32: loss_topk, loss_ce [rows]; loss_sum [2] (any of the
 * three may be NULL).  scratch: spec_topk_loss_scratch_bytes(rows, vocab, k)
 * bytes of device memory, 256-byte aligned, owned by the caller; it holds the
 * fp32 logits of at most 512 positions at a time (sized to stay in the
 * last-level cache between the GEMM and the loss kernels) and per-slice
 * candidates.  The logits themselves are
 * not returned.  Errors: SPEC_EINVAL for bad arguments or a scratch that is too
 * small (nothing is launched), SPEC_EHIP if a launch fails. */
uint64_t spec_topk_loss_scratch_bytes(int32_t rows, int32_t vocab, int32_t k);
int spec_topk_loss(int32_t dtype, const void *feat_target, const void *feat_draft, int32_t rows, int32_t d,
                   const void *lm_head, int32_t vocab, int32_t k, void *scratch, uint64_t scratch_bytes, float *loss_topk,
                   float *loss_ce, float *loss_sum, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_TRAIN_H_ */
