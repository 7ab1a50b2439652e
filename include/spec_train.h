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

#ifdef __cplusplus
}
#endif
#endif /* SPEC_TRAIN_H_ */
