// Tree attention for the decode path: each query row attends to the committed KV cache and
// to the nodes on its own root-to-node path.
//
// Row i sits at key position p = base + depth[i].  Key position q < base lives in cache
// slot q; position q >= base lives in slot base + anc[i][q - base], i.e. the row's own
// ancestors (anc == nullptr: a causal chain, slot q).  The keys of a row are therefore
// visited in POSITION order, which is exactly the order plain decoding visits them after
// the accepted nodes have been compacted to consecutive slots: the arithmetic of a row is
// a function of (its query, the key/value rows by position) only, so speculative and
// plain decoding agree bit for bit.
//
// Two code paths share one definition of the key order:
//
//  * vector path (attn_part_kernel): one wavefront handles (row, kv head, part of the key positions:
//    kAttnPart = 128 of them below position kAttnNear, kAttnFarPart beyond) and all G query heads that share the kv head; keys are taken 64 at a time,
//    lane = position offset for the scores (wave shuffles give the running max and sum of the
//    online softmax), then lane = output dim for P*V, which runs over the value rows staged in
//    LDS key by key in position order.  Used for fp32 storage, and for the TAIL
//    of every row in bf16 storage.
//
//  * matrix-core path (bulk workgroups of attn_hybrid_kernel, bf16 storage): the BULK of a row's keys, positions
//    [0, A(p)) with A(p) = 32 * floor(max(p - kMaxDepth, 0) / 32), lies in the committed cache
//    for every row of a tree (depth <= kMaxDepth), is the same key set for spec and plain decoding,
//    and is shared by all rows, so it runs as dense 32-key blocks on the MFMA units: S^T = K Q^T
//    and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16, K/V blocks staged once in LDS for all rows
//    (V transposed on the way in), queries and probabilities split into bf16 hi + lo parts so
//    that they keep fp32-class accuracy.  The remaining positions [A(p), p] (16..47 keys: the end
//    of the cache plus the row's own path) take the vector path.  A(p) depends on the position
//    only, so a row is computed by the same instructions over the same key groups whether it is
//    alone or part of a tree.
//
// Parts (fixed absolute boundaries: attn_part_begin; larger parts for far keys, where a long context would otherwise
// mean many partials to merge and many short workgroups) are merged per row in ascending order, the tail
// last, by attn_combine_kernel.  In the hybrid path the bulk and the tail are independent and run in ONE
// launch (different workgroups), so the chain per layer is two dependent kernels.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace spec {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

template <int N, int I = 0, typename F>
__device__ __forceinline__ void unrolled(F &&f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    unrolled<N, I + 1>(f);
  }
}

template <typename T> struct Chunk;   // 16-byte chunk -> floats
template <> struct Chunk<float> {
  static constexpr int kEpl = 4;
  static __device__ __forceinline__ void unpack(const u32x4_t &c, float *f) {
    f[0] = __uint_as_float(c.x); f[1] = __uint_as_float(c.y); f[2] = __uint_as_float(c.z); f[3] = __uint_as_float(c.w);
  }
};
template <> struct Chunk<bf16_t> {
  static constexpr int kEpl = 8;
  static __device__ __forceinline__ void unpack(const u32x4_t &c, float *f) {
    f[0] = __uint_as_float(c.x << 16); f[1] = __uint_as_float(c.x & 0xFFFF0000u);
    f[2] = __uint_as_float(c.y << 16); f[3] = __uint_as_float(c.y & 0xFFFF0000u);
    f[4] = __uint_as_float(c.z << 16); f[5] = __uint_as_float(c.z & 0xFFFF0000u);
    f[6] = __uint_as_float(c.w << 16); f[7] = __uint_as_float(c.w & 0xFFFF0000u);
  }
};

// End of the bulk region of a row at position p: the tail is the last kMaxDepth + 1 positions.  See the header.
__device__ __host__ __forceinline__ int bulk_end(int p) { return p > kMaxDepth ? p - kMaxDepth : 0; }

// Orders this wavefront's LDS writes before its later LDS reads of other lanes' data.  The LDS executes
// one wavefront's operations in issue order, so only the compiler has to be kept from reordering them.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// One wavefront: row i, kv head hk, part `part` (full mode) or the tail range (tail mode).  `qs` and `vs`
// are this wavefront's own LDS areas ([G][HD] floats and 64 staged value rows); no workgroup barrier is
// used, so wavefronts of one workgroup may work on different items.  `store` = false discards the result.
template <typename T> struct PartLds {
  static constexpr int vrow(int hd) { return hd * (int)sizeof(T) + 16; }   // +16: conflict-free row writes
};
template <typename T, int HD, int G>
__device__ __forceinline__ void attn_part_body(const AttnArgs &a, int i, int hk, int part, int lane, float (*qs)[HD],
                                               unsigned char *vs, bool store) {
  constexpr int EPL = Chunk<T>::kEpl;
  constexpr int DPL = HD / 64;                       // output dims per lane (contiguous)
  constexpr int VROW = PartLds<T>::vrow(HD);         // LDS bytes per staged value row
  const int base = a.base_ptr ? *a.base_ptr : a.base;  // device-resident when the launch is replayed from a graph
  const int p = base + a.depth[i];
  const int k_lo = attn_part_begin(part);
  const int k_hi = min(p + 1, attn_part_begin(part + 1));
  if (k_lo >= k_hi) return;

  const float *qrow = (const float *)a.q + ((size_t)i * a.hq + (size_t)hk * G) * HD;   // queries are fp32
  for (int e = lane; e < G * HD; e += 64) qs[e / HD][e % HD] = qrow[e];

  float m_run[G], l_run[G], o[G][DPL];
#pragma unroll
  for (int gh = 0; gh < G; gh++) {
    m_run[gh] = -INFINITY; l_run[gh] = 0.f;
#pragma unroll
    for (int dd = 0; dd < DPL; dd++) o[gh][dd] = 0.f;
  }
  const int *anc = a.anc ? a.anc + (size_t)i * kAncStride : nullptr;
  const size_t row_stride = (size_t)a.hkv * HD;
  const T *kbase = (const T *)a.kcache + (size_t)hk * HD;
  const T *vbase = (const T *)a.vcache + (size_t)hk * HD;

  for (int kb = k_lo; kb < k_hi; kb += 64) {
    // lane = key: this lane's key row and value row (all loads issued before anything is used)
    const int kq = kb + lane;
    const bool valid = kq < k_hi;
    // lanes past the range re-read the last key of the range (initialised data; their weight is 0)
    const int kr = valid ? kq : k_hi - 1;
    const int slot = kr < base ? kr : base + (anc ? anc[kr - base] : kr - base);
    const T *kptr = kbase + (size_t)slot * row_stride;
    const T *vptr = vbase + (size_t)slot * row_stride;
    u32x4_t kc[HD / EPL], vc[HD / EPL];
#pragma unroll
    for (int dc = 0; dc < HD / EPL; dc++) kc[dc] = *(const u32x4_t *)(kptr + dc * EPL);
#pragma unroll
    for (int dc = 0; dc < HD / EPL; dc++) vc[dc] = *(const u32x4_t *)(vptr + dc * EPL);
    wave_lds_sync();                                   // qs written (first pass) / previous block's vs reads done
    float s[G];
#pragma unroll
    for (int gh = 0; gh < G; gh++) s[gh] = 0.f;
#pragma unroll
    for (int dc = 0; dc < HD / EPL; dc++) {
      float kf[EPL];
      Chunk<T>::unpack(kc[dc], kf);
#pragma unroll
      for (int gh = 0; gh < G; gh++)
#pragma unroll
        for (int e = 0; e < EPL; e++) s[gh] = fmaf(qs[gh][dc * EPL + e], kf[e], s[gh]);
    }
    // stage the value rows: row `lane` of vs
#pragma unroll
    for (int dc = 0; dc < HD / EPL; dc++) *(u32x4_t *)(vs + lane * VROW + dc * 16) = vc[dc];
    float pk[G];
#pragma unroll
    for (int gh = 0; gh < G; gh++) {
      const float sc = valid ? s[gh] * a.scale : -INFINITY;
      const float m_new = fmaxf(m_run[gh], wave_max(sc));
      const float corr = __expf(m_run[gh] - m_new);      // first block: exp(-inf) = 0
      pk[gh] = valid ? __expf(sc - m_new) : 0.f;
      l_run[gh] = l_run[gh] * corr + wave_sum(pk[gh]);
#pragma unroll
      for (int dd = 0; dd < DPL; dd++) o[gh][dd] *= corr;
      m_run[gh] = m_new;
    }
    wave_lds_sync();                                   // value rows staged
    // lane = output dims lane*DPL ..: accumulate key by key in position order
    // Eight keys per step so that the LDS reads of a step are in flight together.  Lanes past the last
    // key hold weight 0 and a finite value row (a copy of the last key's), so rounding a step up to eight adds zeros.
    const int nk = min(64, k_hi - kb);
    const unsigned char *vcol = vs + lane * DPL * (int)sizeof(T);
    for (int k0 = 0; k0 < nk; k0 += 8) {
      float vv[8][DPL];
#pragma unroll
      for (int kk = 0; kk < 8; kk++)
#pragma unroll
        for (int dd = 0; dd < DPL; dd++) vv[kk][dd] = to_f32(*(const T *)(vcol + (k0 + kk) * VROW + dd * (int)sizeof(T)));
#pragma unroll
      for (int kk = 0; kk < 8; kk++)
#pragma unroll
        for (int gh = 0; gh < G; gh++) {
          const float w = __shfl(pk[gh], k0 + kk, 64);
#pragma unroll
          for (int dd = 0; dd < DPL; dd++) o[gh][dd] = fmaf(w, vv[kk][dd], o[gh][dd]);
        }
    }
  }
  if (!store) return;
#pragma unroll
  for (int gh = 0; gh < G; gh++) {
    float *dst = a.part + (((size_t)i * a.hq + hk * G + gh) * a.max_parts + part) * (HD + 2);
    if (lane == 0) { dst[0] = m_run[gh]; dst[1] = l_run[gh]; }
#pragma unroll
    for (int dd = 0; dd < DPL; dd++) dst[2 + lane * DPL + dd] = o[gh][dd];
  }
}

// The tail of a row in the hybrid path: positions [max(p - kMaxDepth, 0), p], at most kTailKeys = 16 keys,
// the end of the committed cache followed by the row's own path.  One wavefront per (row, kv head): four
// lanes share a key (each takes a quarter of the head dim for the score, summed over the quad in a fixed
// order), then lane = output dim for P*V over the value rows staged in LDS, key by key in position order.
// The result goes to the last part slot.
constexpr int kTailKeys = kMaxDepth + 1;
static_assert(kTailKeys * 4 == 64, "one wavefront = 16 keys x 4 lanes");
template <typename T, int HD, int G>
__device__ __forceinline__ void attn_tail_body(const AttnArgs &a, int i, int hk, int lane, float (*qs)[HD],
                                               unsigned char *vs, bool store) {
  constexpr int EPL = Chunk<T>::kEpl;
  constexpr int DPL = HD / 64;                       // output dims per lane (contiguous)
  constexpr int VROW = PartLds<T>::vrow(HD);
  constexpr int QD = HD / 4;                         // dims per lane of a key quad
  constexpr int QC = QD / EPL;                       // 16-byte chunks per lane
  const int base = a.base_ptr ? *a.base_ptr : a.base;
  const int p = base + a.depth[i];
  const int k_lo = bulk_end(p);
  const int kk = lane >> 2, qt = lane & 3;
  const int kq = k_lo + kk;
  const bool valid = kq <= p;
  const int *anc = a.anc ? a.anc + (size_t)i * kAncStride : nullptr;
  // lanes past position p re-read the row's own key (initialised data; their weight is 0)
  const int kr = valid ? kq : p;
  const int slot = kr < base ? kr : base + (anc ? anc[kr - base] : kr - base);
  const size_t row_stride = (size_t)a.hkv * HD;
  const T *kptr = (const T *)a.kcache + (size_t)slot * row_stride + (size_t)hk * HD + qt * QD;
  const T *vptr = (const T *)a.vcache + (size_t)slot * row_stride + (size_t)hk * HD + qt * QD;
  u32x4_t kc[QC], vc[QC];
#pragma unroll
  for (int dc = 0; dc < QC; dc++) kc[dc] = *(const u32x4_t *)(kptr + dc * EPL);
#pragma unroll
  for (int dc = 0; dc < QC; dc++) vc[dc] = *(const u32x4_t *)(vptr + dc * EPL);
  const float *qrow = (const float *)a.q + ((size_t)i * a.hq + (size_t)hk * G) * HD;   // queries are fp32
  for (int e = lane; e < G * HD; e += 64) qs[e / HD][e % HD] = qrow[e];
  wave_lds_sync();
  float s[G];
#pragma unroll
  for (int gh = 0; gh < G; gh++) s[gh] = 0.f;
#pragma unroll
  for (int dc = 0; dc < QC; dc++) {
    float kf[EPL];
    Chunk<T>::unpack(kc[dc], kf);
#pragma unroll
    for (int gh = 0; gh < G; gh++)
#pragma unroll
      for (int e = 0; e < EPL; e++) s[gh] = fmaf(qs[gh][qt * QD + dc * EPL + e], kf[e], s[gh]);
  }
#pragma unroll
  for (int dc = 0; dc < QC; dc++) *(u32x4_t *)(vs + kk * VROW + qt * QD * (int)sizeof(T) + dc * 16) = vc[dc];
  float m_run[G], l_run[G], pk[G];
#pragma unroll
  for (int gh = 0; gh < G; gh++) {
    float t = s[gh];
    t += __shfl_xor(t, 1, 64);                       // quad sum, fixed order
    t += __shfl_xor(t, 2, 64);
    const float sc = valid ? t * a.scale : -INFINITY;
    m_run[gh] = wave_max(sc);                        // at least key p itself is valid
    pk[gh] = valid ? __expf(sc - m_run[gh]) : 0.f;
    l_run[gh] = wave_sum(qt == 0 ? pk[gh] : 0.f);
  }
  wave_lds_sync();                                   // value rows staged
  float o[G][DPL];
#pragma unroll
  for (int gh = 0; gh < G; gh++)
#pragma unroll
    for (int dd = 0; dd < DPL; dd++) o[gh][dd] = 0.f;
  // Lanes of keys past p hold weight 0 and a finite value row (a copy of the row's own), so all 16 rows can be summed.
  const unsigned char *vcol = vs + lane * DPL * (int)sizeof(T);
#pragma unroll
  for (int k0 = 0; k0 < kTailKeys; k0 += 8) {
    float vv[8][DPL];
#pragma unroll
    for (int u = 0; u < 8; u++)
#pragma unroll
      for (int dd = 0; dd < DPL; dd++) vv[u][dd] = to_f32(*(const T *)(vcol + (k0 + u) * VROW + dd * (int)sizeof(T)));
#pragma unroll
    for (int u = 0; u < 8; u++)
#pragma unroll
      for (int gh = 0; gh < G; gh++) {
        const float w = __shfl(pk[gh], (k0 + u) * 4, 64);
#pragma unroll
        for (int dd = 0; dd < DPL; dd++) o[gh][dd] = fmaf(w, vv[u][dd], o[gh][dd]);
      }
  }
  if (!store) return;
#pragma unroll
  for (int gh = 0; gh < G; gh++) {
    float *dst = a.part + (((size_t)i * a.hq + hk * G + gh) * a.max_parts + a.max_parts - 1) * (HD + 2);
    if (lane == 0) { dst[0] = m_run[gh]; dst[1] = l_run[gh]; }
#pragma unroll
    for (int dd = 0; dd < DPL; dd++) dst[2 + lane * DPL + dd] = o[gh][dd];
  }
}

// grid (rows, kv heads, parts); one wavefront per workgroup.
template <typename T, int HD, int G>
__global__ __launch_bounds__(64) void attn_part_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) float qs[G][HD];
  __shared__ __attribute__((aligned(16))) unsigned char vs[64 * PartLds<T>::vrow(HD)];
  attn_part_body<T, HD, G>(a, blockIdx.x, blockIdx.y, blockIdx.z, threadIdx.x, qs, vs, true);
}

// grid (rows, hq); block HD threads.  Merges the row's parts in ascending order; in hybrid mode these are
// the bulk parts followed by the tail (kept in the last slot).  The (max, sum) pairs of up to kCombineChunk
// parts are fetched by one thread each and turned into weights in LDS, so that the per-dim pass issues
// independent, coalesced loads; the sums themselves run in ascending part order.
constexpr int kCombineChunk = 64;
constexpr int kCombineFew = 8;         // up to this many parts a thread keeps everything in registers
template <typename T, int HD>
__global__ __launch_bounds__(HD) void attn_combine_kernel(AttnArgs a) {
  __shared__ float pm[kCombineChunk], pl[kCombineChunk];
  __shared__ float red[2];
  const int i = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
  const int p = (a.base_ptr ? *a.base_ptr : a.base) + a.depth[i];
  const int n_front = attn_parts_covering(a.tail_only ? bulk_end(p) : p + 1);
  const int n_parts = n_front + (a.tail_only ? 1 : 0);
  const float *src = a.part + ((size_t)i * a.hq + h) * a.max_parts * (HD + 2);
  auto slot = [&](int t) { return (size_t)(t < n_front ? t : a.max_parts - 1) * (HD + 2); };
  if (n_parts <= kCombineFew) {
    // Few parts (short contexts): every value is requested up front (clamped to a valid part; absent ones are not used),
    // then the same arithmetic as below runs out of registers: one memory round trip instead of three.
    float pm_[kCombineFew], pl_[kCombineFew], pv_[kCombineFew];
#pragma unroll
    for (int t = 0; t < kCombineFew; t++) {
      const float *sp = src + slot(t < n_parts ? t : 0);
      pm_[t] = sp[0]; pl_[t] = sp[1]; pv_[t] = sp[2 + d];
    }
    float m = -INFINITY;
#pragma unroll
    for (int t = 0; t < kCombineFew; t++) if (t < n_parts) m = fmaxf(m, pm_[t]);
    float l = 0.f, o = 0.f;
#pragma unroll
    for (int t = 0; t < kCombineFew; t++)
      if (t < n_parts) {
        const float w = __expf(pm_[t] - m);
        l += pl_[t] * w; o += pv_[t] * w;
      }
    ((T *)a.out)[((size_t)i * a.hq + h) * HD + d] = from_f32<T>(o / l);
    return;
  }
  // pass 1: the row's maximum
  float m = -INFINITY;
  for (int t = d; t < n_parts; t += HD) m = fmaxf(m, src[slot(t)]);
  m = wave_max(m);
  if (HD > 64) {
    if ((d & 63) == 0) red[d >> 6] = m;
    __syncthreads();
    m = fmaxf(red[0], red[1]);
  }
  // pass 2: chunks of parts; weights once per part, then every thread adds its dim in ascending order
  float l = 0.f, o = 0.f;
  for (int t0 = 0; t0 < n_parts; t0 += kCombineChunk) {
    const int nt = min(kCombineChunk, n_parts - t0);
    __syncthreads();
    if (d < nt) {
      const float *sp = src + slot(t0 + d);
      const float w = __expf(sp[0] - m);
      pm[d] = w; pl[d] = sp[1] * w;
    }
    __syncthreads();
    int t = 0;
    for (; t + 4 <= nt; t += 4) {
      const float v0 = src[slot(t0 + t) + 2 + d], v1 = src[slot(t0 + t + 1) + 2 + d];
      const float v2 = src[slot(t0 + t + 2) + 2 + d], v3 = src[slot(t0 + t + 3) + 2 + d];
      l += pl[t]; o += v0 * pm[t];
      l += pl[t + 1]; o += v1 * pm[t + 1];
      l += pl[t + 2]; o += v2 * pm[t + 2];
      l += pl[t + 3]; o += v3 * pm[t + 3];
    }
    for (; t < nt; t++) { l += pl[t]; o += src[slot(t0 + t) + 2 + d] * pm[t]; }
  }
  ((T *)a.out)[((size_t)i * a.hq + h) * HD + d] = from_f32<T>(o / l);
}

// ---- matrix-core path for the bulk region (bf16 storage) -----------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

// x = hi + lo with hi, lo bf16: the pair keeps ~16 mantissa bits of an fp32 value.
__device__ __forceinline__ void split8(const float (&x)[8], u32x4_t &hi, u32x4_t &lo) {
  uint32_t h[4], l[4];
#pragma unroll
  for (int e = 0; e < 4; e++) {
    h[e] = pack_bf16x2(x[2 * e], x[2 * e + 1]);
    l[e] = pack_bf16x2(x[2 * e] - __uint_as_float(h[e] << 16), x[2 * e + 1] - __uint_as_float(h[e] & 0xFFFF0000u));
  }
  hi = u32x4_t{h[0], h[1], h[2], h[3]};
  lo = u32x4_t{l[0], l[1], l[2], l[3]};
}
__device__ __forceinline__ f32x16_t mfma_bf16(const u32x4_t &a, const u32x4_t &b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}


// One launch covers both regions of the hybrid path.  Workgroups [0, n_bulk) (n_bulk = bulk_parts * kv heads
// * q_groups, part fastest) run the matrix-core bulk: NW waves, wave w owns 32 "query rows" (row i, head gh
// of the kv group), r = (qgroup*NW + w)*32 + lane%32, i = r / G, gh = r % G.  The remaining workgroups run
// the vector tail, one (row, kv head) item per wavefront on the first kTailWaves wavefronts, and leave it in
// the last part slot.  The two kinds of work are independent; attn_combine_kernel merges them afterwards.
#ifndef SPEC_ATTN_RING
#define SPEC_ATTN_RING 1
#endif
constexpr int kBulkRing = SPEC_ATTN_RING;   // register sets for K/V blocks in flight per bulk workgroup
template <int NW> struct TailWaves { static constexpr int value = NW < 4 ? NW : 4; };
template <int HD, int G, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_hybrid_kernel(AttnArgs a) {
  constexpr int DB = HD / 32;                 // 32-dim blocks of the output
  constexpr int KK = HD / 16;                 // MFMA steps of q.k
  constexpr int KSTR = HD * 2 + 16;           // LDS bytes per key row (+16: conflict-free b128 reads)
  constexpr int VSTR = 32 * 2 + 8;            // LDS bytes per dim row of V^T (+8: conflict-free b64 reads)
  constexpr int NT = NW * 64;
  constexpr int PIECES = (32 * HD * 2 / 16 + NT - 1) / NT;   // 16-byte pieces of one K (or V) block per thread
  constexpr int kTailWaves = TailWaves<NW>::value;
  constexpr int kTailQ = G * HD * 4;                                         // a tail wavefront's query area
  constexpr int kTailWave = kTailQ + kTailKeys * PartLds<bf16_t>::vrow(HD);  // ... plus its staged value rows
  constexpr int kBulkBuf = 32 * KSTR + HD * VSTR;                            // one staged K block + V^T block
  constexpr int kBulkLds = 2 * kBulkBuf;                                     // double-buffered
  constexpr int kLds = kBulkLds > kTailWaves * kTailWave ? kBulkLds : kTailWaves * kTailWave;
  __shared__ __attribute__((aligned(16))) unsigned char lds[kLds];

  const int n_bulk = a.bulk_parts * a.hkv * a.q_groups;
  if ((int)blockIdx.x >= n_bulk) {
    const int w = threadIdx.x >> 6;
    if (w >= kTailWaves) return;
    int item = ((int)blockIdx.x - n_bulk) * kTailWaves + w;
    const bool active = item < a.rows * a.hkv;
    if (!active) item = a.rows * a.hkv - 1;               // valid addresses; result discarded
    unsigned char *mine = lds + w * kTailWave;
    attn_tail_body<bf16_t, HD, G>(a, item / a.hkv, item % a.hkv, threadIdx.x & 63, (float (*)[HD])mine, mine + kTailQ, active);
    return;
  }
  const int part = (int)blockIdx.x % a.bulk_parts, hk = ((int)blockIdx.x / a.bulk_parts) % a.hkv;
  const int qgroup = (int)blockIdx.x / (a.bulk_parts * a.hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 31, g = lane >> 5;
  // With a device-resident base (graph replay) the grid is sized for the longest context and the
  // blocks that exist are derived here; otherwise the host has computed them.
  const int base = a.base_ptr ? *a.base_ptr : a.base;
  // keys [0, key_lim) are the union of the rows' bulk regions: all of them exist and are initialised
  const int key_lim = a.base_ptr ? min(a.bulk_keys, bulk_end(base + kMaxDepth)) : a.bulk_keys;
  const int n_blocks = (key_lim + 31) / 32;
  const int b_lo = attn_part_begin(part) / 32;
  const int b_hi = min(attn_part_begin(part + 1) / 32, n_blocks);
  if (b_lo >= b_hi) return;

  const int r = (qgroup * NW + wave) * 32 + c;
  const bool valid_q = r < a.rows * G;
  const int i = valid_q ? r / G : 0, gh = valid_q ? r % G : 0;
  const int k_end = valid_q ? bulk_end(base + a.depth[i]) : 0;               // keys [0, k_end) belong to this row's bulk

  const size_t row_stride = (size_t)a.hkv * HD;              // elements between consecutive cache slots
  const bf16_t *kg = (const bf16_t *)a.kcache + (size_t)hk * HD;
  const bf16_t *vg = (const bf16_t *)a.vcache + (size_t)hk * HD;
  constexpr int PPR = HD * 2 / 16;                           // pieces per key row
  // The global loads of a block land in one of R register sets, so that R blocks are in flight.  Measured on
  // MI355X, more than one set does not pay: the arithmetic of a block, not the wait for its loads, is what a
  // workgroup spends its time on.
  constexpr int R = kBulkRing;
  u32x4_t kreg[R][PIECES], vreg[R][PIECES];
  auto prefetch = [&](auto set_tag, int b) {
    constexpr int SET = decltype(set_tag)::value;
#pragma unroll
    for (int e = 0; e < PIECES; e++) {
      const int q = tid + e * NT;
      const int key = (q / PPR) & 31, piece = q % PPR;       // (& 31: threads past the block re-read a valid key)
      // The last block may reach past key_lim; those keys are masked for every row, so they are read from
      // key key_lim - 1 instead (initialised, inside the cache; key_lim >= 1 for every block that runs).
      const size_t off = (size_t)min(b * 32 + key, key_lim - 1) * row_stride + piece * 8;
      kreg[SET][e] = *(const u32x4_t *)(kg + off);
      vreg[SET][e] = *(const u32x4_t *)(vg + off);
    }
  };
  // A wavefront whose 32 query rows all lie past the last row only helps to load and stage the blocks.
  const bool computes = __builtin_amdgcn_readfirstlane((qgroup * NW + wave) * 32 < a.rows * G ? 1 : 0) != 0;
  u32x4_t qhi[KK], qlo[KK];                                  // query fragments: step kk covers dims kk*16 + g*8 .. +8
  f32x16_t o[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int v = 0; v < 16; v++) o[db][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  auto stage = [&](auto set_tag, int buf) {
    constexpr int SET = decltype(set_tag)::value;
    unsigned char *k_lds = lds + buf * kBulkBuf, *vt_lds = k_lds + 32 * KSTR;
#pragma unroll
    for (int e = 0; e < PIECES; e++) {
      const int q = tid + e * NT;
      if (q < 32 * PPR) {
        const int key = q / PPR, piece = q % PPR;
        *(u32x4_t *)(k_lds + key * KSTR + piece * 16) = kreg[SET][e];
        const uint32_t w[4] = {vreg[SET][e].x, vreg[SET][e].y, vreg[SET][e].z, vreg[SET][e].w};
#pragma unroll
        for (int d2 = 0; d2 < 8; d2++)                       // V^T[dim][key]
          *(uint16_t *)(vt_lds + (piece * 8 + d2) * VSTR + key * 2) = (uint16_t)(w[d2 >> 1] >> ((d2 & 1) * 16));
      }
    }
  };

  // One part = NB blocks, b_lo .. b_lo + NB - 1, as straight-line code: every load and every wait for a load
  // is unconditional, so the compiler counts outstanding loads exactly and a block waits for its own set only.
  // Blocks at or past b_hi (a part cut short by the end of the keys) are loaded from clamped addresses, staged
  // and skipped by the arithmetic.  K/V blocks alternate between two LDS buffers: block j+1 is staged between the
  // two matrix-core phases of block j and its register set is refilled right away with block j+1+R; one barrier
  // per block.
  auto run = [&](auto nb_tag) {
    constexpr int NB = decltype(nb_tag)::value;
    static_assert(NB >= 1 && NB <= 16, "a part is unrolled block by block");
    unrolled<(R < NB ? R : NB)>([&](auto t_tag) { prefetch(t_tag, b_lo + decltype(t_tag)::value); });
    {
      const float *qrow = (const float *)a.q + ((size_t)i * a.hq + (size_t)hk * G + gh) * HD;
#pragma unroll
      for (int kk = 0; kk < KK; kk++) {
        float x[8];
        const float4 x0 = *(const float4 *)(qrow + kk * 16 + g * 8), x1 = *(const float4 *)(qrow + kk * 16 + g * 8 + 4);
        x[0] = x0.x; x[1] = x0.y; x[2] = x0.z; x[3] = x0.w; x[4] = x1.x; x[5] = x1.y; x[6] = x1.z; x[7] = x1.w;
        split8(x, qhi[kk], qlo[kk]);
      }
    }
    stage(std::integral_constant<int, 0>{}, 0);
    __syncthreads();
    if constexpr (R < NB) prefetch(std::integral_constant<int, 0>{}, b_lo + R);
    unrolled<NB>([&](auto j_tag) {
      constexpr int j = decltype(j_tag)::value, cur = j & 1;
      const int b = b_lo + j;
      const bool live = computes && b < b_hi;                // same for all lanes of a wavefront
      const unsigned char *k_lds = lds + cur * kBulkBuf, *vt_lds = k_lds + 32 * KSTR;
      float pv[16];
      if (live) {
        f32x16_t s;
#pragma unroll
        for (int v = 0; v < 16; v++) s[v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; kk++) {
          const u32x4_t kf = *(const u32x4_t *)(k_lds + c * KSTR + kk * 32 + g * 16);
          s = mfma_bf16(kf, qhi[kk], s);
          s = mfma_bf16(kf, qlo[kk], s);
        }
        // s[v] = q . k for key 8*(v/4) + 4*g + v%4 of the block and query row c
        // keys at or past k_end are masked: they add exact zeros, so a row's result does not depend on them
        const int key0 = b * 32 + 4 * g;
        float mb = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; v++) {
          s[v] = key0 + 8 * (v >> 2) + (v & 3) < k_end ? s[v] * a.scale : -INFINITY;
          mb = fmaxf(mb, s[v]);
        }
        mb = fmaxf(mb, __shfl_xor(mb, 32, 64));
        const float m_new = fmaxf(m_run, mb);
        const float corr = m_new == -INFINITY ? 1.f : __expf(m_run - m_new);
        float ls = 0.f;
#pragma unroll
        for (int v = 0; v < 16; v++) { pv[v] = s[v] == -INFINITY ? 0.f : __expf(s[v] - m_new); ls += pv[v]; }
        ls += __shfl_xor(ls, 32, 64);
        l_run = l_run * corr + ls;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
          for (int v = 0; v < 16; v++) o[db][v] *= corr;
      }
      if constexpr (j + 1 < NB) {
        constexpr int NEXT = (j + 1) % R;
        stage(std::integral_constant<int, NEXT>{}, cur ^ 1);   // every wave left that buffer at the last barrier
        if constexpr (j + 1 + R < NB) prefetch(std::integral_constant<int, NEXT>{}, b + 1 + R);
      }
      if (live) {
        // O^T += V^T P^T over two 16-key steps; step u uses the lane's own values v = 8u .. 8u+7,
        // i.e. keys 16u + 8*(e/4) + 4g + e%4, and V^T supplies the same keys per dim.
#pragma unroll
        for (int u = 0; u < 2; u++) {
          float x[8];
#pragma unroll
          for (int e = 0; e < 8; e++) x[e] = pv[8 * u + e];
          u32x4_t phi, plo;
          split8(x, phi, plo);
#pragma unroll
          for (int db = 0; db < DB; db++) {
            const unsigned char *vp = vt_lds + (db * 32 + c) * VSTR + (16 * u + 4 * g) * 2;
            const u32x2_t v0 = *(const u32x2_t *)vp, v1 = *(const u32x2_t *)(vp + 16);
            const u32x4_t vf = {v0.x, v0.y, v1.x, v1.y};
            o[db] = mfma_bf16(vf, phi, o[db]);
            o[db] = mfma_bf16(vf, plo, o[db]);
          }
        }
      }
      if constexpr (j + 1 < NB) __syncthreads();             // block j+1 staged; everyone is done with block j
    });
  };
  if (part < kAttnNear / kAttnPart) run(std::integral_constant<int, kAttnPart / 32>{});
  else run(std::integral_constant<int, kAttnFarPart / 32>{});
  if (!valid_q) return;
  float *dst = a.part + (((size_t)i * a.hq + hk * G + gh) * a.max_parts + part) * (HD + 2);
  if (g == 0) { dst[0] = m_run; dst[1] = l_run; }
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int v = 0; v < 16; v++) dst[2 + db * 32 + 8 * (v >> 2) + 4 * g + (v & 3)] = o[db][v];
}

template <int HD, int G, int NW>
static hipError_t launch_hybrid(AttnArgs a, int q_groups, hipStream_t st) {
  a.q_groups = q_groups;
  const int n_tail = (a.rows * a.hkv + TailWaves<NW>::value - 1) / TailWaves<NW>::value;
  hipLaunchKernelGGL((attn_hybrid_kernel<HD, G, NW>), dim3(a.bulk_parts * a.hkv * q_groups + n_tail), dim3(NW * 64), 0, st, a);
  return hipGetLastError();
}

template <typename T, int HD, int G>
static hipError_t launch_thg(AttnArgs a, int max_pos, hipStream_t st) {
  hipError_t e;
  if (sizeof(T) == 2) {
    // hybrid: matrix-core bulk over [0, A(max_pos)) and the vector tail of every row in one launch
    a.tail_only = 1;
    a.bulk_keys = bulk_end(max_pos);
    a.bulk_blocks = (a.bulk_keys + 31) / 32;
    a.bulk_parts = attn_parts_covering(a.bulk_keys);
    if (a.bulk_parts + 1 > a.max_parts) return hipErrorInvalidValue;
    // At least four wavefronts per bulk workgroup, also for fewer than four blocks of 32 query rows: the ones
    // without rows still take their share of loading and staging the K/V blocks.
    const int qblocks = (a.rows * G + 31) / 32;
    if (qblocks <= 4) e = launch_hybrid<HD, G, 4>(a, 1, st);
    else e = launch_hybrid<HD, G, 8>(a, (qblocks + 7) / 8, st);
  } else {
    a.tail_only = 0;
    a.bulk_blocks = 0;
    const int n_parts = attn_parts_covering(max_pos + 1);
    if (n_parts > a.max_parts) return hipErrorInvalidValue;
    hipLaunchKernelGGL((attn_part_kernel<T, HD, G>), dim3(a.rows, a.hkv, n_parts), dim3(64), 0, st, a);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_combine_kernel<T, HD>), dim3(a.rows, a.hq), dim3(HD), 0, st, a);
  return hipGetLastError();
}
template <typename T, int HD>
static hipError_t launch_th(const AttnArgs &a, int max_pos, hipStream_t st) {
  switch (a.hq / a.hkv) {
    case 1: return launch_thg<T, HD, 1>(a, max_pos, st);
    case 2: return launch_thg<T, HD, 2>(a, max_pos, st);
    case 4: return launch_thg<T, HD, 4>(a, max_pos, st);
    case 8: return launch_thg<T, HD, 8>(a, max_pos, st);
    default: return hipErrorInvalidValue;
  }
}

// max_pos: largest key position any row attends to (host-known bound: base + max depth).
hipError_t launch_attention(int dtype, const AttnArgs &a, int max_pos, hipStream_t st) {
  if (a.rows < 1 || a.hkv < 1 || a.hq % a.hkv != 0) return hipErrorInvalidValue;
  if (a.hd == 128) return dtype == 1 ? launch_th<bf16_t, 128>(a, max_pos, st) : launch_th<float, 128>(a, max_pos, st);
  if (a.hd == 64) return dtype == 1 ? launch_th<bf16_t, 64>(a, max_pos, st) : launch_th<float, 64>(a, max_pos, st);
  return hipErrorInvalidValue;
}

}  // namespace spec
