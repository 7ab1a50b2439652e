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
// One wavefront handles (row, kv head, part of kAttnPart = 256 key positions) and all G
// query heads that share the kv head.  Parts have fixed absolute boundaries; within a part
// keys are taken 64 at a time, lane = position offset, with wave shuffles for the running
// max and sum of the online softmax; P*V is accumulated key by key in position order.  A
// second kernel merges the parts of a row in ascending order.
#include "common.h"
#include "kernels.h"

namespace spec {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

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

template <typename T, int HD, int G>
__global__ __launch_bounds__(64) void attn_part_kernel(AttnArgs a) {
  constexpr int EPL = Chunk<T>::kEpl;
  constexpr int DPL = HD / 64;                       // output dims per lane
  __shared__ __attribute__((aligned(16))) float qs[G][HD];
  const int i = blockIdx.x, hk = blockIdx.y, part = blockIdx.z, lane = threadIdx.x;
  const int p = a.base + a.depth[i];
  const int k_lo = part * kAttnPart;
  const int k_hi = min(p + 1, k_lo + kAttnPart);
  if (k_lo >= k_hi) return;

  const float *qrow = (const float *)a.q + ((size_t)i * a.hq + (size_t)hk * G) * HD;   // queries are fp32
  for (int e = lane; e < G * HD; e += 64) qs[e / HD][e % HD] = qrow[e];
  __syncthreads();

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
  const T *vbase = (const T *)a.vcache + (size_t)hk * HD + lane * DPL;

  for (int kb = k_lo; kb < k_hi; kb += 64) {
    const int kq = kb + lane;
    const bool valid = kq < k_hi;
    int slot = 0;
    if (valid) slot = kq < a.base ? kq : a.base + (anc ? anc[kq - a.base] : kq - a.base);
    const T *kptr = kbase + (size_t)slot * row_stride;
    float s[G];
#pragma unroll
    for (int gh = 0; gh < G; gh++) s[gh] = 0.f;
#pragma unroll 4
    for (int dc = 0; dc < HD / EPL; dc++) {
      const u32x4_t ck = *(const u32x4_t *)(kptr + dc * EPL);
      float kf[EPL];
      Chunk<T>::unpack(ck, kf);
#pragma unroll
      for (int gh = 0; gh < G; gh++)
#pragma unroll
        for (int e = 0; e < EPL; e++) s[gh] = fmaf(qs[gh][dc * EPL + e], kf[e], s[gh]);
    }
    float pk[G];
#pragma unroll
    for (int gh = 0; gh < G; gh++) {
      const float sc = valid ? s[gh] * a.scale : -INFINITY;
      const float m_new = fmaxf(m_run[gh], wave_max(sc));
      const float corr = expf(m_run[gh] - m_new);        // first block: exp(-inf) = 0
      pk[gh] = valid ? expf(sc - m_new) : 0.f;
      l_run[gh] = l_run[gh] * corr + wave_sum(pk[gh]);
#pragma unroll
      for (int dd = 0; dd < DPL; dd++) o[gh][dd] *= corr;
      m_run[gh] = m_new;
    }
    const int nk = min(64, k_hi - kb);
    for (int k = 0; k < nk; k++) {
      const int sl = __shfl(slot, k, 64);
      const T *vp = vbase + (size_t)sl * row_stride;
      float vv[DPL];
#pragma unroll
      for (int dd = 0; dd < DPL; dd++) vv[dd] = to_f32(vp[dd]);
#pragma unroll
      for (int gh = 0; gh < G; gh++) {
        const float w = __shfl(pk[gh], k, 64);
#pragma unroll
        for (int dd = 0; dd < DPL; dd++) o[gh][dd] = fmaf(w, vv[dd], o[gh][dd]);
      }
    }
  }
#pragma unroll
  for (int gh = 0; gh < G; gh++) {
    float *dst = a.part + (((size_t)i * a.hq + hk * G + gh) * a.max_parts + part) * (HD + 2);
    if (lane == 0) { dst[0] = m_run[gh]; dst[1] = l_run[gh]; }
#pragma unroll
    for (int dd = 0; dd < DPL; dd++) dst[2 + lane * DPL + dd] = o[gh][dd];
  }
}

// grid (rows, hq); block HD threads.  Merges the row's parts in ascending order.
template <typename T, int HD>
__global__ void attn_combine_kernel(AttnArgs a) {
  const int i = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
  const int p = a.base + a.depth[i];
  const int n_parts = p / kAttnPart + 1;
  const float *src = a.part + ((size_t)i * a.hq + h) * a.max_parts * (HD + 2);
  float m = src[0];
  for (int t = 1; t < n_parts; t++) m = fmaxf(m, src[(size_t)t * (HD + 2)]);
  float l = 0.f, o = 0.f;
  for (int t = 0; t < n_parts; t++) {
    const float *s = src + (size_t)t * (HD + 2);
    const float w = expf(s[0] - m);
    l += s[1] * w;
    o += s[2 + d] * w;
  }
  ((T *)a.out)[((size_t)i * a.hq + h) * HD + d] = from_f32<T>(o / l);
}

template <typename T, int HD, int G>
static hipError_t launch_thg(const AttnArgs &a, int n_parts, hipStream_t st) {
  hipLaunchKernelGGL((attn_part_kernel<T, HD, G>), dim3(a.rows, a.hkv, n_parts), dim3(64), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_combine_kernel<T, HD>), dim3(a.rows, a.hq), dim3(HD), 0, st, a);
  return hipGetLastError();
}
template <typename T, int HD>
static hipError_t launch_th(const AttnArgs &a, int n_parts, hipStream_t st) {
  switch (a.hq / a.hkv) {
    case 1: return launch_thg<T, HD, 1>(a, n_parts, st);
    case 2: return launch_thg<T, HD, 2>(a, n_parts, st);
    case 4: return launch_thg<T, HD, 4>(a, n_parts, st);
    case 8: return launch_thg<T, HD, 8>(a, n_parts, st);
    default: return hipErrorInvalidValue;
  }
}

// max_pos: largest key position any row attends to (host-known bound: base + max depth).
hipError_t launch_attention(int dtype, const AttnArgs &a, int max_pos, hipStream_t st) {
  if (a.rows < 1 || a.hkv < 1 || a.hq % a.hkv != 0) return hipErrorInvalidValue;
  const int n_parts = max_pos / kAttnPart + 1;
  if (n_parts > a.max_parts) return hipErrorInvalidValue;
  if (a.hd == 128) return dtype == 1 ? launch_th<bf16_t, 128>(a, n_parts, st) : launch_th<float, 128>(a, n_parts, st);
  if (a.hd == 64) return dtype == 1 ? launch_th<bf16_t, 64>(a, n_parts, st) : launch_th<float, 64>(a, n_parts, st);
  return hipErrorInvalidValue;
}

}  // namespace spec
