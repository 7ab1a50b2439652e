// Row-wise kernels around the weight-streaming GEMMs: embedding gather, RMSNorm,
// rotary embedding + KV-cache write, SwiGLU, residual add.  Each also folds in the
// fixed-order sum over the GEMM's K splits, so a split-K projection costs no extra pass.
// All arithmetic is fp32; storage type T is fp32 or bf16.
//
// Every output row depends only on its own input row (and the split count, which is a
// function of the matrix shape), so results are bit-identical for a token whether it is
// processed alone or as one row of a tree.
#include "common.h"
#include "kernels.h"

namespace spec {

constexpr int kRowThreads = 256;      // threads of the elementwise kernels
constexpr int kNormThreads = 1024;    // threads of the kernels that hold one row per workgroup

// ---- rotary table: cos/sin of pos[i] * theta^(-2j/hd) for j < hd/2 ------------------------
// (cos, sin) of pos * theta^(-j/half), the angle formed in double so that large positions keep their phase
__device__ __forceinline__ float2 rope_entry(int pos, int j, int half, double log2_theta) {
  const double inv = exp2(-(double)j / (double)half * log2_theta);
  const double ang = (double)pos * inv;
  double s, c;
  sincos(ang, &s, &c);
  return make_float2((float)c, (float)s);
}
// The kernels that open a forward (one workgroup per row) also fill the row's part of the rotary table, which saves a launch.
struct RopeFill { const int *pos; int half; double log2_theta; float2 *table; };   // table == nullptr: nothing to fill
__device__ __forceinline__ void rope_fill_row(const RopeFill &r, int i) {
  if (r.table != nullptr && (int)threadIdx.x < r.half) r.table[i * r.half + threadIdx.x] = rope_entry(r.pos[i], threadIdx.x, r.half, r.log2_theta);
}
static RopeFill make_rope_fill(const int *pos, int head_dim, float theta, float2 *table) {
  return RopeFill{pos, head_dim / 2, log2((double)theta), table};
}

// ---- row kernels that end in an RMSNorm: one workgroup per row, the whole row held in registers ----
// Thread t owns the 4-column groups t, t + 1024, ... (PER of them, guarded), so all global loads of a
// row are independent 16-byte loads issued up front, and the row is written exactly once.  With 1024
// threads a 4096-wide row is one group per thread: the kernel is three dependent memory round trips.
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

template <typename T> __device__ __forceinline__ f32x4_t load4(const T *p);
template <> __device__ __forceinline__ f32x4_t load4<float>(const float *p) { return *(const f32x4_t *)p; }
template <> __device__ __forceinline__ f32x4_t load4<bf16_t>(const bf16_t *p) {
  const uint2 u = *(const uint2 *)p;
  return f32x4_t{__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                 __uint_as_float(u.y & 0xFFFF0000u)};
}
template <typename T> __device__ __forceinline__ void store4(T *p, f32x4_t v);
template <> __device__ __forceinline__ void store4<float>(float *p, f32x4_t v) { *(f32x4_t *)p = v; }
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t *p, f32x4_t v) {
  uint2 u;
  u.x = (uint32_t)f32_to_bf16_bits(v.x) | ((uint32_t)f32_to_bf16_bits(v.y) << 16);
  u.y = (uint32_t)f32_to_bf16_bits(v.z) | ((uint32_t)f32_to_bf16_bits(v.w) << 16);
  *(uint2 *)p = u;
}

template <typename T, int PER>
__device__ __forceinline__ void finish_row(f32x4_t (&v)[PER], int d, const T *norm_w, float eps, float *h_row, T *x_row,
                                           float *sh) {
  // the norm weights are requested before the row-wide reduction, so that their latency hides behind it
  f32x4_t nw[PER];
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = (e * kNormThreads + threadIdx.x) * 4;
    nw[e] = (norm_w != nullptr && c < d) ? load4<T>(norm_w + c) : f32x4_t{1.f, 1.f, 1.f, 1.f};
  }
  float ss = 0.f;
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = (e * kNormThreads + threadIdx.x) * 4;
    if (c < d) {
      *(f32x4_t *)(h_row + c) = v[e];
      ss += v[e].x * v[e].x + v[e].y * v[e].y + v[e].z * v[e].z + v[e].w * v[e].w;
    }
  }
  float r = 1.f;
  if (norm_w != nullptr) r = 1.0f / sqrtf(block_sum(ss, sh) / (float)d + eps);
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = (e * kNormThreads + threadIdx.x) * 4;
    if (c < d) {
      f32x4_t o = v[e];
      if (norm_w != nullptr) o = o * r * nw[e];
      store4<T>(x_row + c, o);
    }
  }
}

template <typename T, int PER>
__global__ __launch_bounds__(kNormThreads) void embed_norm_kernel(const T *embed, const int *token, int d, const T *norm_w,
                                                                 float eps, float *h, T *x, RopeFill rf) {
  __shared__ float sh[16];
  const int i = blockIdx.x;
  rope_fill_row(rf, i);
  const T *src = embed + (size_t)token[i] * d;
  f32x4_t v[PER];
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = (e * kNormThreads + threadIdx.x) * 4;
    v[e] = c < d ? load4<T>(src + c) : f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  finish_row<T, PER>(v, d, norm_w, eps, h + (size_t)i * d, x + (size_t)i * d, sh);
}

template <typename T, int PER>
static void embed_norm_launch(const void *embed, const int *token, int rows, int d, const void *norm_w, float eps, float *h,
                              void *x, const RopeFill &rf, hipStream_t st) {
  hipLaunchKernelGGL((embed_norm_kernel<T, PER>), dim3(rows), dim3(kNormThreads), 0, st, (const T *)embed, token, d,
                     (const T *)norm_w, eps, h, (T *)x, rf);
}

hipError_t launch_embed_norm(int dtype, const void *embed, const int *token, int rows, int d, const void *norm_w,
                             float eps, float *h, void *x, hipStream_t st, const int *pos, int head_dim, float theta, float2 *table) {
  if (rows < 1 || d < 4 || d % 4 || d > kNormThreads * 4 * 4 || (table != nullptr && (head_dim < 2 || head_dim / 2 > kNormThreads)))
    return hipErrorInvalidValue;
  const RopeFill rf = make_rope_fill(pos, head_dim, theta, table);
  const int per = (d + kNormThreads * 4 - 1) / (kNormThreads * 4);
  if (dtype == 1) {
    if (per <= 1) embed_norm_launch<bf16_t, 1>(embed, token, rows, d, norm_w, eps, h, x, rf, st);
    else if (per <= 2) embed_norm_launch<bf16_t, 2>(embed, token, rows, d, norm_w, eps, h, x, rf, st);
    else embed_norm_launch<bf16_t, 4>(embed, token, rows, d, norm_w, eps, h, x, rf, st);
  } else {
    if (per <= 1) embed_norm_launch<float, 1>(embed, token, rows, d, norm_w, eps, h, x, rf, st);
    else if (per <= 2) embed_norm_launch<float, 2>(embed, token, rows, d, norm_w, eps, h, x, rf, st);
    else embed_norm_launch<float, 4>(embed, token, rows, d, norm_w, eps, h, x, rf, st);
  }
  return hipGetLastError();
}

// One workgroup per row; 16-byte pieces, all loads of a thread issued before its stores.
template <typename T>
__global__ __launch_bounds__(kRowThreads) void concat_feat_embed_kernel(const T *feat, const int *src_row, const T *embed,
                                                                        const int *token, int d, T *xcat, RopeFill rf) {
  typedef __attribute__((ext_vector_type(4))) uint32_t piece_t;
  constexpr int MAXP = 4;                                   // pieces per thread and half handled per pass
  const int i = blockIdx.x;
  rope_fill_row(rf, i);
  const piece_t *f = (const piece_t *)(feat + (size_t)(src_row ? src_row[i] : i) * d);
  const piece_t *e = (const piece_t *)(embed + (size_t)token[i] * d);
  piece_t *o = (piece_t *)(xcat + (size_t)i * 2 * d);
  const int np = d * (int)sizeof(T) / 16;                   // pieces per half (d * sizeof(T) is a multiple of 16)
  for (int c0 = 0; c0 < np; c0 += MAXP * kRowThreads) {
    piece_t a[MAXP], b[MAXP];
#pragma unroll
    for (int u = 0; u < MAXP; u++) {
      const int c = min(c0 + u * kRowThreads + (int)threadIdx.x, np - 1);
      a[u] = f[c]; b[u] = e[c];
    }
#pragma unroll
    for (int u = 0; u < MAXP; u++) {
      const int c = c0 + u * kRowThreads + (int)threadIdx.x;
      if (c < np) { o[c] = a[u]; o[np + c] = b[u]; }
    }
  }
}

hipError_t launch_concat_feat_embed(int dtype, const void *feat, const int *src_row, const void *embed,
                                    const int *token, int rows, int d, void *xcat, hipStream_t st, const int *pos, int head_dim, float theta,
                                    float2 *table) {
  if (rows < 1 || (table != nullptr && (head_dim < 2 || head_dim / 2 > kRowThreads))) return hipErrorInvalidValue;
  const RopeFill rf = make_rope_fill(pos, head_dim, theta, table);
  if (dtype == 1)
    hipLaunchKernelGGL(concat_feat_embed_kernel<bf16_t>, dim3(rows), dim3(kRowThreads), 0, st, (const bf16_t *)feat, src_row,
                       (const bf16_t *)embed, token, d, (bf16_t *)xcat, rf);
  else
    hipLaunchKernelGGL(concat_feat_embed_kernel<float>, dim3(rows), dim3(kRowThreads), 0, st, (const float *)feat, src_row,
                       (const float *)embed, token, d, (float *)xcat, rf);
  return hipGetLastError();
}

// ---- split sum (+ residual) + RMSNorm ------------------------------------------------------
template <typename T, int PER>
__global__ __launch_bounds__(kNormThreads) void reduce_add_norm_kernel(const float *part, int n_split, int m_pad, int ldp,
                                                                      int d, int residual, const T *norm_w, float eps,
                                                                      float *h, T *x) {
  __shared__ float sh[16];
  const int i = blockIdx.x;
  float *h_row = h + (size_t)i * d;
  f32x4_t v[PER];
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = (e * kNormThreads + threadIdx.x) * 4;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    if (c < d) {
      // all loads first (independent, clamped to a valid split), then the sum in ascending split order
      f32x4_t p[8];
      const f32x4_t res = *(const f32x4_t *)(h_row + c);
#pragma unroll
      for (int s = 0; s < 8; s++) p[s] = *(const f32x4_t *)(part + ((size_t)(s < n_split ? s : 0) * m_pad + i) * ldp + c);
      acc = p[0];
#pragma unroll
      for (int s = 1; s < 8; s++) {
        const float k = s < n_split ? 1.f : 0.f;            // absent splits add exactly zero
        acc += p[s] * k;
      }
      for (int s = 8; s < n_split; s++) acc += *(const f32x4_t *)(part + ((size_t)s * m_pad + i) * ldp + c);
      if (residual) acc = res + acc;
    }
    v[e] = acc;
  }
  finish_row<T, PER>(v, d, norm_w, eps, h_row, x + (size_t)i * d, sh);
}

template <typename T, int PER>
static void reduce_add_norm_launch(const float *part, int n_split, int m_pad, int ldp, int rows, int d, int residual,
                                   const void *norm_w, float eps, float *h, void *x, hipStream_t st) {
  hipLaunchKernelGGL((reduce_add_norm_kernel<T, PER>), dim3(rows), dim3(kNormThreads), 0, st, part, n_split, m_pad, ldp, d,
                     residual, (const T *)norm_w, eps, h, (T *)x);
}

hipError_t launch_reduce_add_norm(int dtype, const float *part, int n_split, int m_pad, int ldp, int rows, int d,
                                  int residual, const void *norm_w, float eps, float *h, void *x, hipStream_t st) {
  if (rows < 1 || d < 4 || d % 4 || ldp % 4 || d > kNormThreads * 4 * 4) return hipErrorInvalidValue;
  const int per = (d + kNormThreads * 4 - 1) / (kNormThreads * 4);
#define SPEC_RAN(T, P) reduce_add_norm_launch<T, P>(part, n_split, m_pad, ldp, rows, d, residual, norm_w, eps, h, x, st)
  if (dtype == 1) {
    if (per <= 1) SPEC_RAN(bf16_t, 1); else if (per <= 2) SPEC_RAN(bf16_t, 2); else SPEC_RAN(bf16_t, 4);
  } else {
    if (per <= 1) SPEC_RAN(float, 1); else if (per <= 2) SPEC_RAN(float, 2); else SPEC_RAN(float, 4);
  }
#undef SPEC_RAN
  return hipGetLastError();
}

// ---- split sum + rotary + KV-cache write ----------------------------------------------------
// grid (rows, hq + 2*hkv); block hd/2 threads; thread j owns the rotary plane (j, j + hd/2).
template <typename T>
__global__ void reduce_rope_kv_kernel(const float *part, int n_split, int m_pad, int ldp, int hq, int hkv, int hd,
                                      const float2 *rope, const int *slot, float *q, T *kcache, T *vcache) {
  const int i = blockIdx.x, head = blockIdx.y, j = threadIdx.x, half = hd >> 1;
  const int col = head * hd + j;                       // q heads, then k heads, then v heads: the GEMM's column order
  // every load is issued before anything is used: partial sums, the row's cache slot, the rotation
  const int sl = slot[i];
  const float2 cs = head < hq + hkv ? rope[i * half + j] : make_float2(1.f, 0.f);
  float pa[8], pb[8];                                  // (clamped to a valid split; absent splits add exactly zero)
#pragma unroll
  for (int s = 0; s < 8; s++) {
    const size_t o = ((size_t)(s < n_split ? s : 0) * m_pad + i) * ldp + col;
    pa[s] = part[o]; pb[s] = part[o + half];
  }
  float a = pa[0], b = pb[0];
#pragma unroll
  for (int s = 1; s < 8; s++) {
    const float k = s < n_split ? 1.f : 0.f;
    a += pa[s] * k; b += pb[s] * k;
  }
  for (int s = 8; s < n_split; s++) {
    a += part[((size_t)s * m_pad + i) * ldp + col];
    b += part[((size_t)s * m_pad + i) * ldp + col + half];
  }
  if (head >= hq + hkv) {                              // value head: stored as is
    T *dst = vcache + ((size_t)sl * hkv + (head - hq - hkv)) * hd;
    dst[j] = from_f32<T>(a);
    dst[j + half] = from_f32<T>(b);
    return;
  }
  const float ra = rope_first(a, b, cs), rb = rope_second(a, b, cs);
  if (head < hq) {                                     // query head: kept in fp32, it is read once and never cached
    float *dst = q + ((size_t)i * hq + head) * hd;
    dst[j] = ra;
    dst[j + half] = rb;
  } else {
    T *dst = kcache + ((size_t)sl * hkv + (head - hq)) * hd;
    dst[j] = from_f32<T>(ra);
    dst[j + half] = from_f32<T>(rb);
  }
}

hipError_t launch_reduce_rope_kv(int dtype, const float *part, int n_split, int m_pad, int ldp, int rows, int hq, int hkv,
                                 int hd, const float2 *rope, const int *slot, void *q, void *kcache, void *vcache,
                                 hipStream_t st) {
  if (rows < 1 || (hd & 1) || hd > 512) return hipErrorInvalidValue;
  dim3 grid(rows, hq + 2 * hkv), block(hd / 2);
  if (dtype == 1)
    hipLaunchKernelGGL(reduce_rope_kv_kernel<bf16_t>, grid, block, 0, st, part, n_split, m_pad, ldp, hq, hkv, hd, rope, slot,
                       (float *)q, (bf16_t *)kcache, (bf16_t *)vcache);
  else
    hipLaunchKernelGGL(reduce_rope_kv_kernel<float>, grid, block, 0, st, part, n_split, m_pad, ldp, hq, hkv, hd, rope, slot,
                       (float *)q, (float *)kcache, (float *)vcache);
  return hipGetLastError();
}

// ---- split sum + SwiGLU ---------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kRowThreads) void reduce_swiglu_kernel(const float *part, int n_split, int m_pad, int ldp, int f,
                                                                    T *act) {
  const int i = blockIdx.y;
  const int c = blockIdx.x * kRowThreads + threadIdx.x;
  if (c >= f) return;
  // the partial sums follow the rows of the packed gate/up matrix: per 16 columns, 16 gate sums and then 16 up sums
  const int cg = (c >> 4) * 32 + (c & 15), cu = cg + 16;
  float g = part[(size_t)i * ldp + cg], u = part[(size_t)i * ldp + cu];
  for (int s = 1; s < n_split; s++) {
    g += part[((size_t)s * m_pad + i) * ldp + cg];
    u += part[((size_t)s * m_pad + i) * ldp + cu];
  }
  act[(size_t)i * f + c] = from_f32<T>(silu_mul(g, u));
}

hipError_t launch_reduce_swiglu(int dtype, const float *part, int n_split, int m_pad, int ldp, int rows, int f, void *act,
                                hipStream_t st) {
  if (rows < 1) return hipErrorInvalidValue;
  dim3 grid((f + kRowThreads - 1) / kRowThreads, rows);
  if (dtype == 1)
    hipLaunchKernelGGL(reduce_swiglu_kernel<bf16_t>, grid, dim3(kRowThreads), 0, st, part, n_split, m_pad, ldp, f, (bf16_t *)act);
  else
    hipLaunchKernelGGL(reduce_swiglu_kernel<float>, grid, dim3(kRowThreads), 0, st, part, n_split, m_pad, ldp, f, (float *)act);
  return hipGetLastError();
}

// ---- index tables of a causal chain of rows (prefill chunks, the draft's root step) -----------
__global__ void chain_rows_kernel(int base, int rows, int pos_offset, int *pos, int *slot, int *depth) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows) return;
  slot[i] = base + i;
  pos[i] = base + i + pos_offset;
  depth[i] = i;
}
hipError_t launch_chain_rows(int base, int rows, int pos_offset, int *pos, int *slot, int *depth, hipStream_t st) {
  if (rows < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(chain_rows_kernel, dim3((rows + 63) / 64), dim3(64), 0, st, base, rows, pos_offset, pos, slot, depth);
  return hipGetLastError();
}

}  // namespace spec
