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

constexpr int kRowThreads = 256;

// ---- rotary table ------------------------------------------------------------------------
__global__ void rope_table_kernel(const int *pos, int rows, int half, double log2_theta, float2 *table) {
  const int i = blockIdx.x, j = threadIdx.x;
  if (i >= rows || j >= half) return;
  // angle = pos * theta^(-j/half), formed in double so that large positions keep their phase
  const double inv = exp2(-(double)j / (double)half * log2_theta);
  const double ang = (double)pos[i] * inv;
  double s, c;
  sincos(ang, &s, &c);
  table[i * half + j] = make_float2((float)c, (float)s);
}

hipError_t launch_rope_table(const int *pos, int rows, int head_dim, float theta, float2 *table, hipStream_t st) {
  if (rows < 1 || head_dim < 2 || head_dim > 512) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rope_table_kernel, dim3(rows), dim3(head_dim / 2), 0, st, pos, rows, head_dim / 2,
                     log2((double)theta), table);
  return hipGetLastError();
}

// ---- shared tail: h_row already holds this thread's fp32 values (each thread re-reads only the
// columns it wrote itself, so no barrier is needed for them); ss is the thread's sum of squares.
template <typename T>
__device__ __forceinline__ void finish_row(float ss, int d, const T *norm_w, float eps, const float *h_row, T *x_row,
                                           float *sh) {
  if (norm_w == nullptr) {
    for (int c = threadIdx.x; c < d; c += kRowThreads) x_row[c] = from_f32<T>(h_row[c]);
    return;
  }
  const float tot = block_sum(ss, sh);
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += kRowThreads) x_row[c] = from_f32<T>(h_row[c] * r * to_f32(norm_w[c]));
}

template <typename T>
__global__ __launch_bounds__(kRowThreads) void embed_norm_kernel(const T *embed, const int *token, int d, const T *norm_w,
                                                                 float eps, float *h, T *x) {
  __shared__ float sh[16];
  const int i = blockIdx.x;
  const T *src = embed + (size_t)token[i] * d;
  float *h_row = h + (size_t)i * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += kRowThreads) {
    const float v = to_f32(src[c]);
    h_row[c] = v;
    ss += v * v;
  }
  finish_row<T>(ss, d, norm_w, eps, h_row, x + (size_t)i * d, sh);
}

hipError_t launch_embed_norm(int dtype, const void *embed, const int *token, int rows, int d, const void *norm_w,
                             float eps, float *h, void *x, hipStream_t st) {
  if (rows < 1 || d < 1) return hipErrorInvalidValue;
  if (dtype == 1)
    hipLaunchKernelGGL(embed_norm_kernel<bf16_t>, dim3(rows), dim3(kRowThreads), 0, st, (const bf16_t *)embed, token, d,
                       (const bf16_t *)norm_w, eps, h, (bf16_t *)x);
  else
    hipLaunchKernelGGL(embed_norm_kernel<float>, dim3(rows), dim3(kRowThreads), 0, st, (const float *)embed, token, d,
                       (const float *)norm_w, eps, h, (float *)x);
  return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(kRowThreads) void concat_feat_embed_kernel(const T *feat, const int *src_row, const T *embed,
                                                                        const int *token, int d, T *xcat) {
  const int i = blockIdx.x;
  const T *f = feat + (size_t)(src_row ? src_row[i] : i) * d;
  const T *e = embed + (size_t)token[i] * d;
  T *o = xcat + (size_t)i * 2 * d;
  for (int c = threadIdx.x; c < d; c += kRowThreads) { o[c] = f[c]; o[d + c] = e[c]; }
}

hipError_t launch_concat_feat_embed(int dtype, const void *feat, const int *src_row, const void *embed,
                                    const int *token, int rows, int d, void *xcat, hipStream_t st) {
  if (rows < 1) return hipErrorInvalidValue;
  if (dtype == 1)
    hipLaunchKernelGGL(concat_feat_embed_kernel<bf16_t>, dim3(rows), dim3(kRowThreads), 0, st, (const bf16_t *)feat, src_row,
                       (const bf16_t *)embed, token, d, (bf16_t *)xcat);
  else
    hipLaunchKernelGGL(concat_feat_embed_kernel<float>, dim3(rows), dim3(kRowThreads), 0, st, (const float *)feat, src_row,
                       (const float *)embed, token, d, (float *)xcat);
  return hipGetLastError();
}

// ---- split sum (+ residual) + RMSNorm ------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kRowThreads) void reduce_add_norm_kernel(const float *part, int n_split, int m_pad, int ldp,
                                                                      int d, int residual, const T *norm_w, float eps,
                                                                      float *h, T *x) {
  __shared__ float sh[16];
  const int i = blockIdx.x;
  float *h_row = h + (size_t)i * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += kRowThreads) {
    float acc = part[(size_t)i * ldp + c];
    for (int s = 1; s < n_split; s++) acc += part[((size_t)s * m_pad + i) * ldp + c];   // fixed split order
    const float v = residual ? h_row[c] + acc : acc;
    h_row[c] = v;
    ss += v * v;
  }
  finish_row<T>(ss, d, norm_w, eps, h_row, x + (size_t)i * d, sh);
}

hipError_t launch_reduce_add_norm(int dtype, const float *part, int n_split, int m_pad, int ldp, int rows, int d,
                                  int residual, const void *norm_w, float eps, float *h, void *x, hipStream_t st) {
  if (rows < 1 || d < 1) return hipErrorInvalidValue;
  if (dtype == 1)
    hipLaunchKernelGGL(reduce_add_norm_kernel<bf16_t>, dim3(rows), dim3(kRowThreads), 0, st, part, n_split, m_pad, ldp, d,
                       residual, (const bf16_t *)norm_w, eps, h, (bf16_t *)x);
  else
    hipLaunchKernelGGL(reduce_add_norm_kernel<float>, dim3(rows), dim3(kRowThreads), 0, st, part, n_split, m_pad, ldp, d,
                       residual, (const float *)norm_w, eps, h, (float *)x);
  return hipGetLastError();
}

// ---- split sum + rotary + KV-cache write ----------------------------------------------------
// grid (rows, hq + 2*hkv); block hd/2 threads; thread j owns the rotary plane (j, j + hd/2).
template <typename T>
__global__ void reduce_rope_kv_kernel(const float *part, int n_split, int m_pad, int ldp, int hq, int hkv, int hd,
                                      const float2 *rope, const int *slot, float *q, T *kcache, T *vcache) {
  const int i = blockIdx.x, head = blockIdx.y, j = threadIdx.x, half = hd >> 1;
  const int col = head * hd + j;                       // q heads, then k heads, then v heads: the GEMM's column order
  float a = part[(size_t)i * ldp + col], b = part[(size_t)i * ldp + col + half];
  for (int s = 1; s < n_split; s++) {
    a += part[((size_t)s * m_pad + i) * ldp + col];
    b += part[((size_t)s * m_pad + i) * ldp + col + half];
  }
  if (head >= hq + hkv) {                              // value head: stored as is
    T *dst = vcache + ((size_t)slot[i] * hkv + (head - hq - hkv)) * hd;
    dst[j] = from_f32<T>(a);
    dst[j + half] = from_f32<T>(b);
    return;
  }
  const float2 cs = rope[i * half + j];
  const float ra = a * cs.x - b * cs.y, rb = b * cs.x + a * cs.y;
  if (head < hq) {                                     // query head: kept in fp32, it is read once and never cached
    float *dst = q + ((size_t)i * hq + head) * hd;
    dst[j] = ra;
    dst[j + half] = rb;
  } else {
    T *dst = kcache + ((size_t)slot[i] * hkv + (head - hq)) * hd;
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
  float g = part[(size_t)i * ldp + c], u = part[(size_t)i * ldp + f + c];
  for (int s = 1; s < n_split; s++) {
    g += part[((size_t)s * m_pad + i) * ldp + c];
    u += part[((size_t)s * m_pad + i) * ldp + f + c];
  }
  act[(size_t)i * f + c] = from_f32<T>(g / (1.0f + expf(-g)) * u);
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
