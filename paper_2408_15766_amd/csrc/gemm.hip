// Weight-streaming skinny GEMM for gfx950:  P[s][i][col] = sum_{k in split s} X[i][k] * W[col][k]
//
// Every projection of the decode path (QKV, O, gate/up, down, draft fc, LM head)
// multiplies a handful of token rows (M <= 128: the verified tree, the draft
// frontier, or one row in plain decoding) by a weight matrix that is read once.
// The step is bound by HBM bandwidth (about 2*M flop per weight byte pair), so
// the design goal is to keep many 16-byte weight loads in flight per lane and
// never touch a weight twice; the matrix cores are used only because M ~ 60
// is too much for the vector ALUs at that rate.
//
// Layout of one MFMA step (v_mfma_f32_32x32x16_bf16 / 32x32x2_f32):
//   A operand = 32 token rows   x k-slice   (from the X slab staged in LDS)
//   B operand = 32 weight rows  x k-slice   (straight from global memory)
//   D         = lane (c = lane%32, g = lane/32) holds weight row c of the
//               wave's 32-row block for tokens 8*(v/4) + 4*g + v%4, v = 0..15
// Lane (c, g) loads 128 contiguous bytes of weight row c per iteration (eight
// 16-byte loads); the k indices of one MFMA are therefore not contiguous, which
// is harmless because A and B are indexed by the same (g, element) pair.
//
// Each wave owns one 32-row block of W for the workgroup's K range and all
// token blocks; the four waves of a workgroup share the X slab.  Weight loads
// run two iterations ahead through a three-stage register ring; the X slab is
// double-buffered in LDS and prefetched one slab ahead through registers.
//
// Determinism: the value of P[s][i][col] depends only on row i of X, row col of
// W and the K split, never on M, on the position of the row in its tile or on
// other rows, so a token computes bit-identical results alone (plain decoding)
// or inside a tree.
#include "common.h"
#include "kernels.h"

namespace spec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;   // native vector: stays in registers (SSA), unlike HIP's u32x4_t struct

constexpr int kGemmWaves = 4;                       // waves per workgroup
constexpr int kGemmThreads = kGemmWaves * kWave;
constexpr int kLaneBytes = 128;                     // contiguous weight bytes per lane per iteration
constexpr int kSlabIters = 2;                       // iterations per LDS slab
constexpr int kSlabRowBytes = 2 * kLaneBytes * kSlabIters;   // 512 B of k per token row per slab
constexpr int kSlabStride = kSlabRowBytes + 16;     // +16 B: conflict-free 16-byte LDS reads

template <typename T> struct GemmTraits;
template <> struct GemmTraits<bf16_t> { static constexpr int kEpl = 8; };   // elements per 16 bytes
template <> struct GemmTraits<float>  { static constexpr int kEpl = 4; };

__device__ __forceinline__ void mfma_step(f32x16_t &acc, const u32x4_t &x, const u32x4_t &w, bf16_t) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, x), __builtin_bit_cast(bf16x8_t, w), acc, 0, 0, 0);
}
__device__ __forceinline__ void mfma_step(f32x16_t &acc, const u32x4_t &x, const u32x4_t &w, float) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(x.x), __uint_as_float(w.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(x.y), __uint_as_float(w.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(x.z), __uint_as_float(w.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(x.w), __uint_as_float(w.w), acc, 0, 0, 0);
}

template <typename T, int TB>
__global__ __launch_bounds__(kGemmThreads, TB <= 2 ? 2 : 1) void gemm_stream_kernel(GemmArgs a) {
  constexpr int EPL = GemmTraits<T>::kEpl;
  constexpr int KI = 2 * kLaneBytes / (int)sizeof(T);         // k elements per iteration
  constexpr int XCH = TB * 32 * (kSlabRowBytes / 16) / kGemmThreads;   // 16-byte X chunks per thread per slab
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int kSlabBytes = TB * 32 * kSlabStride;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, g = lane >> 5;

  // which 32-row block of which weight segment this wave streams (no dynamic indexing of the
  // argument struct: that would push it to private memory)
  // A wave past the last block recomputes the last block and stores nothing, so that every wave
  // runs the same branch-free loop and the same barriers.
  const int blk_raw = blockIdx.x * kGemmWaves + wave;
  const bool active = blk_raw < a.total_blocks;
  const int blk = active ? blk_raw : a.total_blocks - 1;
  const int e0 = a.seg_blocks[0], e1 = e0 + (a.nseg > 1 ? a.seg_blocks[1] : 0);
  const int seg = blk < e0 ? 0 : (blk < e1 ? 1 : 2);
  const int b0 = seg == 0 ? 0 : (seg == 1 ? e0 : e1);
  const int seg_rows = seg == 0 ? a.seg_rows[0] : (seg == 1 ? a.seg_rows[1] : a.seg_rows[2]);
  const int seg_col0 = seg == 0 ? a.seg_col0[0] : (seg == 1 ? a.seg_col0[1] : a.seg_col0[2]);
  const void *seg_w = seg == 0 ? a.seg_w[0] : (seg == 1 ? a.seg_w[1] : a.seg_w[2]);
  const int row = (blk - b0) * 32 + c;
  const int row_c = min(row, seg_rows - 1);
  const char *wrow = (const char *)seg_w + (size_t)row_c * (size_t)a.in * sizeof(T);

  // K splits are balanced to within one slab: split y covers slabs [y*S/n, (y+1)*S/n)
  constexpr int KSLAB = kSlabRowBytes / (int)sizeof(T);
  const int n_slabs_total = (a.in + KSLAB - 1) / KSLAB;
  const int k_begin = (int)((long long)blockIdx.y * n_slabs_total / a.n_split) * KSLAB;
  const int k_end = min(a.in, (int)((long long)(blockIdx.y + 1) * n_slabs_total / a.n_split) * KSLAB);
  const int n_iter = (k_end - k_begin + KI - 1) / KI;
  const int n_slab = (n_iter + kSlabIters - 1) / kSlabIters;

  f32x16_t acc[TB];
#pragma unroll
  for (int t = 0; t < TB; t++)
#pragma unroll
    for (int v = 0; v < 16; v++) acc[t][v] = 0.f;

  u32x4_t ring[3][8];
  u32x4_t xr[XCH];

  // Full iterations load without any guard, so nothing forces a wait between the load and its
  // use two iterations later.  Only a ragged last iteration (K range not a multiple of KI) takes
  // the guarded form, which zeroes the weight fragment beyond k_end; X never needs zeroing:
  // out-of-range X addresses are clamped to valid finite data that meets a zero weight or a
  // token row that is never stored.
  const int n_full = (k_end - k_begin) / KI;
  auto load_w = [&](u32x4_t (&dst)[8], int it) {
    const char *p = wrow + (size_t)(k_begin + it * KI + g * (KI / 2)) * sizeof(T);
#pragma unroll
    for (int j = 0; j < 8; j++) dst[j] = *(const u32x4_t *)(p + j * 16);
  };
  auto load_w_tail = [&](u32x4_t (&dst)[8], int it) {
    const int k = k_begin + it * KI + g * (KI / 2);
#pragma unroll
    for (int j = 0; j < 8; j++) {
      const int kk = k + j * EPL;
      const bool ok = kk < k_end;
      const u32x4_t v = *(const u32x4_t *)(wrow + (size_t)(ok ? kk : k_begin) * sizeof(T));
      dst[j] = ok ? v : u32x4_t{0u, 0u, 0u, 0u};
    }
  };
  const char *xbase = (const char *)a.x;
  auto load_x = [&](int slab) {
    const int k0 = k_begin + slab * kSlabIters * KI;
#pragma unroll
    for (int i = 0; i < XCH; i++) {
      const int q = tid + i * kGemmThreads;
      const int r = q / (kSlabRowBytes / 16), cc = q % (kSlabRowBytes / 16);
      const int kk = k0 + cc * EPL;
      xr[i] = *(const u32x4_t *)(xbase + ((size_t)(r < a.m ? r : 0) * a.ldx + (kk < k_end ? kk : k_begin)) * sizeof(T));
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XCH; i++) {
      const int q = tid + i * kGemmThreads;
      const int r = q / (kSlabRowBytes / 16), cc = q % (kSlabRowBytes / 16);
      *(u32x4_t *)(lds + buf * kSlabBytes + r * kSlabStride + cc * 16) = xr[i];
    }
  };
  auto compute = [&](const u32x4_t (&w)[8], int buf, int ii) {
    const unsigned char *base = lds + buf * kSlabBytes + c * kSlabStride + ii * (2 * kLaneBytes) + g * kLaneBytes;
#pragma unroll
    for (int j = 0; j < 8; j++) {
#pragma unroll
      for (int t = 0; t < TB; t++) {
        const u32x4_t xf = *(const u32x4_t *)(base + t * 32 * kSlabStride + j * 16);
        mfma_step(acc[t], xf, w[j], T{});
      }
    }
  };

  load_x(0);
#define SPEC_LOADW(R, IT)                                                    \
  { if ((IT) < n_full) load_w(ring[R], (IT)); else if ((IT) < n_iter) load_w_tail(ring[R], (IT)); }
  SPEC_LOADW(0, 0)
  SPEC_LOADW(1, 1)
  store_x(0);
  __syncthreads();

  // One slab = kSlabIters (2) iterations; the ring stage of iteration `it` is it % 3, so three
  // slabs (six iterations) form one period and are unrolled to keep register indices static.
  // Steady state: every load of the slab is a full, in-range iteration and a next slab exists,
  // so the body has no branch and the compiler can keep exact outstanding-load counts.
#define SPEC_FAST_SLAB(S, R0, R1, R2)                                        \
  {                                                                          \
    const int buf = (S) & 1;                                                 \
    load_x((S) + 1);                                                         \
    load_w(ring[R2], (S) * 2 + 2);                                           \
    __builtin_amdgcn_sched_barrier(0); /* keep the prefetches ahead of the MFMAs */ \
    compute(ring[R0], buf, 0);                                               \
    __builtin_amdgcn_sched_barrier(0);                                       \
    load_w(ring[R0], (S) * 2 + 3);                                           \
    __builtin_amdgcn_sched_barrier(0);                                       \
    compute(ring[R1], buf, 1);                                               \
    __builtin_amdgcn_sched_barrier(0);                                       \
    store_x(buf ^ 1);                                                        \
    __syncthreads();                                                         \
  }
#define SPEC_SLAB(S, R0, R1, R2)                                             \
  if ((S) < n_slab) {                                                        \
    const int buf = (S) & 1;                                                 \
    const bool more = (S) + 1 < n_slab;                                      \
    if (more) load_x((S) + 1);                                               \
    SPEC_LOADW(R2, (S) * 2 + 2)                                              \
    compute(ring[R0], buf, 0);                                               \
    SPEC_LOADW(R0, (S) * 2 + 3)                                              \
    if ((S) * 2 + 1 < n_iter) compute(ring[R1], buf, 1);                     \
    if (more) store_x(buf ^ 1);                                              \
    __syncthreads();                                                         \
  }
  const int n_steady = n_full >= 2 ? (n_full - 2) / 2 : 0;   // slabs S with 2S+3 < n_full (and so S+1 < n_slab)
  int s = 0;
  for (; s + 3 <= n_steady; s += 3) {
    SPEC_FAST_SLAB(s, 0, 1, 2)        // iterations 6q+0, 6q+1 ; loads 6q+2 -> stage 2, 6q+3 -> stage 0
    SPEC_FAST_SLAB(s + 1, 2, 0, 1)    // iterations 6q+2, 6q+3 ; loads 6q+4 -> stage 1, 6q+5 -> stage 2
    SPEC_FAST_SLAB(s + 2, 1, 2, 0)    // iterations 6q+4, 6q+5 ; loads 6q+6 -> stage 0, 6q+7 -> stage 1
  }
  for (; s < n_slab; s += 3) {
    SPEC_SLAB(s, 0, 1, 2)
    SPEC_SLAB(s + 1, 2, 0, 1)
    SPEC_SLAB(s + 2, 1, 2, 0)
  }
#undef SPEC_SLAB
#undef SPEC_FAST_SLAB
#undef SPEC_LOADW

  if (!active || row >= seg_rows) return;
  float *out = a.part + ((size_t)blockIdx.y * a.m_pad) * a.ldp + seg_col0 + row;
#pragma unroll
  for (int t = 0; t < TB; t++)
#pragma unroll
    for (int v = 0; v < 16; v++) {
      const int i = t * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
      if (i < a.m) out[(size_t)i * a.ldp] = acc[t][v];
    }
}

template <typename T>
static hipError_t launch_t(const GemmArgs &a, hipStream_t st) {
  const int tb = (a.m + 31) / 32;
  dim3 grid((a.total_blocks + kGemmWaves - 1) / kGemmWaves, a.n_split);
  const size_t lds = (size_t)2 * tb * 32 * kSlabStride;
  // the double-buffered slab exceeds the 64 KiB default for dynamic LDS from two token blocks on
  static bool attr_set = false;
  if (!attr_set) {
    const int big = 4 * 2 * 32 * kSlabStride;
    hipError_t e = hipFuncSetAttribute((const void *)gemm_stream_kernel<T, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, big);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_stream_kernel<T, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, big);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_stream_kernel<T, 3>, hipFuncAttributeMaxDynamicSharedMemorySize, big);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_stream_kernel<T, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, big);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  switch (tb) {
    case 1: hipLaunchKernelGGL((gemm_stream_kernel<T, 1>), grid, dim3(kGemmThreads), lds, st, a); break;
    case 2: hipLaunchKernelGGL((gemm_stream_kernel<T, 2>), grid, dim3(kGemmThreads), lds, st, a); break;
    case 3: hipLaunchKernelGGL((gemm_stream_kernel<T, 3>), grid, dim3(kGemmThreads), lds, st, a); break;
    case 4: hipLaunchKernelGGL((gemm_stream_kernel<T, 4>), grid, dim3(kGemmThreads), lds, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

int gemm_k_per_iter(int dtype) { return dtype == 1 ? 128 : 64; }
int gemm_k_per_slab(int dtype) { return kSlabIters * gemm_k_per_iter(dtype); }
int gemm_rows_per_group() { return 32 * kGemmWaves; }

hipError_t launch_gemm(int dtype, const GemmArgs &a, hipStream_t st) {
  if (a.m < 1 || a.m > 128 || a.nseg < 1 || a.nseg > 3 || a.n_split < 1 || a.in < 1) return hipErrorInvalidValue;
  if (a.n_split > (a.in + gemm_k_per_slab(dtype) - 1) / gemm_k_per_slab(dtype)) return hipErrorInvalidValue;   // no empty split
  return dtype == 1 ? launch_t<bf16_t>(a, st) : launch_t<float>(a, st);
}

}  // namespace spec
