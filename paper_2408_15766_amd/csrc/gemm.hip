// Weight-streaming skinny GEMM for gfx950:  P[s][i][col] = sum_{k in split s} X[i][k] * W[col][k]
//
// Every projection of the decode path (QKV, O, gate/up, down, draft fc, LM head)
// multiplies a handful of token rows (M <= 128 per tile: the verified tree, the draft
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
// Weights are read in the library's PACKED layout (pack_weight_kernel below): the
// matrix is cut into tiles of 32 rows x KI k-elements (8 KiB; KI = 128 bf16 / 64 fp32),
// tiles of one 32-row block are consecutive along k, and inside a tile the 16-byte piece
// that lane (c, g) needs for MFMA step j sits at byte j*1024 + lane*16.  One wave-wide
// load instruction therefore reads 1 KiB of consecutive bytes (eight full cache lines),
// and a wave streams one contiguous region from start to end: measured on MI355X this
// is worth ~1.4x in achieved HBM bandwidth over reading the same 16-byte pieces from a
// row-major matrix (64 partial lines per instruction).  Piece (c, g, j) of tile (rb, it)
// holds W[rb*32 + c][it*KI + g*KI/2 + j*EPL .. + EPL), zero beyond the matrix, so neither
// ragged rows nor a ragged K need a special path.  The k indices of one MFMA are not
// contiguous, which is harmless because A and B are indexed by the same (g, element) pair.
//
// Each wave owns one 32-row block of W for the workgroup's K range and all
// token blocks; the four waves of a workgroup share the X slab.  Which blocks a
// workgroup takes is the launch's choice (four adjacent ones, or fewer, spread so
// that every compute unit has a workgroup: launch_t).  Weight loads
// run kStages - 1 iterations ahead through a register ring; the X slab is
// double-buffered in LDS and prefetched one slab ahead through registers.
//
// Determinism: the value of P[s][i][col] depends only on row i of X, row col of
// W and the K split, never on M, on the position of the row in its tile or on
// other rows, so a token computes bit-identical results alone (plain decoding)
// or inside a tree.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace spec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;   // native vector: stays in registers (SSA), unlike HIP's u32x4_t struct

#ifndef SPEC_GEMM_WAVES
#define SPEC_GEMM_WAVES 4
#endif
#ifndef SPEC_GEMM_SLAB_ITERS
#define SPEC_GEMM_SLAB_ITERS 2
#endif
#ifndef SPEC_GEMM_STAGES
#define SPEC_GEMM_STAGES 3
#endif
constexpr int kGemmWaves = SPEC_GEMM_WAVES;         // waves per workgroup
constexpr int kStages = SPEC_GEMM_STAGES;           // register ring: weight loads run kStages - 1 iterations ahead
constexpr int kGemmThreads = kGemmWaves * kWave;
constexpr int kLaneBytes = 128;                     // contiguous weight bytes per lane per iteration
constexpr int kSlabIters = SPEC_GEMM_SLAB_ITERS;    // iterations per LDS slab
constexpr int kSlabRowBytes = 2 * kLaneBytes * kSlabIters;   // 512 B of k per token row per slab
constexpr int kSlabStride = kSlabRowBytes + 16;     // +16 B: conflict-free 16-byte LDS reads
constexpr int kTileBytes = 32 * 2 * kLaneBytes;     // one packed tile: 32 rows x 256 B of k

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

constexpr int gcd_ce(int a, int b) { return b == 0 ? a : gcd_ce(b, a % b); }
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

// SwiGLU epilogue of a block of the gate/up matrix.  Lane c < 16 holds the gate sums of column col = block * 16 + c
// and lane c + 16 the up sums of the same column and tokens.  Each finishes half of the values (the low lane the
// accumulator entries v < 8, the high lane v >= 8) after one exchange with its partner of the entries the partner
// finishes.  In phases (all exchanges, all activations, all neighbour shifts, all stores), so that the lane exchanges
// overlap instead of each waiting for the one before.  act: the block's first token row, column col.
template <typename T, int TB>
__device__ __forceinline__ void swiglu_epilogue(const f32x16_t (&acc)[TB], T *act, int f, int col, bool store, int m_loc, int c, int g) {
  const bool hi = c >= 16;
  float r[TB][8], nx[TB][8];
#pragma unroll
  for (int t = 0; t < TB; t++)
#pragma unroll
    for (int v8 = 0; v8 < 8; v8++) r[t][v8] = __shfl_xor(hi ? acc[t][v8] : acc[t][8 + v8], 16, 64);
#pragma unroll
  for (int t = 0; t < TB; t++)
#pragma unroll
    for (int v8 = 0; v8 < 8; v8++) {
      const float mine = hi ? acc[t][8 + v8] : acc[t][v8], other = r[t][v8];
      r[t][v8] = silu_mul(hi ? other : mine, hi ? mine : other);
    }
#pragma unroll
  for (int t = 0; t < TB; t++)
#pragma unroll
    for (int v8 = 0; v8 < 8; v8++) nx[t][v8] = __shfl_down(r[t][v8], 1, 64);
  const bool pairs = (f & 1) == 0, next = col + 1 < f;
#pragma unroll
  for (int t = 0; t < TB; t++)
#pragma unroll
    for (int v8 = 0; v8 < 8; v8++) {
      const int v = hi ? 8 + v8 : v8;
      const int i = t * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
      store_act(act + (size_t)i * f, r[t][v8], nx[t][v8], store && i < m_loc, pairs, next, c);
    }
}

template <typename T, int TB>
__global__ __launch_bounds__(kGemmThreads, (TB <= 2 && kStages <= 3) ? 2 : 1) void gemm_stream_kernel(GemmArgs a) {
  constexpr int EPL = GemmTraits<T>::kEpl;
  constexpr int KI = 2 * kLaneBytes / (int)sizeof(T);         // k elements per iteration
  constexpr int XCH = TB * 32 * (kSlabRowBytes / 16) / kGemmThreads;   // 16-byte X chunks per thread per slab
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int kSlabBytes = TB * 32 * kSlabStride;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, g = lane >> 5;

  // which 32-row block of which weight segment this wave streams (no dynamic indexing of the
  // argument struct: that would push it to private memory).
  // A wave past the last block recomputes the last block and stores nothing, so that every wave
  // runs the same branch-free loop and the same barriers.
  // SwiGLU mode streams the one gate/up matrix (see pack_gate_up_kernel): a block holds 16 gate rows in the lanes
  // c < 16 and the up rows of the same 16 columns in the lanes c >= 16; seg_rows[0] is the number of columns.
  const int bx = blockIdx.x, by = blockIdx.y, mt = 0;
  const int m_loc = a.m;                                       // (more than 128 rows go to gemm_tiled_kernel)
  const bool swiglu = a.act != nullptr;
  const int e0 = a.seg_blocks[0], e1 = e0 + (a.nseg > 1 ? a.seg_blocks[1] : 0);
  const int blk_raw = bx * a.blk_per_wg + wave * a.blk_per_wave;   // four adjacent blocks, or strided over more workgroups: see launch_t
  const bool active = blk_raw < a.total_blocks;
  const int blk = active ? blk_raw : a.total_blocks - 1;
  const int seg = blk < e0 ? 0 : (blk < e1 ? 1 : 2);
  const int b0 = seg == 0 ? 0 : (seg == 1 ? e0 : e1);
  const int seg_rows = seg == 0 ? a.seg_rows[0] : (seg == 1 ? a.seg_rows[1] : a.seg_rows[2]);
  const int seg_col0 = seg == 0 ? a.seg_col0[0] : (seg == 1 ? a.seg_col0[1] : a.seg_col0[2]);
  const void *seg_w = seg == 0 ? a.seg_w[0] : (seg == 1 ? a.seg_w[1] : a.seg_w[2]);
  const int row = (blk - b0) * 32 + c;

  // K splits are balanced to within one slab: split y covers slabs [y*S/n, (y+1)*S/n)
  const int n_it_total = (a.in + KI - 1) / KI;                         // tiles along k (K zero-padded to KI)
  const int n_slabs_total = (n_it_total + kSlabIters - 1) / kSlabIters;
  const int it_begin = (int)((long long)by * n_slabs_total / a.n_split) * kSlabIters;
  const int it_end = min(n_it_total, (int)((long long)(by + 1) * n_slabs_total / a.n_split) * kSlabIters);
  const int k_begin = it_begin * KI;
  const int n_iter = it_end - it_begin;
  const int n_slab = (n_iter + kSlabIters - 1) / kSlabIters;
  // A wave without a block of its own only helps to stage the X slabs (same barriers, no weight loads, no MFMAs).
  const int n_iter_w = __builtin_amdgcn_readfirstlane(active ? n_iter : 0);
  // this wave's stream: tiles it_begin .. it_end of row block (blk - b0), one contiguous region
  const char *wstream = (const char *)seg_w + ((size_t)(blk - b0) * n_it_total + it_begin) * (size_t)kTileBytes + lane * 16;

  f32x16_t acc[TB];
#pragma unroll
  for (int t = 0; t < TB; t++)
#pragma unroll
    for (int v = 0; v < 16; v++) acc[t][v] = 0.f;

  u32x4_t ring[kStages][8];
  u32x4_t xr[XCH];

  // Every tile is complete in the packed layout (zero-padded), so weight loads need no guard and
  // nothing forces a wait between a load and its use two iterations later.  X never needs
  // zeroing either: out-of-range X addresses are clamped to valid finite data that meets a zero
  // weight or a token row that is never stored.
  auto load_w = [&](u32x4_t (&dst)[8], int it) {
    const char *p = wstream + (size_t)it * kTileBytes;
#pragma unroll
    for (int j = 0; j < 8; j++) dst[j] = __builtin_nontemporal_load((const u32x4_t *)(p + j * 1024));   // read once: do not keep in cache
  };
  const char *xbase = (const char *)a.x + (size_t)mt * 128 * a.ldx * sizeof(T);
  auto load_x = [&](int slab) {
    const int k0 = k_begin + slab * kSlabIters * KI;
#pragma unroll
    for (int i = 0; i < XCH; i++) {
      const int q = tid + i * kGemmThreads;
      const int r = q / (kSlabRowBytes / 16), cc = q % (kSlabRowBytes / 16);
      const int kk = k0 + cc * EPL;
      xr[i] = *(const u32x4_t *)(xbase + ((size_t)(r < m_loc ? r : 0) * a.ldx + (kk < a.in ? kk : 0)) * sizeof(T));
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
#pragma unroll
  for (int it = 0; it < kStages - 1; it++)
    if (it < n_iter_w) load_w(ring[it], it);
  store_x(0);
  __syncthreads();

  // The ring stage of iteration `it` is it % kStages.  A slab is kSlabIters iterations, so kPeriod slabs
  // form one period of the stage pattern and are unrolled with compile-time stage indices
  // (P = slab index mod kPeriod).  Steady state (FAST): every load of the slab is a full, in-range
  // iteration and a next slab exists, so the body has no branch and the compiler keeps exact
  // outstanding-load counts; the remaining slabs take the guarded form.
  auto slab = [&](auto p_tag, auto fast_tag, int S) {
    constexpr int P = decltype(p_tag)::value;
    constexpr bool FAST = decltype(fast_tag)::value;
    if (!FAST && S >= n_slab) return;
    const int buf = S & 1;
    const bool more = FAST || S + 1 < n_slab;
    if (more) load_x(S + 1);
#pragma unroll
    for (int ii = 0; ii < kSlabIters; ii++) {
      constexpr int base_stage = (kSlabIters * P) % kStages;
      const int it = S * kSlabIters + ii;
      // stage indices are compile-time after unrolling
      const int st_use = (base_stage + ii) % kStages, st_load = (base_stage + ii + kStages - 1) % kStages;
      if (FAST || it + kStages - 1 < n_iter_w) load_w(ring[st_load], it + kStages - 1);
      __builtin_amdgcn_sched_barrier(0);                     // keep the prefetch ahead of the MFMAs
      if (FAST || it < n_iter_w) compute(ring[st_use], buf, ii);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (more) store_x(buf ^ 1);
    __syncthreads();
  };
  constexpr int kPeriod = kStages / gcd_ce(kStages, kSlabIters);
  auto period = [&](auto fast_tag, int S0) {
    static_for<kPeriod>([&](auto p_tag) { slab(p_tag, fast_tag, S0 + decltype(p_tag)::value); });
  };
  // slabs S whose last prefetch, iteration S*kSlabIters + kSlabIters - 1 + kStages - 1, is in range
  const int n_steady = n_iter_w >= kSlabIters + kStages - 1 ? (n_iter_w - kStages + 1) / kSlabIters : 0;
  int s = 0;
  for (; s + kPeriod <= n_steady; s += kPeriod) period(std::true_type{}, s);
  for (; s < n_slab; s += kPeriod) period(std::false_type{}, s);

  if (swiglu) {
    const int col = blk * 16 + (c & 15);
    swiglu_epilogue<T, TB>(acc, (T *)a.act + (size_t)mt * 128 * seg_rows + col, seg_rows, col, active && col < seg_rows, m_loc, c, g);
    return;
  }
  if (!active || row >= seg_rows) return;
  float *out = a.part + ((size_t)by * a.m_pad + (size_t)mt * 128) * a.ldp + seg_col0 + row;
#pragma unroll
  for (int t = 0; t < TB; t++)
#pragma unroll
    for (int v = 0; v < 16; v++) {
      const int i = t * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
      if (i < m_loc) store_through(&out[(size_t)i * a.ldp], acc[t][v]);
    }
}

// ---- more than 128 token rows (prefill) -------------------------------------------------------
// The same contraction when X has several 128-row tiles.  One launch covers all tiles; a workgroup owns
// (256 weight rows, one K split, one tile).  Here the matrix cores are the limit, and with one weight block
// per wave every MFMA would need its own token fragment from LDS (LDS bandwidth runs out first), so a wave
// streams TWO weight blocks and uses each fragment twice.  In SwiGLU mode the blocks are those of the gate/up
// matrix (gate rows in the lanes c < 16, up rows of the same columns in the lanes c >= 16) and the activation is
// formed in registers after one exchange between the two lane halves.  Tiles of the same weight rows
// take workgroup ids 8 apart inside a window of 8 * m_tiles ids: they run together on one XCD and share the
// weights through its L2 (default cache policy instead of the read-once hint).
template <typename T>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_tiled_kernel(GemmArgs a) {
  constexpr int TB = 4, WB = 2;
  constexpr int EPL = GemmTraits<T>::kEpl;
  constexpr int KI = 2 * kLaneBytes / (int)sizeof(T);
  constexpr int XCH = TB * 32 * (kSlabRowBytes / 16) / kGemmThreads;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int kSlabBytes = TB * 32 * kSlabStride;
  static_assert(kSlabIters == 2, "the two ring stages alternate with the two iterations of a slab");

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, g = lane >> 5;
  const int per = 8 * a.m_tiles;
  const int q = ((int)blockIdx.x / per) * 8 + ((int)blockIdx.x % 8);
  const int mt = ((int)blockIdx.x % per) / 8;
  if (q >= a.grid_x * a.n_split) return;                       // padding of the id space; whole workgroup
  const int bx = q % a.grid_x, by = q / a.grid_x;
  const int m_loc = min(a.m - mt * 128, 128);

  const bool swiglu = a.act != nullptr;
  const int e0 = a.seg_blocks[0], e1 = e0 + (a.nseg > 1 ? a.seg_blocks[1] : 0);
  const int unit = bx * kGemmWaves + wave;                     // pair of consecutive blocks
  bool active[WB]; int seg_rows[WB], seg_col0[WB], row[WB], blk_of[WB];
  const char *wstream[WB];
  const int n_it_total = (a.in + KI - 1) / KI;
  const int n_slabs_total = (n_it_total + kSlabIters - 1) / kSlabIters;
  const int it_begin = (int)((long long)by * n_slabs_total / a.n_split) * kSlabIters;
  const int it_end = min(n_it_total, (int)((long long)(by + 1) * n_slabs_total / a.n_split) * kSlabIters);
  const int k_begin = it_begin * KI;
  const int n_iter = it_end - it_begin;
  const int n_slab = (n_iter + kSlabIters - 1) / kSlabIters;
#pragma unroll
  for (int wb = 0; wb < WB; wb++) {
    const int blk_raw = unit * WB + wb;
    active[wb] = blk_raw < a.total_blocks;
    const int blk = active[wb] ? blk_raw : a.total_blocks - 1;
    blk_of[wb] = blk;
    const int seg = blk < e0 ? 0 : (blk < e1 ? 1 : 2);
    const int b0 = seg == 0 ? 0 : (seg == 1 ? e0 : e1);
    seg_rows[wb] = seg == 0 ? a.seg_rows[0] : (seg == 1 ? a.seg_rows[1] : a.seg_rows[2]);
    seg_col0[wb] = seg == 0 ? a.seg_col0[0] : (seg == 1 ? a.seg_col0[1] : a.seg_col0[2]);
    const void *seg_w = seg == 0 ? a.seg_w[0] : (seg == 1 ? a.seg_w[1] : a.seg_w[2]);
    row[wb] = (blk - b0) * 32 + c;
    wstream[wb] = (const char *)seg_w + ((size_t)(blk - b0) * n_it_total + it_begin) * (size_t)kTileBytes + lane * 16;
  }

  f32x16_t acc[WB][TB];
#pragma unroll
  for (int wb = 0; wb < WB; wb++)
#pragma unroll
    for (int t = 0; t < TB; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[wb][t][v] = 0.f;
  u32x4_t ring[2][WB][8];
  u32x4_t xr[XCH];

  auto load_w = [&](u32x4_t (&dst)[WB][8], int it) {
#pragma unroll
    for (int wb = 0; wb < WB; wb++) {
      const char *p = wstream[wb] + (size_t)it * kTileBytes;
#pragma unroll
      for (int j = 0; j < 8; j++) dst[wb][j] = *(const u32x4_t *)(p + j * 1024);
    }
  };
  const char *xbase = (const char *)a.x + (size_t)mt * 128 * a.ldx * sizeof(T);
  auto load_x = [&](int slab) {
    const int k0 = k_begin + slab * kSlabIters * KI;
#pragma unroll
    for (int i = 0; i < XCH; i++) {
      const int qq = tid + i * kGemmThreads;
      const int r = qq / (kSlabRowBytes / 16), cc = qq % (kSlabRowBytes / 16);
      const int kk = k0 + cc * EPL;
      xr[i] = *(const u32x4_t *)(xbase + ((size_t)(r < m_loc ? r : 0) * a.ldx + (kk < a.in ? kk : 0)) * sizeof(T));
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XCH; i++) {
      const int qq = tid + i * kGemmThreads;
      const int r = qq / (kSlabRowBytes / 16), cc = qq % (kSlabRowBytes / 16);
      *(u32x4_t *)(lds + buf * kSlabBytes + r * kSlabStride + cc * 16) = xr[i];
    }
  };
  auto compute = [&](const u32x4_t (&w)[WB][8], int buf, int ii) {
    const unsigned char *base = lds + buf * kSlabBytes + c * kSlabStride + ii * (2 * kLaneBytes) + g * kLaneBytes;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      u32x4_t xf[TB];
#pragma unroll
      for (int t = 0; t < TB; t++) xf[t] = *(const u32x4_t *)(base + t * 32 * kSlabStride + j * 16);
#pragma unroll
      for (int wb = 0; wb < WB; wb++)
#pragma unroll
        for (int t = 0; t < TB; t++) mfma_step(acc[wb][t], xf[t], w[wb][j], T{});
    }
  };

  load_x(0);
  if (0 < n_iter) load_w(ring[0], 0);
  store_x(0);
  __syncthreads();
  // Steady state: a next slab exists, so every load below is unconditional and the compiler can count the
  // outstanding loads exactly (a guarded load would make it wait for everything before each compute).
  // The ring stage of iteration it = 2 S + ii is ii.
  int S = 0;
  for (; S + 1 < n_slab; S++) {
    const int buf = S & 1;
    load_x(S + 1);
#pragma unroll
    for (int ii = 0; ii < kSlabIters; ii++) {
      load_w(ring[(ii + 1) & 1], S * kSlabIters + ii + 1);
      __builtin_amdgcn_sched_barrier(0);                       // keep the prefetch ahead of the MFMAs
      compute(ring[ii & 1], buf, ii);
      __builtin_amdgcn_sched_barrier(0);
    }
    store_x(buf ^ 1);
    __syncthreads();
  }
  for (; S < n_slab; S++) {                                    // last slab: one or two iterations, nothing follows
    const int buf = S & 1;
#pragma unroll
    for (int ii = 0; ii < kSlabIters; ii++) {
      const int it = S * kSlabIters + ii;
      if (it + 1 < n_iter) load_w(ring[(ii + 1) & 1], it + 1);
      if (it < n_iter) compute(ring[ii & 1], buf, ii);
    }
  }

  if (swiglu) {
    const int f = a.seg_rows[0];
#pragma unroll
    for (int wb = 0; wb < WB; wb++) {
      const int col = blk_of[wb] * 16 + (c & 15);
      swiglu_epilogue<T, TB>(acc[wb], (T *)a.act + (size_t)mt * 128 * f + col, f, col, active[wb] && col < f, m_loc, c, g);
    }
    return;
  }
#pragma unroll
  for (int wb = 0; wb < WB; wb++) {
    if (!active[wb] || row[wb] >= seg_rows[wb]) continue;
    float *out = a.part + ((size_t)by * a.m_pad + (size_t)mt * 128) * a.ldp + seg_col0[wb] + row[wb];
#pragma unroll
    for (int t = 0; t < TB; t++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int i = t * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
        if (i < m_loc) out[(size_t)i * a.ldp] = acc[wb][t][v];
      }
  }
}

// ---- packing ---------------------------------------------------------------------------------
// One thread moves one 16-byte piece: dst piece index p = ((rb * n_it + it) * 8 + j) * 64 + lane.
template <typename T>
__global__ __launch_bounds__(256) void pack_weight_kernel(const T *src, int rows, int in, u32x4_t *dst, size_t n_pieces) {
  constexpr int EPL = GemmTraits<T>::kEpl;
  constexpr int KI = 2 * kLaneBytes / (int)sizeof(T);
  const int n_it = (in + KI - 1) / KI;
  for (size_t p = (size_t)blockIdx.x * 256 + threadIdx.x; p < n_pieces; p += (size_t)gridDim.x * 256) {
    const int lane = (int)(p & 63), j = (int)((p >> 6) & 7);
    const size_t tile = p >> 9;
    const int it = (int)(tile % n_it);
    const int rb = (int)(tile / n_it);
    const int row = rb * 32 + (lane & 31);
    const int k = it * KI + (lane >> 5) * (KI / 2) + j * EPL;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (row < rows && k < in) v = *(const u32x4_t *)(src + (size_t)row * in + k);     // in % EPL == 0: whole piece in range
    dst[p] = v;
  }
}

// The gate and up projections as ONE packed matrix: block b holds, in the row order of the layout above, the gate
// rows 16 b .. 16 b + 15 and then the up rows 16 b .. 16 b + 15 (zero rows past the last column), so that one wave
// owns both sums of a column and SwiGLU needs no second pass and no exchange between waves.
template <typename T>
__global__ __launch_bounds__(256) void pack_gate_up_kernel(const T *gate, const T *up, int rows, int in, u32x4_t *dst, size_t n_pieces) {
  constexpr int EPL = GemmTraits<T>::kEpl;
  constexpr int KI = 2 * kLaneBytes / (int)sizeof(T);
  const int n_it = (in + KI - 1) / KI;
  for (size_t p = (size_t)blockIdx.x * 256 + threadIdx.x; p < n_pieces; p += (size_t)gridDim.x * 256) {
    const int lane = (int)(p & 63), j = (int)((p >> 6) & 7);
    const size_t tile = p >> 9;
    const int it = (int)(tile % n_it);
    const int rb = (int)(tile / n_it);
    const int c = lane & 31;
    const int row = rb * 16 + (c & 15);
    const T *src = c < 16 ? gate : up;
    const int k = it * KI + (lane >> 5) * (KI / 2) + j * EPL;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (row < rows && k < in) v = *(const u32x4_t *)(src + (size_t)row * in + k);
    dst[p] = v;
  }
}

size_t packed_gate_up_bytes(int dtype, int rows, int in) {
  const int ki = gemm_k_per_iter(dtype);
  return (size_t)((rows + 15) / 16) * (size_t)((in + ki - 1) / ki) * kTileBytes;
}

hipError_t launch_pack_gate_up(int dtype, const void *gate, const void *up, int rows, int in, void *dst, hipStream_t st) {
  const int epl = dtype == 1 ? 8 : 4;
  if (rows < 1 || in < 1 || in % epl) return hipErrorInvalidValue;
  const size_t n_pieces = packed_gate_up_bytes(dtype, rows, in) / 16;
  const int blocks = (int)std::min<size_t>((n_pieces + 255) / 256, 65536);
  if (dtype == 1)
    hipLaunchKernelGGL(pack_gate_up_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t *)gate, (const bf16_t *)up, rows, in,
                       (u32x4_t *)dst, n_pieces);
  else
    hipLaunchKernelGGL(pack_gate_up_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float *)gate, (const float *)up, rows, in,
                       (u32x4_t *)dst, n_pieces);
  return hipGetLastError();
}

size_t packed_weight_bytes(int dtype, int rows, int in) {
  const int ki = gemm_k_per_iter(dtype);
  return (size_t)((rows + 31) / 32) * (size_t)((in + ki - 1) / ki) * kTileBytes;
}

hipError_t launch_pack_weight(int dtype, const void *src, int rows, int in, void *dst, hipStream_t st) {
  const int epl = dtype == 1 ? 8 : 4;
  if (rows < 1 || in < 1 || in % epl) return hipErrorInvalidValue;
  const size_t n_pieces = packed_weight_bytes(dtype, rows, in) / 16;
  const int blocks = (int)std::min<size_t>((n_pieces + 255) / 256, 65536);
  if (dtype == 1)
    hipLaunchKernelGGL(pack_weight_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t *)src, rows, in, (u32x4_t *)dst, n_pieces);
  else
    hipLaunchKernelGGL(pack_weight_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float *)src, rows, in, (u32x4_t *)dst, n_pieces);
  return hipGetLastError();
}

// The double-buffered slab exceeds the 64 KiB default for dynamic LDS from two token blocks on: raise the
// limit once per kernel, at context creation (never during a stream capture).
template <typename T>
static hipError_t init_t() {
  const void *fn[4] = {(const void *)gemm_stream_kernel<T, 1>, (const void *)gemm_stream_kernel<T, 2>,
                       (const void *)gemm_stream_kernel<T, 3>, (const void *)gemm_stream_kernel<T, 4>};
  for (int tb = 1; tb <= 4; tb++) {
    const size_t lds = (size_t)2 * tb * 32 * kSlabStride;
    if (lds > 160 * 1024) continue;
    hipError_t e = hipFuncSetAttribute(fn[tb - 1], hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  return hipFuncSetAttribute((const void *)gemm_tiled_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             2 * 4 * 32 * kSlabStride);
}
hipError_t gemm_init() {
  // kernel attributes belong to the device's copy of the code: once per device, for the current device
  static bool done[64] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < 64 && done[dev]) return hipSuccess;
  e = init_t<bf16_t>();
  if (e == hipSuccess) e = init_t<float>();
  if (dev >= 0 && dev < 64) done[dev] = e == hipSuccess;
  return e;
}

template <typename T>
static hipError_t launch_t(GemmArgs a, hipStream_t st) {
  a.m_tiles = (a.m + 127) / 128;
  const int tb = a.m_tiles > 1 ? 4 : (a.m + 31) / 32;
  // Workgroups along the rows.  A compute unit sustains about 30 GB/s whatever the number of its waves, so what counts is
  // the largest number of blocks any workgroup streams.  With four blocks per workgroup the launch may leave compute
  // units idle (7B gate/up: 688 blocks = 172 workgroups); if the blocks fit in three, two or one per workgroup on at
  // most 256 workgroups (all splits together), the launch takes that form: wave w streams block x + w * grid_x and
  // the waves left without a block only help to stage the X slab (7B gate/up 36.1 -> 33.6 us, O 10.8 -> 10.0, down with
  // 4 splits 24.3 -> 20.3).  Otherwise four adjacent blocks per workgroup: spreading without lowering the largest count
  // measured 1 - 4 % slower at the 13B shapes.
  {
    const int cap = std::max(1, 256 / a.n_split);
    const int per_wg = (a.total_blocks + cap - 1) / cap;
    if (per_wg < kGemmWaves) {
      a.grid_x = (a.total_blocks + per_wg - 1) / per_wg;
      a.blk_per_wg = 1; a.blk_per_wave = a.grid_x;
    } else {
      a.grid_x = (a.total_blocks + kGemmWaves - 1) / kGemmWaves;
      a.blk_per_wg = kGemmWaves; a.blk_per_wave = 1;
    }
  }
  // SwiGLU mode: the one gate/up matrix, 16 columns per block, whole K (the activation is not linear)
  if (a.act != nullptr && (a.nseg != 1 || a.n_split != 1 || a.seg_blocks[0] != (a.seg_rows[0] + 15) / 16)) return hipErrorInvalidValue;
  dim3 grid(a.grid_x, a.n_split);
  if (a.m_tiles > 1) {                                         // two blocks per wave; see gemm_tiled_kernel's id decoding
    a.grid_x = (a.total_blocks + 2 * kGemmWaves - 1) / (2 * kGemmWaves);
    const dim3 tgrid((a.grid_x * a.n_split + 7) / 8 * 8 * a.m_tiles, 1);
    hipLaunchKernelGGL((gemm_tiled_kernel<T>), tgrid, dim3(kGemmThreads), (size_t)2 * 4 * 32 * kSlabStride, st, a);
    return hipGetLastError();
  }
  const size_t lds = (size_t)2 * tb * 32 * kSlabStride;
  if (lds > 160 * 1024) return hipErrorInvalidValue;
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

hipError_t launch_gemm(int dtype, const GemmArgs &a, hipStream_t st) {
  { hipError_t e = gemm_init(); if (e != hipSuccess) return e; }
  if (a.m < 1 || a.m_pad < a.m || a.nseg < 1 || a.nseg > 3 || a.n_split < 1 || a.in < 1) return hipErrorInvalidValue;
  if (a.n_split > (a.in + gemm_k_per_slab(dtype) - 1) / gemm_k_per_slab(dtype)) return hipErrorInvalidValue;   // no empty split
  return dtype == 1 ? launch_t<bf16_t>(a, st) : launch_t<float>(a, st);
}

}  // namespace spec
