// Selection kernels of the speculative-decoding cycle: vocabulary reductions (argmax,
// softmax statistics, top-k log-probabilities), the draft tree's candidate pool (expansion,
// frontier choice, rerank), acceptance (greedy walk, multi-round rejection sampling with a
// counter-based RNG) and the KV-cache compaction that commits the accepted path.
//
// Ordering rule everywhere: larger value first, equal values by lower index, so results are
// unique and independent of how the work is split over lanes.
#include <limits.h>

#include "common.h"
#include "kernels.h"

namespace spec {

constexpr int kSelThreads = 256;

// ---- counter-based RNG: splitmix64 finaliser chained over (seed, cycle, node, draw) --------
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27; x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}
__device__ __forceinline__ uint64_t rng_stream(uint64_t seed, uint32_t cycle, uint32_t node) {
  uint64_t s = mix64(seed + 0x9E3779B97F4A7C15ull);
  s = mix64(s + cycle);
  return mix64(s + node);
}
// 23 random bits centred in their cell: never 0 or 1, exact in fp32.
__device__ __forceinline__ float rng_uniform(uint64_t stream, uint64_t draw) {
  return ((float)(mix64(stream + draw) >> 41) + 0.5f) * 1.1920928955078125e-07f;
}
__device__ __forceinline__ float rng_gumbel(uint64_t stream, int v) {
  return -logf(-logf(rng_uniform(stream, (1ull << 32) + (uint64_t)v)));
}

// ---- per-row argmax ------------------------------------------------------------------------
// Stage 1: one workgroup per (slice of kTopkSlice entries, row) leaves the slice's best (value, index)
// in part_val / part_idx [rows][n_slices].  The consumer (greedy acceptance, or the finishing kernel)
// merges a row's slices with the same ordering rule, so the result is the row's first maximum.
__global__ __launch_bounds__(kSelThreads) void argmax_slice_kernel(const float *logits, int vocab, int n_slices,
                                                                   float *part_val, int *part_idx) {
  constexpr int PER = kTopkSlice / kSelThreads;   // 16
  __shared__ float shv[16];
  __shared__ int shi[16];
  const int slice = blockIdx.x, rowi = blockIdx.y, t = threadIdx.x;
  const int c0 = slice * kTopkSlice;
  const float *row = logits + (size_t)rowi * vocab;
  float v[PER];
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = c0 + t + e * kSelThreads;
    v[e] = c < vocab ? row[c] : -INFINITY;
  }
  ValIdx b{-INFINITY, INT_MAX};
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = c0 + t + e * kSelThreads;
    if (c < vocab && (v[e] > b.v || b.i == INT_MAX)) { b.v = v[e]; b.i = c; }   // ascending c: strict > keeps the lower index
  }
  b = block_best(b, shv, shi);
  if (t == 0) { part_val[(size_t)rowi * n_slices + slice] = b.v; part_idx[(size_t)rowi * n_slices + slice] = b.i; }
}
// One wavefront: best of a row's slice results.
__device__ __forceinline__ int merge_argmax(const float *part_val, const int *part_idx, int n_slices, int row, int lane) {
  ValIdx b{-INFINITY, INT_MAX};
  for (int sl = lane; sl < n_slices; sl += 64) {
    const float x = part_val[(size_t)row * n_slices + sl];
    const int c = part_idx[(size_t)row * n_slices + sl];
    if (better(x, c, b.v, b.i)) { b.v = x; b.i = c; }
  }
  return wave_best(b).i;
}
__global__ __launch_bounds__(64) void argmax_finish_kernel(const float *part_val, const int *part_idx, int n_slices, int *out) {
  const int best = merge_argmax(part_val, part_idx, n_slices, blockIdx.x, threadIdx.x);
  if (threadIdx.x == 0) out[blockIdx.x] = best;
}
int argmax_slices(int vocab) { return (vocab + kTopkSlice - 1) / kTopkSlice; }
hipError_t launch_rows_argmax(const float *logits, int rows, int vocab, float *part_val, int *part_idx, int *out,
                              hipStream_t st) {
  if (rows < 1 || vocab < 1) return hipErrorInvalidValue;
  const int n_slices = argmax_slices(vocab);
  hipLaunchKernelGGL(argmax_slice_kernel, dim3(n_slices, rows), dim3(kSelThreads), 0, st, logits, vocab, n_slices, part_val,
                     part_idx);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || out == nullptr) return e;
  hipLaunchKernelGGL(argmax_finish_kernel, dim3(rows), dim3(64), 0, st, part_val, part_idx, n_slices, out);
  return hipGetLastError();
}

// ---- per-row softmax statistics at temperature T, x = logit / T ----------------------------
// One workgroup per (slice of kTopkSlice entries, row): part[row][slice] = {max x, sum exp(x - max x)} over the
// slice.  merge_softmax_stats (one wavefront) turns a row's slices into {max x, sum exp(x - max x)} of the row.
__global__ __launch_bounds__(kSelThreads) void softmax_slice_kernel(const float *logits, int vocab, float temp, int n_slices,
                                                                    float2 *part) {
  constexpr int PER = kTopkSlice / kSelThreads;   // 16
  __shared__ float sh[16];
  const int slice = blockIdx.x, rowi = blockIdx.y, t = threadIdx.x;
  const int c0 = slice * kTopkSlice;
  const float *row = logits + (size_t)rowi * vocab;
  float v[PER];
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = c0 + t + e * kSelThreads;
    v[e] = c < vocab ? row[c] / temp : -INFINITY;
  }
  float m = v[0];
#pragma unroll
  for (int e = 1; e < PER; e++) m = fmaxf(m, v[e]);
  m = block_max(m, sh);
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < PER; e++) s += expf(v[e] - m);        // exp(-inf) = 0 for padding
  s = block_sum(s, sh);
  if (t == 0) part[(size_t)rowi * n_slices + slice] = make_float2(m, s);
}
__device__ __forceinline__ float2 merge_softmax_stats(const float2 *part, int n_slices, int row, int lane) {
  const float2 *stat = part + (size_t)row * n_slices;
  float m = -INFINITY;
  for (int sl = lane; sl < n_slices; sl += 64) m = fmaxf(m, stat[sl].x);
  m = wave_max(m);
  float tot = 0.f;
  for (int s0 = 0; s0 < n_slices; s0 += 64) {              // slices in ascending groups of 64, fixed butterfly inside
    const int sl = s0 + lane;
    tot += wave_sum(sl < n_slices ? stat[sl].y * expf(stat[sl].x - m) : 0.f);
  }
  return make_float2(m, tot);
}
hipError_t launch_rows_softmax_stats(const float *logits, int rows, int vocab, float temp, float2 *part, hipStream_t st) {
  if (rows < 1 || vocab < 1 || !(temp > 0.f)) return hipErrorInvalidValue;
  const int n_slices = argmax_slices(vocab);
  hipLaunchKernelGGL(softmax_slice_kernel, dim3(n_slices, rows), dim3(kSelThreads), 0, st, logits, vocab, temp, n_slices, part);
  return hipGetLastError();
}

// ---- per-row top-k log-probabilities -------------------------------------------------------
// Stage 1: one workgroup per (slice of kTopkSlice entries, row): slice max, slice sum-exp and the
// slice's k best entries.  Each wavefront finds the k best of its own 1024 register-resident values by k
// rounds of a wave-wide argmax (shuffles only); the 4k finalists are then placed by rank.
__global__ __launch_bounds__(kSelThreads) void topk_slice_kernel(const float *logits, int vocab, int k, int n_slices,
                                                                 float *sc_val, int *sc_idx, float2 *sc_stat) {
  constexpr int PER = kTopkSlice / kSelThreads;   // 16
  constexpr int NWV = kSelThreads / 64;
  __shared__ float shv[16];
  __shared__ float cv[NWV * kMaxTopK];
  __shared__ __attribute__((aligned(16))) uint64_t keys[NWV * kMaxTopK + 2];
  const int slice = blockIdx.x, rowi = blockIdx.y, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int c0 = slice * kTopkSlice;
  const float *row = logits + (size_t)rowi * vocab;
  float v[PER];
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = c0 + t + e * kSelThreads;
    v[e] = c < vocab ? row[c] : -INFINITY;
  }
  float m = v[0];
#pragma unroll
  for (int e = 1; e < PER; e++) m = fmaxf(m, v[e]);
  m = block_max(m, shv);
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < PER; e++) s += expf(v[e] - m);        // exp(-inf) = 0 for padding
  s = block_sum(s, shv);
  const size_t o = ((size_t)rowi * n_slices + slice);
  if (t == 0) sc_stat[o] = make_float2(m, s);
  uint32_t taken = 0;
  for (int r = 0; r < k; r++) {
    // best remaining value of the wave, then the lowest index carrying it
    float mv = -INFINITY;
#pragma unroll
    for (int e = 0; e < PER; e++) mv = fmaxf(mv, ((taken >> e) & 1u) ? -INFINITY : v[e]);
    const float best_v = wave_max_dpp(mv);
    int mi = INT_MAX;
#pragma unroll
    for (int e = PER - 1; e >= 0; e--) {
      const int c = c0 + t + e * kSelThreads;
      if (!((taken >> e) & 1u) && c < vocab && v[e] == best_v) mi = c;
    }
    const int best_i = wave_min_dpp(mi);
    if (lane == 0) { keys[wave * k + r] = order_key(best_v, best_i); cv[wave * k + r] = best_v; }
    if (best_i != INT_MAX && (best_i - c0) % kSelThreads == t) taken |= 1u << ((best_i - c0) / kSelThreads);
  }
  if (t < 2) keys[NWV * k + t] = 0ull;                       // padding for the pairwise reads
  __syncthreads();
  if (t < NWV * k) {
    const uint64_t key = keys[t];
    const int rank = key_rank(keys, (NWV * k + 1) & ~1, key, t);
    if (rank < k) {
      const bool valid = key != 0ull;
      sc_val[o * kMaxTopK + rank] = valid ? cv[t] : -INFINITY;
      sc_idx[o * kMaxTopK + rank] = valid ? 0x7FFFFFFF - (int)(uint32_t)key : INT_MAX;
    }
  }
}
// Stage 2: one workgroup per row merges the slices: log-sum-exp (first wavefront) and the k best of all
// slice candidates, placed by rank.
constexpr int kMaxMergeCand = 4096;
__global__ __launch_bounds__(kSelThreads) void topk_merge_kernel(int k, int n_slices, const float *sc_val, const int *sc_idx,
                                                                 const float2 *sc_stat, int *top_tok, float *top_lp) {
  __shared__ __attribute__((aligned(16))) uint64_t keys[kMaxMergeCand + 2];
  __shared__ float lse_sh;
  const int rowi = blockIdx.x, t = threadIdx.x;
  const int n_cand = n_slices * k;                          // candidate id = slice * k + r
  const int n2 = (n_cand + 1) & ~1;
  const float *val = sc_val + (size_t)rowi * n_slices * kMaxTopK;
  const int *idx = sc_idx + (size_t)rowi * n_slices * kMaxTopK;
  for (int id = t; id < n2; id += kSelThreads) {
    const int sl = id / k, rr = id % k;
    keys[id] = id < n_cand ? order_key(val[sl * kMaxTopK + rr], idx[sl * kMaxTopK + rr]) : 0ull;
  }
  if (t < 64) {
    const float2 *stat = sc_stat + (size_t)rowi * n_slices;
    float m = -INFINITY;
    for (int sl = t; sl < n_slices; sl += 64) m = fmaxf(m, stat[sl].x);
    m = wave_max(m);
    float tot = 0.f;
    for (int s0 = 0; s0 < n_slices; s0 += 64) {            // slices in ascending groups of 64, fixed butterfly inside
      const int sl = s0 + t;
      tot += wave_sum(sl < n_slices ? stat[sl].y * expf(stat[sl].x - m) : 0.f);
    }
    if (t == 0) lse_sh = m + logf(tot);
  }
  __syncthreads();
  const float lse = lse_sh;
  for (int id = t; id < n_cand; id += kSelThreads) {
    const uint64_t key = keys[id];
    const int rank = key_rank(keys, n2, key, id);
    if (rank < k) {
      const int sl = id / k, rr = id % k;
      top_tok[rowi * kMaxTopK + rank] = idx[sl * kMaxTopK + rr];
      top_lp[rowi * kMaxTopK + rank] = val[sl * kMaxTopK + rr] - lse;
    }
  }
}
hipError_t launch_rows_topk_logprob(const float *logits, int rows, int vocab, int k, float *sc_val, int *sc_idx,
                                    float2 *sc_stat, int *top_tok, float *top_lp, hipStream_t st) {
  const int n_slices = (vocab + kTopkSlice - 1) / kTopkSlice;
  if (rows < 1 || k < 1 || k > kMaxTopK || k > vocab || n_slices * k > kMaxMergeCand) return hipErrorInvalidValue;
  hipLaunchKernelGGL(topk_slice_kernel, dim3(n_slices, rows), dim3(kSelThreads), 0, st, logits, vocab, k, n_slices, sc_val,
                     sc_idx, sc_stat);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(topk_merge_kernel, dim3(rows), dim3(kSelThreads), 0, st, k, n_slices, sc_val, sc_idx, sc_stat, top_tok, top_lp);
  return hipGetLastError();
}

// ---- candidate pool ------------------------------------------------------------------------
// top_tok / top_lp rows have stride kMaxTopK.
__global__ void pool_init_kernel(DraftState s, const int *top_tok, const float *top_lp, int k, int root_row,
                                 const int *n_draft_ptr) {
  const int r = threadIdx.x;
  const int n_draft = *n_draft_ptr;
  if (r < k) {
    s.pool_tok[r] = top_tok[r]; s.pool_par[r] = -1; s.pool_dep[r] = 1; s.pool_sc[r] = top_lp[r];
    s.front_pool[r] = r; s.front_tok[r] = top_tok[r]; s.front_src[r] = root_row; s.front_depth[r] = 0;
    s.front_anc[r * kAncStride] = r;
    s.front_slot[r] = n_draft + r;
    s.front_pos[r] = n_draft + 1;
  }
  if (r == 0) *s.n_pool = k;
}
hipError_t launch_pool_init(const DraftState &s, const int *top_tok, const float *top_lp, int k, int root_row,
                            const int *n_draft, hipStream_t st) {
  if (k < 1 || k > kMaxTopK) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pool_init_kernel, dim3(1), dim3(64), 0, st, s, top_tok, top_lp, k, root_row, n_draft);
  return hipGetLastError();
}

// `step` t in 2..D: the k frontier rows are nodes of depth t-1; their children have depth t.
__global__ __launch_bounds__(kSelThreads) void pool_expand_kernel(DraftState s, const int *top_tok, const float *top_lp,
                                                                  int k, int step, const int *n_draft_ptr, int select_next) {
  __shared__ float sc[kMaxTopK * kMaxTopK];
  __shared__ int old_anc[kMaxTopK * kAncStride];
  __shared__ int old_pool[kMaxTopK];
  const int t = threadIdx.x, kk = k * k;
  const int n_draft = *n_draft_ptr;
  const int base = *s.n_pool;
  if (t < k) old_pool[t] = s.front_pool[t];
  for (int e = t; e < k * kAncStride; e += kSelThreads) old_anc[e] = s.front_anc[e];
  __syncthreads();
  int r = 0, j = 0, tok = 0;
  if (t < kk) {
    r = t / k; j = t % k;                                   // children in (frontier order, best first) order
    tok = top_tok[r * kMaxTopK + j];
    const float v = s.pool_sc[old_pool[r]] + top_lp[r * kMaxTopK + j];
    sc[t] = v;
    s.pool_tok[base + t] = tok; s.pool_par[base + t] = old_pool[r]; s.pool_dep[base + t] = step; s.pool_sc[base + t] = v;
  }
  __syncthreads();
  if (t == 0) *s.n_pool = base + kk;
  if (!select_next || t >= kk) return;
  int rank = 0;
  for (int c = 0; c < kk; c++) rank += better(sc[c], c, sc[t], t) ? 1 : 0;
  if (rank >= k) return;
  // this child is row `rank` of the next expansion step (step + 1): depth argument step - 1
  s.front_pool[rank] = base + t; s.front_tok[rank] = tok; s.front_src[rank] = r; s.front_depth[rank] = step - 1;
  for (int a = 0; a < step - 1; a++) s.front_anc[rank * kAncStride + a] = old_anc[r * kAncStride + a];
  s.front_anc[rank * kAncStride + step - 1] = (step - 1) * k + rank;
  s.front_slot[rank] = n_draft + (step - 1) * k + rank;
  s.front_pos[rank] = n_draft + 1 + (step - 1);
}
hipError_t launch_pool_expand(const DraftState &s, const int *top_tok, const float *top_lp, int k, int step,
                              const int *n_draft, int select_next, hipStream_t st) {
  if (k < 1 || k > kMaxTopK || step < 2 || step > kMaxDepth) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pool_expand_kernel, dim3(1), dim3(kSelThreads), 0, st, s, top_tok, top_lp, k, step, n_draft, select_next);
  return hipGetLastError();
}

// ---- rerank --------------------------------------------------------------------------------
constexpr int kMaxPool = kMaxTopK + (kMaxDepth - 1) * kMaxTopK * kMaxTopK;    // 3600
constexpr int kPoolWords = (kMaxPool + 31) / 32;
constexpr int kRerankThreads = 1024;
__global__ __launch_bounds__(kRerankThreads) void rerank_kernel(DraftState s, int total, const int *root_tok, int *tree_n,
                                                                int *tree_tok, int *tree_par, int *tree_dep, float *tree_sc) {
  typedef __attribute__((ext_vector_type(4))) float f32x4_t;
  __shared__ __attribute__((aligned(16))) float sc[kMaxPool + 4];
  __shared__ uint32_t kept[kPoolWords];                     // bit c: pool entry c is in the tree
  __shared__ int before[kPoolWords];                        // kept entries in earlier words
  const int t = threadIdx.x, n = *s.n_pool;
  const int keep = min(total - 1, n);
  const int n_words = (n + 31) / 32, n4 = (n + 3) & ~3;
  for (int c = t; c < n4; c += kRerankThreads) sc[c] = c < n ? s.pool_sc[c] + 0.f : -INFINITY;
  for (int w = t; w < n_words; w += kRerankThreads) kept[w] = 0u;
  __syncthreads();
  for (int c = t; c < n; c += kRerankThreads) {
    // rank = entries with a larger score, plus equal scores at a lower pool index
    const float v = sc[c];
    int rank = 0;
#pragma unroll 2
    for (int o = 0; o < n4; o += 4) {
      const f32x4_t x = *(const f32x4_t *)(sc + o);
      rank += (x.x > v || (x.x == v && o < c)) ? 1 : 0;
      rank += (x.y > v || (x.y == v && o + 1 < c)) ? 1 : 0;
      rank += (x.z > v || (x.z == v && o + 2 < c)) ? 1 : 0;
      rank += (x.w > v || (x.w == v && o + 3 < c)) ? 1 : 0;
    }
    if (rank < keep) atomicOr(&kept[c >> 5], 1u << (c & 31));
  }
  __syncthreads();
  for (int w = t; w < n_words; w += kRerankThreads) {
    int cnt = 0;
    for (int u = 0; u < w; u++) cnt += __popc(kept[u]);
    before[w] = cnt;
  }
  __syncthreads();
  // node index = 1 + number of kept entries with a lower pool index (kept in pool order: parents first)
  auto node_of = [&](int c) { return 1 + before[c >> 5] + __popc(kept[c >> 5] & ((1u << (c & 31)) - 1u)); };
  for (int c = t; c < n; c += kRerankThreads) {
    if (!((kept[c >> 5] >> (c & 31)) & 1u)) continue;
    const int j = node_of(c);
    const int par = s.pool_par[c];
    tree_tok[j] = s.pool_tok[c];
    tree_par[j] = par < 0 ? 0 : node_of(par);               // a parent outscores (or ties at a lower index) its children, so it is kept
    tree_dep[j] = s.pool_dep[c];
    tree_sc[j] = s.pool_sc[c];
  }
  if (t == 0) { tree_tok[0] = *root_tok; tree_par[0] = -1; tree_dep[0] = 0; tree_sc[0] = 0.f; *tree_n = keep + 1; }
}
hipError_t launch_rerank(const DraftState &s, int total, const int *root_tok, int *tree_n, int *tree_tok, int *tree_par,
                         int *tree_dep, float *tree_sc, hipStream_t st) {
  if (total < 1 || total > kMaxNodes) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rerank_kernel, dim3(1), dim3(kRerankThreads), 0, st, s, total, root_tok, tree_n, tree_tok, tree_par, tree_dep,
                     tree_sc);
  return hipGetLastError();
}

// ---- acceptance ----------------------------------------------------------------------------
// First child of `cur` (lowest node index) carrying `tok`, or INT_MAX.  One wavefront.
__device__ __forceinline__ int find_child(const int *tree_tok, const int *tree_par, int n_nodes, int cur, int tok, int lane) {
  int best = INT_MAX;
  for (int c = lane; c < n_nodes; c += 64)
    if (c > cur && tree_par[c] == cur && tree_tok[c] == tok) best = min(best, c);
  return wave_min_i(best);
}

__global__ __launch_bounds__(64) void accept_greedy_kernel(const float *amax_val, const int *amax_idx, int n_slices,
                                                           const int *tree_tok, const int *tree_par, int n_nodes,
                                                           AcceptResult *res) {
  const int lane = threadIdx.x;
  int cur = 0, m = 0;
  if (lane == 0) res->node[0] = 0;
  for (int step = 0; step <= kMaxDepth; step++) {
    const int best = merge_argmax(amax_val, amax_idx, n_slices, cur, lane);   // argmax of the target's row
    const int c = m < kMaxDepth ? find_child(tree_tok, tree_par, n_nodes, cur, best, lane) : INT_MAX;
    if (lane == 0) res->token[m] = best;                    // accepted token, or the bonus when the walk stops
    if (c == INT_MAX) break;
    cur = c; m++;
    if (lane == 0) res->node[m] = cur;
  }
  if (lane == 0) res->n_acc = m;
}
hipError_t launch_accept_greedy(const float *amax_val, const int *amax_idx, int n_slices, const int *tree_tok,
                                const int *tree_par, int n_nodes, AcceptResult *res, hipStream_t st) {
  if (n_nodes < 1 || n_nodes > kMaxNodes || n_slices < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(accept_greedy_kernel, dim3(1), dim3(64), 0, st, amax_val, amax_idx, n_slices, tree_tok, tree_par, n_nodes,
                     res);
  return hipGetLastError();
}

// Gumbel-max over one row, skipping `n_rem` removed tokens.  Whole block; result to every thread.
__device__ __forceinline__ int gumbel_argmax(const float *row, int vocab, float temp, uint64_t stream, const int *rem,
                                             int n_rem, float *shv, int *shi) {
  ValIdx b{-INFINITY, INT_MAX};
  for (int v = threadIdx.x; v < vocab; v += blockDim.x) {
    bool skip = false;
    for (int r = 0; r < n_rem; r++) skip |= rem[r] == v;
    if (skip) continue;
    const float z = row[v] / temp + rng_gumbel(stream, v);
    if (z > b.v || b.i == INT_MAX) { b.v = z; b.i = v; }
  }
  return block_best(b, shv, shi).i;
}

// Multi-round rejection sampling down the tree.  The children of a node were chosen
// deterministically by the draft (top-k), so each is a point-mass proposal: child c is accepted
// with probability p'(c), where p' is the target distribution with the already rejected siblings
// removed and renormalised; when all children are rejected the bonus token is drawn from p'.
// One workgroup.  Per visited node: the first wavefront merges the row's softmax slices and lists the
// node's children, all threads fetch the children's logits together, thread 0 runs the (inherently
// sequential) accept/reject chain on those values, and the bonus draw uses the whole workgroup.
constexpr int kAcceptThreads = 1024;
__global__ __launch_bounds__(kAcceptThreads) void accept_sample_kernel(const float *logits, int vocab, const float2 *stat_part,
                                                                       int n_slices, float temp, const int *tree_tok,
                                                                       const int *tree_par, int n_nodes, uint64_t seed,
                                                                       uint32_t cycle, AcceptResult *res) {
  __shared__ float shv[16];
  __shared__ int shi[16];
  __shared__ int rem[kMaxNodes];
  __shared__ int kid[kMaxNodes];
  __shared__ float kid_x[kMaxNodes];
  __shared__ int sh_next, sh_nrem, sh_nkid;
  __shared__ float2 sh_stat;
  const int t = threadIdx.x;
  int cur = 0, m = 0;
  if (t == 0) res->node[0] = 0;
  for (int step = 0; step <= kMaxDepth; step++) {
    const uint64_t stream = rng_stream(seed, cycle, (uint32_t)cur);
    const float *row = logits + (size_t)cur * vocab;
    if (t < 64) {
      const float2 st = merge_softmax_stats(stat_part, n_slices, cur, t);
      if (t == 0) {
        sh_stat = st;
        int nk = 0;
        if (m < kMaxDepth)
          for (int c = cur + 1; c < n_nodes; c++)
            if (tree_par[c] == cur) kid[nk++] = c;            // node order = descending draft probability
        sh_nkid = nk;
      }
    }
    __syncthreads();
    const int n_kid = sh_nkid;
    if (t < n_kid) kid_x[t] = row[tree_tok[kid[t]]];
    __syncthreads();
    if (t == 0) {
      const float2 st = sh_stat;
      float removed = 0.f;                                  // probability mass of the rejected siblings
      int n_rem = 0, next = -1;
      for (int ord = 0; ord < n_kid && next < 0; ord++) {
        const int c = kid[ord];
        const int tok = tree_tok[c];
        bool dup = false;
        for (int r = 0; r < n_rem; r++) dup |= rem[r] == tok;
        const float p0 = dup ? 0.f : expf(kid_x[ord] / temp - st.x) / st.y;
        const float rest = 1.0f - removed;
        const float u = rng_uniform(stream, (uint64_t)ord);
        if (u < p0 / rest) { next = c; break; }
        if (!dup) { removed += p0; rem[n_rem++] = tok; }
        if (!(1.0f - removed > 0.f)) { next = c; break; }   // nothing left in the residual: c was certain
      }
      sh_next = next; sh_nrem = n_rem;
    }
    __syncthreads();
    const int next = sh_next, n_rem = sh_nrem;
    if (next >= 0) {
      if (t == 0) { res->token[m] = tree_tok[next]; res->node[m + 1] = next; }
      cur = next; m++;
      __syncthreads();
      continue;
    }
    const int bonus = gumbel_argmax(row, vocab, temp, stream, rem, n_rem, shv, shi);
    if (t == 0) res->token[m] = bonus;
    break;
  }
  if (t == 0) res->n_acc = m;
}
hipError_t launch_accept_sample(const float *logits, int vocab, const float2 *stat_part, float temp, const int *tree_tok,
                                const int *tree_par, int n_nodes, uint64_t seed, uint32_t cycle, AcceptResult *res,
                                hipStream_t st) {
  if (n_nodes < 1 || n_nodes > kMaxNodes || !(temp > 0.f)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(accept_sample_kernel, dim3(1), dim3(kAcceptThreads), 0, st, logits, vocab, stat_part, argmax_slices(vocab),
                     temp, tree_tok, tree_par, n_nodes, seed, cycle, res);
  return hipGetLastError();
}

// The ratio rule for SAMPLED children (the textbook speculative-sampling acceptance, Sec. 2 third step): at
// node `cur` with target distribution p and draft distribution q (both softmax(row / temp)), the children,
// drawn from q without replacement and tried in node order, are accepted with probability min(1, p_j / q_j);
// a rejection replaces p by normalise(max(p - q, 0)) and removes the child from q; when every child is
// rejected the next token is drawn from the current p (Gumbel-max).  One workgroup.  The current p lives in
// `work` (vocab floats, unnormalised, with its normaliser in a register); a thread only ever re-reads the
// entries it wrote itself, and the entry of a child's token is handed to the others through LDS.
__global__ __launch_bounds__(kAcceptThreads) void accept_qratio_kernel(const float *p_logits, const float *q_logits,
                                                                       const int *qrow_of, int vocab, float temp,
                                                                       const int *tree_tok, const int *tree_par, int n_nodes,
                                                                       uint64_t seed, uint32_t cycle, float *work,
                                                                       AcceptResult *res) {
  __shared__ float shv[16];
  __shared__ int shi[16];
  __shared__ int rem[kMaxNodes];
  __shared__ int kid[kMaxNodes];
  __shared__ int sh_nkid;
  __shared__ float sh_px, sh_q0;
  const int t = threadIdx.x;
  int cur = 0, m = 0;
  if (t == 0) res->node[0] = 0;
  for (int step = 0; step <= kMaxDepth; step++) {
    const uint64_t stream = rng_stream(seed, cycle, (uint32_t)cur);
    if (t == 0) {
      int nk = 0;
      if (m < kMaxDepth)
        for (int c = cur + 1; c < n_nodes; c++)
          if (tree_par[c] == cur) kid[nk++] = c;              // node order = draw order
      sh_nkid = nk;
    }
    __syncthreads();
    const int n_kid = sh_nkid;
    const float *prow = p_logits + (size_t)cur * vocab;
    // the draft row of a node without children is never read (it may not exist: qrow_of[cur] < 0)
    const float *qrow = n_kid == 0 ? prow : q_logits + (size_t)(qrow_of ? qrow_of[cur] : cur) * vocab;
    float mp = -INFINITY, mq = -INFINITY;
    for (int v = t; v < vocab; v += kAcceptThreads) { mp = fmaxf(mp, prow[v] / temp); mq = fmaxf(mq, qrow[v] / temp); }
    mp = block_max(mp, shv);
    mq = block_max(mq, shv);
    float sp = 0.f, sq = 0.f;
    for (int v = t; v < vocab; v += kAcceptThreads) {
      const float e = expf(prow[v] / temp - mp);
      work[v] = e;                                            // p, unnormalised: p(v) = work[v] * inv_zp
      sp += e;
      sq += expf(qrow[v] / temp - mq);
    }
    sp = block_sum(sp, shv);
    sq = block_sum(sq, shv);
    float inv_zp = 1.f / sp;
    float removed = 0.f, inv_zq = 1.f;                        // q_j(v) = q(v) * inv_zq for v not removed, else 0
    int next = -1, n_rem = 0;
    for (int ord = 0; ord < n_kid && next < 0; ord++) {
      const int c = kid[ord];
      const int x = tree_tok[c];
      bool dup = false;
      for (int r = 0; r < n_rem; r++) dup |= rem[r] == x;
      if (x % kAcceptThreads == t) { sh_px = work[x] * inv_zp; sh_q0 = expf(qrow[x] / temp - mq) / sq; }
      __syncthreads();
      const float px = sh_px, q0 = dup ? 0.f : sh_q0;
      const float u = rng_uniform(stream, (uint64_t)ord);
      if (u * (q0 * inv_zq) < px) { next = c; break; }
      // rejected: p <- max(p - q_j, 0), renormalised; q_{j+1} <- q_j without x
      float part = 0.f;
      for (int v = t; v < vocab; v += kAcceptThreads) {
        bool gone = false;
        for (int r = 0; r < n_rem; r++) gone |= rem[r] == v;
        const float qv = gone ? 0.f : expf(qrow[v] / temp - mq) / sq * inv_zq;
        const float nv = fmaxf(work[v] * inv_zp - qv, 0.f);
        work[v] = nv;
        part += nv;
      }
      const float zp = block_sum(part, shv);                  // (its barriers also order the LDS traffic of this round)
      if (!(zp > 0.f)) { next = c; break; }                   // nothing left in the residual: c was certain
      inv_zp = 1.f / zp;
      if (!dup) {
        if (t == 0) rem[n_rem] = x;
        n_rem++;
        removed += q0;
        inv_zq = 1.f - removed > 0.f ? 1.f / (1.f - removed) : 0.f;
      }
      __syncthreads();
    }
    if (next >= 0) {
      if (t == 0) { res->token[m] = tree_tok[next]; res->node[m + 1] = next; }
      cur = next; m++;
      __syncthreads();
      continue;
    }
    ValIdx b{-INFINITY, INT_MAX};
    for (int v = t; v < vocab; v += kAcceptThreads) {
      const float pv = work[v] * inv_zp;
      if (!(pv > 0.f)) continue;
      const float z = logf(pv) + rng_gumbel(stream, v);
      if (z > b.v || b.i == INT_MAX) { b.v = z; b.i = v; }
    }
    const int bonus = block_best(b, shv, shi).i;
    if (t == 0) res->token[m] = bonus;
    break;
  }
  if (t == 0) res->n_acc = m;
}
hipError_t launch_accept_qratio(const float *p_logits, const float *q_logits, const int *qrow_of, int vocab, float temp,
                                const int *tree_tok, const int *tree_par, int n_nodes, uint64_t seed, uint32_t cycle, float *work,
                                AcceptResult *res, hipStream_t st) {
  if (n_nodes < 1 || n_nodes > kMaxNodes || vocab < 1 || !(temp > 0.f)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(accept_qratio_kernel, dim3(1), dim3(kAcceptThreads), 0, st, p_logits, q_logits, qrow_of, vocab, temp, tree_tok,
                     tree_par, n_nodes, seed, cycle, work, res);
  return hipGetLastError();
}

// ---- static tree shapes ----------------------------------------------------------------------
// After the proposals of the nodes of depth d-1 are known (top_tok / top_lp, row = the node's row in its
// depth's forward, 0 for the root): fill token / parent / depth / score of the nodes of depth d, and for those
// of them that have children set up their row of the next draft forward (the same tables the dynamic
// expansion builds: token, source row of the parent's predicted feature, depth argument, ancestor slots).
__global__ void static_step_kernel(StaticTables tb, int d, const int *top_tok, const float *top_lp, int root_row,
                                   const int *root_tok, const int *n_draft_ptr, int with_scores, DraftState s, int *t_n,
                                   int *t_tok, int *t_par, int *t_dep, float *t_sc) {
  const int i = threadIdx.x;
  const int n_draft = *n_draft_ptr;
  if (i == 0 && d == 1) { *t_n = tb.n_nodes; t_tok[0] = *root_tok; t_par[0] = -1; t_dep[0] = 0; t_sc[0] = 0.f; }
  if (i < 1 || i >= tb.n_nodes || tb.depth[i] != d) return;
  const int p = tb.parent[i];
  const int pr = d == 1 ? 0 : tb.erow[p];
  const int tok = top_tok[pr * kMaxTopK + tb.rank[i]];
  t_tok[i] = tok; t_par[i] = p; t_dep[i] = d;
  t_sc[i] = with_scores ? (d == 1 ? 0.f : t_sc[p]) + top_lp[pr * kMaxTopK + tb.rank[i]] : 0.f;
  const int r = tb.erow[i];
  if (r < 0) return;
  s.front_tok[r] = tok;
  s.front_src[r] = d == 1 ? root_row : tb.erow[p];
  s.front_depth[r] = d - 1;
  s.front_slot[r] = n_draft + tb.eoff[i];
  s.front_pos[r] = n_draft + d;
  for (int a = i, q = d - 1; q >= 0; q--, a = tb.parent[a]) s.front_anc[r * kAncStride + q] = tb.eoff[a];
}
hipError_t launch_static_step(const StaticTables &tb, int d, const int *top_tok, const float *top_lp, int root_row,
                              const int *root_tok, const int *n_draft, int with_scores, const DraftState &s, int *t_n, int *t_tok,
                              int *t_par, int *t_dep, float *t_sc, hipStream_t st) {
  if (tb.n_nodes < 1 || tb.n_nodes > kMaxNodes || d < 1 || d > kMaxDepth) return hipErrorInvalidValue;
  hipLaunchKernelGGL(static_step_kernel, dim3(1), dim3(kMaxNodes), 0, st, tb, d, top_tok, top_lp, root_row, root_tok, n_draft,
                     with_scores, s, t_n, t_tok, t_par, t_dep, t_sc);
  return hipGetLastError();
}

// z[r][v] = logits[r][v] / temp + Gumbel noise of stream (seed, cycle, node_stream[r]) for rows r < rows.
__global__ __launch_bounds__(kSelThreads) void perturb_rows_kernel(const float *logits, int vocab, float temp, uint64_t seed,
                                                                   uint32_t cycle, const int *node_stream, float *z) {
  const int r = blockIdx.y;
  const uint64_t stream = rng_stream(seed, cycle, (uint32_t)node_stream[r]);
  const float *row = logits + (size_t)r * vocab;
  float *zr = z + (size_t)r * vocab;
  for (int v = blockIdx.x * kSelThreads + threadIdx.x; v < vocab; v += gridDim.x * kSelThreads)
    zr[v] = row[v] / temp + rng_gumbel(stream, v);
}
hipError_t launch_perturb_rows(const float *logits, int rows, int vocab, float temp, uint64_t seed, uint32_t cycle,
                               const int *node_stream, float *z, hipStream_t st) {
  if (rows < 1 || rows > kMaxTopK || vocab < 1 || !(temp > 0.f)) return hipErrorInvalidValue;
  const int blocks = (vocab + kSelThreads - 1) / kSelThreads;
  hipLaunchKernelGGL(perturb_rows_kernel, dim3(blocks > 256 ? 256 : blocks, rows), dim3(kSelThreads), 0, st, logits, vocab, temp, seed,
                     cycle, node_stream, z);
  return hipGetLastError();
}

// out[i] = the i-th of m tokens drawn without replacement from softmax(logits / temp): the m largest of
// logits / temp + Gumbel noise of stream (seed, cycle, node), found by the two-stage top-k above on the
// perturbed row (written to `z`, vocab floats).
__global__ __launch_bounds__(kSelThreads) void perturb_gumbel_kernel(const float *logits, int vocab, float temp, uint64_t seed,
                                                                     uint32_t cycle, uint32_t node, float *z) {
  const uint64_t stream = rng_stream(seed, cycle, node);
  for (int v = blockIdx.x * kSelThreads + threadIdx.x; v < vocab; v += gridDim.x * kSelThreads)
    z[v] = logits[v] / temp + rng_gumbel(stream, v);
}
__global__ void copy_ints_kernel(const int *src, int n, int *dst) {
  if ((int)threadIdx.x < n) dst[threadIdx.x] = src[threadIdx.x];
}
hipError_t launch_sample_children(const float *logits, int vocab, float temp, int m, uint64_t seed, uint32_t cycle, uint32_t node,
                                  float *z, float *sc_val, int *sc_idx, float2 *sc_stat, int *top_tok, float *top_lp, int *out,
                                  hipStream_t st) {
  if (vocab < 1 || m < 1 || m > kMaxTopK || m > vocab || !(temp > 0.f)) return hipErrorInvalidValue;
  const int blocks = (vocab + kSelThreads - 1) / kSelThreads;
  hipLaunchKernelGGL(perturb_gumbel_kernel, dim3(blocks > 1024 ? 1024 : blocks), dim3(kSelThreads), 0, st, logits, vocab, temp, seed,
                     cycle, node, z);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = launch_rows_topk_logprob(z, 1, vocab, m, sc_val, sc_idx, sc_stat, top_tok, top_lp, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(copy_ints_kernel, dim3(1), dim3(64), 0, st, top_tok, m, out);
  return hipGetLastError();
}

__global__ __launch_bounds__(kAcceptThreads) void sample_row_kernel(const float *logits, int vocab, float temp, uint64_t seed,
                                                                    uint32_t cycle, uint32_t node, int *out) {
  __shared__ float shv[16];
  __shared__ int shi[16];
  const int tok = gumbel_argmax(logits, vocab, temp, rng_stream(seed, cycle, node), nullptr, 0, shv, shi);
  if (threadIdx.x == 0) *out = tok;
}
hipError_t launch_sample_row(const float *logits, int vocab, float temp, uint64_t seed, uint32_t cycle, uint32_t node,
                             int *out, hipStream_t st) {
  if (vocab < 1 || !(temp > 0.f)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(sample_row_kernel, dim3(1), dim3(kAcceptThreads), 0, st, logits, vocab, temp, seed, cycle, node, out);
  return hipGetLastError();
}

// ---- commit: KV compaction + hand-off ------------------------------------------------------
// Thread = one 16-byte chunk of one (layer, key|value) row; it moves that chunk for depths 1..m in
// ascending order.  Depth d's destination slot n+d is never a later depth's source (sources
// n+node[d'] have node[d'] > d for d' > d), and a chunk column is owned by one thread, so the
// in-place move is race-free.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
__global__ __launch_bounds__(kSelThreads) void compact_kv_kernel(const AcceptResult *res, char *kv_base, size_t layer_bytes,
                                                                 size_t kv_bytes, int n_layers, int row_bytes, int n) {
  const int m = res->n_acc;
  if (m == 0) return;
  const int chunks = row_bytes / 16;
  const size_t total = (size_t)n_layers * 2 * chunks;
  for (size_t w = (size_t)blockIdx.x * kSelThreads + threadIdx.x; w < total; w += (size_t)gridDim.x * kSelThreads) {
    const int ch = (int)(w % chunks);
    const int kv = (int)((w / chunks) & 1);
    const int l = (int)(w / chunks / 2);
    char *base = kv_base + (size_t)l * layer_bytes + (size_t)kv * kv_bytes + (size_t)ch * 16;
    for (int d = 1; d <= m; d++) {
      const int src = n + res->node[d], dst = n + d;
      if (src != dst) *(u32x4_t *)(base + (size_t)dst * row_bytes) = *(const u32x4_t *)(base + (size_t)src * row_bytes);
    }
  }
}
// Features of root + accepted rows and the matching tokens for the next draft root step.
template <typename T>
__global__ __launch_bounds__(kSelThreads) void handoff_kernel(const AcceptResult *res, const T *feat, int d, T *pend_feat,
                                                              int *pend_tok, int *root_tok, int *n_committed) {
  const int r = blockIdx.x, m = res->n_acc;
  if (r == 0 && threadIdx.x == 0) *n_committed += 1 + m;      // root + accepted tokens are now in the cache
  if (r > m) return;
  const T *src = feat + (size_t)res->node[r] * d;
  T *dst = pend_feat + (size_t)r * d;
  for (int c = threadIdx.x; c < d; c += kSelThreads) dst[c] = src[c];
  if (threadIdx.x == 0) {
    pend_tok[r] = res->token[r];
    if (r == m) *root_tok = res->token[m];
  }
}
hipError_t launch_commit(int dtype, const AcceptResult *res, void *kv_base, size_t layer_stride, size_t kv_stride,
                         int n_layers, int row_elems, int n, const void *feat, int d, void *pend_feat, int *pend_tok,
                         int *root_tok, int *n_committed, hipStream_t st) {
  const size_t esz = dtype == 1 ? 2 : 4;
  const int row_bytes = (int)(row_elems * esz);
  if (row_bytes % 16 != 0 || n_layers < 1) return hipErrorInvalidValue;
  const size_t total = (size_t)n_layers * 2 * (row_bytes / 16);
  const int blocks = (int)((total + kSelThreads - 1) / kSelThreads);
  hipLaunchKernelGGL(compact_kv_kernel, dim3(blocks > 2048 ? 2048 : blocks), dim3(kSelThreads), 0, st, res, (char *)kv_base,
                     layer_stride * esz, kv_stride * esz, n_layers, row_bytes, n);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (dtype == 1)
    hipLaunchKernelGGL(handoff_kernel<bf16_t>, dim3(kMaxDepth + 1), dim3(kSelThreads), 0, st, res, (const bf16_t *)feat, d,
                       (bf16_t *)pend_feat, pend_tok, root_tok, n_committed);
  else
    hipLaunchKernelGGL(handoff_kernel<float>, dim3(kMaxDepth + 1), dim3(kSelThreads), 0, st, res, (const float *)feat, d,
                       (float *)pend_feat, pend_tok, root_tok, n_committed);
  return hipGetLastError();
}

}  // namespace spec
