// Top-K distillation loss (Sec. 3.1, Eq. 1) and the whole-vocabulary cross-entropy, from two fp32 logit
// rows per position: zq (target) and zp (draft), both produced by the LM-head GEMM.
//
//   loss_topk = - sum over the K tokens x of largest zq of  softmax(zq)(x) * log_softmax(zp)(x)
//   loss_ce   = - sum over all tokens                        of the same product
//
// Every logit is read once.  Stage 1, one workgroup per (slice of kTopkSlice tokens, position): the
// slice's softmax statistics of both rows, the cross term sum exp(zq - max) * zp, and the slice's K best
// target logits together with the draft logits at the same tokens.  Stage 2, one workgroup per position:
// merges the slices in ascending order (fixed order: the result does not depend on timing), ranks the
// candidates and forms both losses.  Ties between equal target logits go to the lower token id.
#include <limits.h>

#include "common.h"
#include "kernels.h"

namespace spec {

namespace {

constexpr int kLossThreads = 256;
constexpr int kLossWaves = kLossThreads / 64;

// Orders this wavefront's LDS writes before its later LDS reads of other lanes' data.  The LDS executes
// one wavefront's operations in issue order, so only the compiler has to be kept from reordering them.
__device__ __forceinline__ void wave_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// scratch per (position, slice): 5 floats of statistics, then K (target logit, token, draft logit) triples
__host__ __device__ inline size_t slice_floats(int k) { return 8 + 3 * (size_t)k; }

__global__ __launch_bounds__(kLossThreads) void loss_slice_kernel(const float *zq, const float *zp, int ldz, int vocab, int k,
                                                                   int n_slices, float *scratch) {
  constexpr int PER = kTopkSlice / kLossThreads;   // 16
  static_assert(kLossWaves == 4, "the reductions below combine four wavefronts");
  __shared__ float red_max[kLossWaves][2], red_sum[kLossWaves][4];
  __shared__ float cq[kLossWaves * kLossMaxK], cp[kLossWaves * kLossMaxK];
  __shared__ __attribute__((aligned(16))) uint64_t keys[kLossWaves * kLossMaxK + 2];
  __shared__ __attribute__((aligned(16))) uint64_t ckey[kLossWaves][64];   // filtered candidates, one per lane
  __shared__ float cqv[kLossWaves][64], cpv[kLossWaves][64];
  const int slice = blockIdx.x, rowi = blockIdx.y, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int c0 = slice * kTopkSlice;
  const float *rq = zq + (size_t)rowi * ldz, *rp = zp + (size_t)rowi * ldz;
  float vq[PER], vp[PER];
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const int c = c0 + t + e * kLossThreads;
    vq[e] = c < vocab ? rq[c] : -INFINITY;
    vp[e] = c < vocab ? rp[c] : -INFINITY;
  }
  // two workgroup-wide reductions, each over several quantities at once (wavefront results in LDS, then every
  // thread combines the four wavefronts in the same fixed order)
  float mq = vq[0], mp = vp[0];
#pragma unroll
  for (int e = 1; e < PER; e++) { mq = fmaxf(mq, vq[e]); mp = fmaxf(mp, vp[e]); }
  mq = wave_max(mq);
  mp = wave_max(mp);
  if (lane == 0) { red_max[wave][0] = mq; red_max[wave][1] = mp; }
  __syncthreads();
  mq = fmaxf(fmaxf(red_max[0][0], red_max[1][0]), fmaxf(red_max[2][0], red_max[3][0]));
  mp = fmaxf(fmaxf(red_max[0][1], red_max[1][1]), fmaxf(red_max[2][1], red_max[3][1]));
  float sq = 0.f, sp = 0.f, cross = 0.f;
#pragma unroll
  for (int e = 0; e < PER; e++) {
    const bool in = c0 + t + e * kLossThreads < vocab;
    const float wq = expf(vq[e] - mq);                       // exp(-inf) = 0 for padding
    sq += wq;
    sp += expf(vp[e] - mp);
    cross += in ? wq * vp[e] : 0.f;
  }
  sq = wave_sum(sq);
  sp = wave_sum(sp);
  cross = wave_sum(cross);
  if (lane == 0) { red_sum[wave][0] = sq; red_sum[wave][1] = sp; red_sum[wave][2] = cross; }
  __syncthreads();
  sq = ((red_sum[0][0] + red_sum[1][0]) + red_sum[2][0]) + red_sum[3][0];
  sp = ((red_sum[0][1] + red_sum[1][1]) + red_sum[2][1]) + red_sum[3][1];
  cross = ((red_sum[0][2] + red_sum[1][2]) + red_sum[2][2]) + red_sum[3][2];
  float *out = scratch + ((size_t)rowi * n_slices + slice) * slice_floats(k);
  if (t == 0) { out[0] = mq; out[1] = sq; out[2] = mp; out[3] = sp; out[4] = cross; }

  // Each wavefront finds the k best of its 1024 register-resident target logits and leaves them, best
  // first, in keys / cq / cp [wave * k ...].
  //
  // Filter first (k <= 64): tau = the k-th largest of the 64 LANE maxima.  At least k values are >= tau, so
  // every member of the wavefront's top k is >= tau; the values that pass are few (about k for scattered
  // data) and are compacted to one per lane, then ranked against each other.  If more than 64 pass (many
  // equal values), or k > 64, the general path below takes over: k rounds of a wave-wide argmax over all
  // 16 values of every lane.
  bool done = false;
  if (k <= 64) {
    float cur = vq[0];
#pragma unroll
    for (int e = 1; e < PER; e++) cur = fmaxf(cur, vq[e]);
    float tau = -INFINITY;
    for (int r = 0; r < k; r++) {                            // remove the largest lane maximum k times
      tau = wave_max_dpp(cur);
      const uint64_t holders = __ballot(cur == tau);
      if (lane == __ffsll((long long)holders) - 1) cur = -INFINITY;   // one lane per round (lowest), ties stay for later rounds
    }
    ckey[wave][lane] = 0ull;
    wave_lds_order();
    int n_pass = 0;
#pragma unroll
    for (int e = 0; e < PER; e++) {
      const int c = c0 + t + e * kLossThreads;
      const bool pass = c < vocab && vq[e] >= tau;
      const uint64_t mask = __ballot(pass);
      const int pos = n_pass + __popcll(mask & ((1ull << lane) - 1ull));
      if (pass && pos < 64) { ckey[wave][pos] = order_key(vq[e], c); cqv[wave][pos] = vq[e]; cpv[wave][pos] = vp[e]; }
      n_pass += __popcll(mask);
    }
    if (n_pass <= 64) {
      for (int r = lane; r < k; r += 64) { keys[wave * k + r] = 0ull; cq[wave * k + r] = -INFINITY; cp[wave * k + r] = 0.f; }
      wave_lds_order();
      const uint64_t mine = ckey[wave][lane];
      const int rank = key_rank(ckey[wave], 64, mine, lane);
      if (mine != 0ull && rank < k) { keys[wave * k + rank] = mine; cq[wave * k + rank] = cqv[wave][lane]; cp[wave * k + rank] = cpv[wave][lane]; }
      done = true;
    }
  }
  if (!done) {
  uint32_t taken = 0;
  for (int r = 0; r < k; r++) {
    float mv = -INFINITY;
#pragma unroll
    for (int e = 0; e < PER; e++) mv = fmaxf(mv, ((taken >> e) & 1u) ? -INFINITY : vq[e]);
    const float best_v = wave_max_dpp(mv);
    int mi = INT_MAX;
#pragma unroll
    for (int e = PER - 1; e >= 0; e--) {
      const int c = c0 + t + e * kLossThreads;
      if (!((taken >> e) & 1u) && c < vocab && vq[e] == best_v) mi = c;
    }
    const int best_i = wave_min_dpp(mi);
    if (lane == 0) { keys[wave * k + r] = order_key(best_v, best_i); cq[wave * k + r] = best_v; }
    if (best_i == INT_MAX) { if (lane == 0) cp[wave * k + r] = 0.f; }            // the wave ran out of tokens
    else if ((best_i - c0) % kLossThreads == t) {            // the owner supplies the draft logit of that token
      const int e_own = (best_i - c0) / kLossThreads;
      taken |= 1u << e_own;
      float pv = 0.f;
#pragma unroll
      for (int e = 0; e < PER; e++) pv = e == e_own ? vp[e] : pv;
      cp[wave * k + r] = pv;
    }
  }
  }
  if (t < 2) keys[kLossWaves * k + t] = 0ull;                // padding for the pairwise reads
  __syncthreads();
  for (int id = t; id < kLossWaves * k; id += kLossThreads) {
    const uint64_t key = keys[id];
    const int rank = key_rank(keys, (kLossWaves * k + 1) & ~1, key, id);
    if (rank < k) {
      const bool valid = key != 0ull;
      out[8 + 3 * rank + 0] = valid ? cq[id] : -INFINITY;
      out[8 + 3 * rank + 1] = __int_as_float(valid ? 0x7FFFFFFF - (int)(uint32_t)key : INT_MAX);
      out[8 + 3 * rank + 2] = valid ? cp[id] : 0.f;
    }
  }
}

constexpr int kLossMaxCand = 4096;
__global__ __launch_bounds__(kLossThreads) void loss_merge_kernel(int k, int n_slices, const float *scratch, float *loss_topk,
                                                                   float *loss_ce) {
  __shared__ __attribute__((aligned(16))) uint64_t keys[kLossMaxCand + 2];
  __shared__ float term[kLossMaxK];
  __shared__ float sh[4];                                    // lse_q, lse_p, cross / sum_q
  const int rowi = blockIdx.x, t = threadIdx.x;
  const float *base = scratch + (size_t)rowi * n_slices * slice_floats(k);
  const int n_cand = n_slices * k, n2 = (n_cand + 1) & ~1;
  for (int id = t; id < n2; id += kLossThreads) {
    const float *c = base + (size_t)(id / k) * slice_floats(k) + 8 + 3 * (id % k);
    keys[id] = id < n_cand ? order_key(c[0], __float_as_int(c[1])) : 0ull;
  }
  if (t < 64) {                                              // slices in ascending groups of 64, fixed butterfly inside
    float mq = -INFINITY, mp = -INFINITY;
    for (int sl = t; sl < n_slices; sl += 64) {
      const float *s = base + (size_t)sl * slice_floats(k);
      mq = fmaxf(mq, s[0]); mp = fmaxf(mp, s[2]);
    }
    mq = wave_max(mq); mp = wave_max(mp);
    float sq = 0.f, sp = 0.f, cr = 0.f;
    for (int s0 = 0; s0 < n_slices; s0 += 64) {
      const int sl = s0 + t;
      const float *s = base + (size_t)sl * slice_floats(k);
      const bool in = sl < n_slices;
      const float fq = in ? expf(s[0] - mq) : 0.f;
      sq += wave_sum(in ? s[1] * fq : 0.f);
      sp += wave_sum(in ? s[3] * expf(s[2] - mp) : 0.f);
      cr += wave_sum(in ? s[4] * fq : 0.f);
    }
    if (t == 0) { sh[0] = mq + logf(sq); sh[1] = mp + logf(sp); sh[2] = cr / sq; }
  }
  if (t < k) term[t] = 0.f;
  __syncthreads();
  const float lse_q = sh[0], lse_p = sh[1];
  for (int id = t; id < n_cand; id += kLossThreads) {
    const uint64_t key = keys[id];
    const int rank = key_rank(keys, n2, key, id);
    if (rank < k && key != 0ull) {
      const float *c = base + (size_t)(id / k) * slice_floats(k) + 8 + 3 * (id % k);
      term[rank] = expf(c[0] - lse_q) * (c[2] - lse_p);
    }
  }
  __syncthreads();
  if (t == 0) {
    float acc = 0.f;
    for (int r = 0; r < k; r++) acc += term[r];              // rank order
    loss_topk[rowi] = -acc;
    loss_ce[rowi] = lse_p - sh[2];                           // - sum q (zp - lse_p)
  }
}

// out[0] = sum of a[0..n), out[1] = sum of b[0..n); one workgroup, fixed order
__global__ __launch_bounds__(kLossThreads) void loss_total_kernel(const float *a, const float *b, int n, float *out) {
  __shared__ float shv[16];
  float sa = 0.f, sb = 0.f;
  for (int i = threadIdx.x; i < n; i += kLossThreads) { sa += a[i]; sb += b[i]; }
  sa = block_sum(sa, shv);
  sb = block_sum(sb, shv);
  if (threadIdx.x == 0) { out[0] = sa; out[1] = sb; }
}

}  // namespace

size_t topk_loss_scratch_floats(int rows, int vocab, int k) {
  const int n_slices = (vocab + kTopkSlice - 1) / kTopkSlice;
  return (size_t)rows * n_slices * slice_floats(k);
}

hipError_t launch_topk_loss_rows(const float *zq, const float *zp, int ldz, int rows, int vocab, int k, float *scratch,
                                 float *loss_topk, float *loss_ce, hipStream_t st) {
  const int n_slices = (vocab + kTopkSlice - 1) / kTopkSlice;
  if (rows < 1 || rows > 65535 || vocab < 1 || ldz < vocab || k < 1 || k > kLossMaxK || k > vocab || n_slices * k > kLossMaxCand)
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(loss_slice_kernel, dim3(n_slices, rows), dim3(kLossThreads), 0, st, zq, zp, ldz, vocab, k, n_slices, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(loss_merge_kernel, dim3(rows), dim3(kLossThreads), 0, st, k, n_slices, scratch, loss_topk, loss_ce);
  return hipGetLastError();
}

hipError_t launch_loss_total(const float *loss_topk, const float *loss_ce, int rows, float *out, hipStream_t st) {
  hipLaunchKernelGGL(loss_total_kernel, dim3(1), dim3(kLossThreads), 0, st, loss_topk, loss_ce, rows, out);
  return hipGetLastError();
}

}  // namespace spec
