// Shared device helpers for the gfx950 kernels: storage types, conversions,
// wavefront (64-lane) reductions.  Nothing here is shared with the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spec {

constexpr int kWave = 64;

// bfloat16 kept as raw bits; arithmetic is always done in fp32.
struct bf16_t { uint16_t v; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {   // round to nearest, ties to even (v_cvt_pk_bf16_f32)
  return __builtin_bit_cast(uint16_t, (__bf16)f);
}
// two floats -> two bf16 in one dword (lo in the low half), one hardware conversion
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 b2_t;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2_t{lo, hi}, b2_t));
}
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_bits_to_f32(x.v); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { bf16_t r; r.v = f32_to_bf16_bits(x); return r; }

// SwiGLU of one (gate, up) pair: silu(g) * u with silu(g) = g / (1 + e^-g), through the hardware's exp2 and reciprocal
// (about 1 ulp each; the result is rounded to the storage type afterwards).  Every kernel that forms the activation
// uses this one expression.
__device__ __forceinline__ float silu_mul(float g, float u) {
  const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);      // e^-g; large |g|: 0 or +inf, both give the right limit
  return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

// Rotary embedding of the plane (a, b) = (dim j, dim j + hd/2) by (cos, sin).  Contraction into fused multiply-adds is
// switched off here: which product the compiler would fuse depends on the surrounding code, and every kernel that
// rotates the same inputs has to get the same bits.
__device__ __forceinline__ float rope_first(float a, float b, float2 cs) {
#pragma clang fp contract(off)
  const float x = a * cs.x, y = b * cs.y;
  return x - y;
}
__device__ __forceinline__ float rope_second(float a, float b, float2 cs) {
#pragma clang fp contract(off)
  const float x = b * cs.x, y = a * cs.y;
  return x + y;
}

// A store of a result that the NEXT kernel reads (on other XCDs), written through to device scope right away
// instead of staying dirty in this XCD's L2 until the end-of-kernel write-back.  Pays for the GEMM's partial sums
// (the reducing kernel that follows starts ~1 % of a cycle earlier, summed over a forward); the same for the row
// kernels changes nothing and for the attention partials, many small stores per lane, it costs 7 % of a verify.
__device__ __forceinline__ void store_through(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void store_through(uint32_t *p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Store of one activation value per lane, adjacent lanes holding adjacent columns of the same row (lane parity = column
// parity).  bf16: the even lane writes its own and its neighbour's value (nx, fetched by the caller with a lane shift) as
// one written-through dword when the row length is even (`pairs`: then p is 4-byte aligned for even columns); `next`
// says that the neighbour's column exists.
__device__ __forceinline__ void store_act(float *p, float r, float, bool ok, bool, bool, int) {
  if (ok) store_through(p, r);
}
__device__ __forceinline__ void store_act(bf16_t *p, float r, float nx, bool ok, bool pairs, bool next, int lane) {
  if (!ok) return;
  if (!pairs) p->v = f32_to_bf16_bits(r);
  else if (!(lane & 1)) {
    if (next) store_through((uint32_t *)p, pack_bf16x2(r, nx));
    else p->v = f32_to_bf16_bits(r);
  }
}

// Butterfly reductions over the 64 lanes of a wavefront; every lane gets the result.
// The exchange pattern is fixed, so the result does not depend on the data.
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ int wave_min_i(int x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = min(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ int wave_sum_i(int x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// Order-independent reductions (max, min) without LDS traffic: four DPP exchanges inside each row of 16
// lanes (xor 1, xor 2, mirror within 8, mirror within 16), then the four row results are read lane by lane.
// Needs all 64 lanes active.  Every lane gets the result.
template <int CTRL> __device__ __forceinline__ int dpp_i32(int x) { return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, true); }
template <int CTRL> __device__ __forceinline__ float dpp_f32(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float wave_max_dpp(float x) {
  x = fmaxf(x, dpp_f32<0xB1>(x));     // quad_perm [1,0,3,2]
  x = fmaxf(x, dpp_f32<0x4E>(x));     // quad_perm [2,3,0,1]
  x = fmaxf(x, dpp_f32<0x141>(x));    // row_half_mirror
  x = fmaxf(x, dpp_f32<0x140>(x));    // row_mirror
  const int b = __float_as_int(x);
  return fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 0)), __int_as_float(__builtin_amdgcn_readlane(b, 16))),
               fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 32)), __int_as_float(__builtin_amdgcn_readlane(b, 48))));
}
__device__ __forceinline__ int wave_min_dpp(int x) {
  x = min(x, dpp_i32<0xB1>(x));
  x = min(x, dpp_i32<0x4E>(x));
  x = min(x, dpp_i32<0x141>(x));
  x = min(x, dpp_i32<0x140>(x));
  return min(min(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
             min(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}

// (value, index) pair ordered by larger value first, then lower index.
struct ValIdx { float v; int i; };
__device__ __forceinline__ bool better(float v, int i, float v2, int i2) { return v > v2 || (v == v2 && i < i2); }
__device__ __forceinline__ ValIdx wave_best(ValIdx a) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(a.v, o, 64);
    int oi = __shfl_xor(a.i, o, 64);
    if (better(ov, oi, a.v, a.i)) { a.v = ov; a.i = oi; }
  }
  return a;
}

// The same order as one unsigned 64-bit key (larger key = earlier): the value mapped monotonically to
// unsigned (-0 folded into +0), then the complemented index.  An empty entry (index INT_MAX) gets key 0,
// below every real entry.
__device__ __forceinline__ uint64_t order_key(float v, int i) {
  if (i == 0x7FFFFFFF) return 0ull;
  uint32_t u = __float_as_uint(v + 0.f);
  u ^= (u >> 31) ? 0xFFFFFFFFu : 0x80000000u;
  return ((uint64_t)u << 32) | (uint32_t)(0x7FFFFFFF - i);
}
// Number of keys ordered before key `k` held at list position `me`: larger keys, and equal keys (empty
// entries) at earlier positions.  `keys` is in LDS, 16-byte aligned, n2 (even) entries, zero-padded.
__device__ __forceinline__ int key_rank(const uint64_t *keys, int n2, uint64_t k, int me) {
  typedef __attribute__((ext_vector_type(2))) uint64_t u64x2_t;
  int rank = 0;
#pragma unroll 4
  for (int o = 0; o < n2; o += 2) {
    const u64x2_t kk = *(const u64x2_t *)(keys + o);
    rank += (kk.x > k || (kk.x == k && o < me)) ? 1 : 0;
    rank += (kk.y > k || (kk.y == k && o + 1 < me)) ? 1 : 0;
  }
  return rank;
}

// Block-wide sum for blocks of up to 16 waves; `sh` needs 16 floats.  Fixed order.
__device__ __forceinline__ float block_sum(float x, float *sh) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  x = wave_sum(x);
  __syncthreads();
  if (lane == 0) sh[w] = x;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; i++) t += sh[i];
  return t;
}
__device__ __forceinline__ float block_max(float x, float *sh) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  x = wave_max(x);
  __syncthreads();
  if (lane == 0) sh[w] = x;
  __syncthreads();
  float t = sh[0];
  for (int i = 1; i < nw; i++) t = fmaxf(t, sh[i]);
  return t;
}
__device__ __forceinline__ ValIdx block_best(ValIdx a, float *shv, int *shi) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  a = wave_best(a);
  __syncthreads();
  if (lane == 0) { shv[w] = a.v; shi[w] = a.i; }
  __syncthreads();
  ValIdx t{shv[0], shi[0]};
  for (int i = 1; i < nw; i++) if (better(shv[i], shi[i], t.v, t.i)) { t.v = shv[i]; t.i = shi[i]; }
  return t;
}

}  // namespace spec
