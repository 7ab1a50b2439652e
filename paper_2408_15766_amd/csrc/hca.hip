// Training attention of harmonized context alignment (Sec. 3.2, appendix A.1) on the matrix cores.
//
// Streams m = 0 .. J-1 each hold keys/values for all T positions (stream 0 from the target's features,
// stream m from the draft features of training step m).  Query t (taken from stream J-1) sees
//   positions s <= t-(J-1)        from stream 0                      -> the "old" region, and
//   position  s  = t-o, o <= J-2  from stream J-1-o                  -> the "band": one key per stream.
// The old region is ordinary causal attention with the diagonal moved J-1 places and runs as a
// flash-attention loop over blocks of kBlockKeys keys staged in LDS.  The band is J-1 single keys per
// query, different for every query, and is folded in afterwards by the lanes that own the query.
//
// Work decomposition: a workgroup = 4 wavefronts = 128 consecutive queries of one (batch, head); a wavefront
// owns 32 queries (one MFMA column block).  S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16, so a
// lane holds, for ITS query (lane % 32), 16 keys of every 32-key tile and 64 of the 128 output dims, and
// the softmax needs one exchange with lane ^ 32 only.
#include "common.h"
#include "kernels.h"

namespace spec {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int kHcaWaves = 4;
constexpr int kHcaThreads = kHcaWaves * 64;
constexpr int kHcaRows = kHcaWaves * 32;      // queries per workgroup
constexpr int kKeyTiles = 2;                  // 32-key MFMA tiles per staged block
constexpr int kBlockKeys = 32 * kKeyTiles;

__device__ __forceinline__ f32x16_t mfma16(const u32x4_t &a, const u32x4_t &b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
__device__ __forceinline__ float lo_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

template <int HD> struct HcaLds {
  static constexpr int kstr = HD * 2 + 16;              // bytes per staged key row (+16: conflict-free b128 reads)
  static constexpr int vstr = kBlockKeys * 2 + 8;       // bytes per dim row of V^T (+8: conflict-free b64 reads)
  static constexpr int buf = kBlockKeys * kstr + HD * vstr;
  static constexpr int brow = HD * 2 + 16;              // band scratch: bytes per key (or value) row
  static constexpr int bwave = 2 * 32 * brow;           // ... per wavefront: 32 key rows + 32 value rows
  static constexpr int total = 2 * buf > kHcaWaves * bwave ? 2 * buf : kHcaWaves * bwave;   // main loop double-buffered
};

// Orders this wavefront's LDS writes before its later LDS reads of other lanes' data.  The LDS executes
// one wavefront's operations in issue order, so only the compiler has to be kept from reordering them.
__device__ __forceinline__ void wave_lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int HD>
__global__ __launch_bounds__(kHcaThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void hca_attention_kernel(HcaArgs a) {
  using L = HcaLds<HD>;
  constexpr int DB = HD / 32;                 // 32-dim blocks of the output
  constexpr int KK = HD / 16;                 // MFMA steps of q.k
  constexpr int PPR = HD * 2 / 16;            // 16-byte pieces per key row
  constexpr int KP = kBlockKeys * PPR / kHcaThreads;          // K pieces per thread per block
  constexpr int VP = kBlockKeys / 2 * PPR / kHcaThreads;      // V (key pair, piece) items per thread per block
  static_assert(kBlockKeys * PPR % kHcaThreads == 0 && (kBlockKeys / 2 * PPR) % kHcaThreads == 0, "staging split");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  // Workgroup id -> (batch, kv head, head of the group, query tile).  Ids 8 apart run on one XCD: all tiles and heads that
  // read the same keys/values are placed there.  An XCD's (batch, kv head) groups are taken in chunks of up to kHcaChunk;
  // inside a chunk the workgroups go LONGEST TILE FIRST across its groups (the causal mask makes the last tile the
  // longest, and a launch of a few workgroups per slot ends when its last long tile does), the heads of one group next to
  // each other so that they share the keys and values through L2.  The chunk bounds the keys and values in use at a time:
  // tile-major order over 64 groups per XCD (batch 16) runs at 490 TFLOP/s where group-major order reaches 659; over the
  // 8 groups of the batch-2 launch it is 23 % faster than group-major.  (With a number of groups that is not a multiple
  // of 8 the XCD placement would leave XCDs idle or uneven; the ids then run chunk by chunk over all groups.)
  constexpr int kHcaChunk = 8;
  const int G = a.hq / a.hkv;
  const int n_qt = (a.seq + kHcaRows - 1) / kHcaRows;
  const int n_grp = a.batch * a.hkv;
  const bool affine = (n_grp & 7) == 0;
  const int grp_per_list = affine ? n_grp >> 3 : n_grp;      // groups whose workgroups form one ordered list
  const int r_id = affine ? (int)blockIdx.x >> 3 : (int)blockIdx.x;
  const int chunk_wgs = kHcaChunk * G * n_qt;                // workgroups of a full chunk
  const int chunk = r_id / chunk_wgs, in_chunk = r_id % chunk_wgs;
  const int chunk_grps = min(kHcaChunk, grp_per_list - chunk * kHcaChunk);   // the last chunk may be short
  const int qt = n_qt - 1 - in_chunk / (chunk_grps * G);
  const int in_tile = in_chunk % (chunk_grps * G);
  const int gh = in_tile % G;
  const int grp_local = chunk * kHcaChunk + in_tile / G;
  const int grp = affine ? grp_local * 8 + ((int)blockIdx.x & 7) : grp_local;
  const int bi = grp / a.hkv, hk = grp % a.hkv;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 31, g = lane >> 5;
  const int T = a.seq, J = a.n_streams;
  const float c2 = a.scale_log2e;
  const size_t kv_stride = (size_t)a.hkv * HD;                // elements between consecutive positions
  const size_t kv_off = (size_t)bi * T * kv_stride + (size_t)hk * HD;
  const bf16_t *kg = (const bf16_t *)a.k[0] + kv_off;
  const bf16_t *vg = (const bf16_t *)a.v[0] + kv_off;

  const int r0 = qt * kHcaRows + wave * 32;   // first query of the wavefront
  const int t = r0 + c;
  const int tq = min(t, T - 1);               // queries past the end compute on the last one and are not stored
  const int lim = tq - (J - 1);               // last old-region key of this query (may be negative: none)
  const int wg_lim = min(qt * kHcaRows + kHcaRows - 1, T - 1) - (J - 1);
  const int nb = wg_lim >= 0 ? wg_lim / kBlockKeys + 1 : 0;
  const int wave_lim = min(r0 + 31, T - 1) - (J - 1);

  // Per-thread byte offsets of its pieces inside a key block, computed once; a block's loads are then a
  // uniform base plus these.  Only a block that reaches past the sequence end needs per-key clamping
  // (keys past the end are masked for every query; they are read from the last position).
  constexpr uint32_t kEsz = 2;
  uint32_t koff[KP], voff[VP];
#pragma unroll
  for (int e = 0; e < KP; e++) {
    const int q = tid + e * kHcaThreads;
    koff[e] = (uint32_t)((q / PPR) * kv_stride + (q % PPR) * 8) * kEsz;
  }
#pragma unroll
  for (int e = 0; e < VP; e++) {
    const int q = tid + e * kHcaThreads;
    voff[e] = (uint32_t)((2 * (q % (kBlockKeys / 2))) * kv_stride + (q / (kBlockKeys / 2)) * 8) * kEsz;
  }
  const uint32_t row_bytes = (uint32_t)kv_stride * kEsz;
  u32x4_t kreg[KP], vreg[VP][2];
  auto prefetch = [&](int blk) {
    const size_t blk_off = (size_t)blk * kBlockKeys * row_bytes;
    const unsigned char *kbase = (const unsigned char *)kg + blk_off, *vbase = (const unsigned char *)vg + blk_off;
    if (blk * kBlockKeys + kBlockKeys <= T) {
#pragma unroll
      for (int e = 0; e < KP; e++) kreg[e] = *(const u32x4_t *)(kbase + koff[e]);
#pragma unroll
      for (int e = 0; e < VP; e++) {
        vreg[e][0] = *(const u32x4_t *)(vbase + voff[e]);
        vreg[e][1] = *(const u32x4_t *)(vbase + voff[e] + row_bytes);
      }
    } else {
#pragma unroll
      for (int e = 0; e < KP; e++) {
        const int q = tid + e * kHcaThreads;
        const int key = min(blk * kBlockKeys + q / PPR, T - 1);
        kreg[e] = *(const u32x4_t *)(kg + (size_t)key * kv_stride + (q % PPR) * 8);
      }
#pragma unroll
      for (int e = 0; e < VP; e++) {
        const int q = tid + e * kHcaThreads;
        const int pair = q % (kBlockKeys / 2), piece = q / (kBlockKeys / 2);
        const int key0 = min(blk * kBlockKeys + 2 * pair, T - 1), key1 = min(blk * kBlockKeys + 2 * pair + 1, T - 1);
        vreg[e][0] = *(const u32x4_t *)(vg + (size_t)key0 * kv_stride + piece * 8);
        vreg[e][1] = *(const u32x4_t *)(vg + (size_t)key1 * kv_stride + piece * 8);
      }
    }
  };
  auto stage = [&](int buf) {
    unsigned char *k_lds = lds + buf * L::buf, *vt_lds = k_lds + kBlockKeys * L::kstr;
#pragma unroll
    for (int e = 0; e < KP; e++) {
      const int q = tid + e * kHcaThreads;
      *(u32x4_t *)(k_lds + (q / PPR) * L::kstr + (q % PPR) * 16) = kreg[e];
    }
#pragma unroll
    for (int e = 0; e < VP; e++) {                            // V^T[dim][key], two keys per 32-bit store
      const int q = tid + e * kHcaThreads;
      const int pair = q % (kBlockKeys / 2), piece = q / (kBlockKeys / 2);
      const uint32_t w0[4] = {vreg[e][0].x, vreg[e][0].y, vreg[e][0].z, vreg[e][0].w};
      const uint32_t w1[4] = {vreg[e][1].x, vreg[e][1].y, vreg[e][1].z, vreg[e][1].w};
#pragma unroll
      for (int d2 = 0; d2 < 8; d2++) {
        const uint32_t x = (d2 & 1) ? ((w0[d2 >> 1] >> 16) | (w1[d2 >> 1] & 0xFFFF0000u))
                                    : ((w0[d2 >> 1] & 0xFFFFu) | (w1[d2 >> 1] << 16));
        *(uint32_t *)(vt_lds + (piece * 8 + d2) * L::vstr + pair * 4) = x;
      }
    }
  };

  // V^T fragment (A operand) of 16-key step st = 2*tile + half and dim block db: keys step*16 + 4g + {0..3, 8..11}
  auto vread = [&](const unsigned char *vt_lds, int st, int db) {
    const unsigned char *vp = vt_lds + (db * 32 + c) * L::vstr + (16 * st + 4 * g) * 2;
    const u32x2_t v0 = *(const u32x2_t *)vp, v1 = *(const u32x2_t *)(vp + 16);
    return u32x4_t{v0.x, v0.y, v1.x, v1.y};
  };

  // query fragments (B operand): step kk covers dims kk*16 + g*8 .. +8 of query c.  They are requested before
  // the band rows and the first key block: loads complete in order, so once that block has arrived nothing in
  // the main loop waits on the memory counter for the queries' sake (such a wait would also stall on the
  // block in flight).
  const bf16_t *qrow = (const bf16_t *)a.q + (((size_t)bi * T + tq) * a.hq + (size_t)hk * G + gh) * HD;
  u32x4_t qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; kk++) qf[kk] = *(const u32x4_t *)(qrow + kk * 16 + g * 8);

  f32x16_t o[DB];
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int v = 0; v < 16; v++) o[db][v] = 0.f;
  // running maximum (of score * scale * log2 e) and sum of 2^(score' - maximum)
  float m_run = -INFINITY, l_run = 0.f;

  // The band first (its loads travel together with the first key block's): key t-off of stream J-1-off,
  // off = J-2 .. 0.  The 32 queries of the wavefront need 32 consecutive rows of that stream: they are read
  // with coalesced 16-byte accesses (a row = PPR lanes) into the wavefront's own LDS area, and then every
  // lane pair (c, c+32) picks up the row of ITS query, splitting the dot product by the dims of its query
  // fragments and the value row by the dims of its output registers.  No other wavefront is involved; the
  // workgroup barrier below separates this use of the LDS from the key blocks'.
  {
    unsigned char *bk = lds + wave * L::bwave, *bv = bk + 32 * L::brow;
    constexpr int BP = 32 * PPR / 64;                         // 16-byte pieces per lane per tensor
    for (int off = J - 2; off >= 0; off--) {
      const bf16_t *kb = (const bf16_t *)a.k[J - 1 - off] + kv_off;
      const bf16_t *vb = (const bf16_t *)a.v[J - 1 - off] + kv_off;
      u32x4_t kw_[BP], vw_[BP];
#pragma unroll
      for (int e = 0; e < BP; e++) {
        const int idx = lane + 64 * e;
        const int row = min(max(r0 + idx / PPR - off, 0), T - 1);
        kw_[e] = *(const u32x4_t *)(kb + (size_t)row * kv_stride + (idx % PPR) * 8);
        vw_[e] = *(const u32x4_t *)(vb + (size_t)row * kv_stride + (idx % PPR) * 8);
      }
#pragma unroll
      for (int e = 0; e < BP; e++) {
        const int idx = lane + 64 * e;
        *(u32x4_t *)(bk + (idx / PPR) * L::brow + (idx % PPR) * 16) = kw_[e];
        *(u32x4_t *)(bv + (idx / PPR) * L::brow + (idx % PPR) * 16) = vw_[e];
      }
      wave_lds_order();
      const bool have = tq - off >= 0;
      float dot = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; kk++) {
        const u32x4_t kw = *(const u32x4_t *)(bk + c * L::brow + kk * 32 + g * 16);
        const uint32_t kx[4] = {kw.x, kw.y, kw.z, kw.w}, qx[4] = {qf[kk].x, qf[kk].y, qf[kk].z, qf[kk].w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
          dot = fmaf(lo_f32(qx[e]), lo_f32(kx[e]), dot);
          dot = fmaf(hi_f32(qx[e]), hi_f32(kx[e]), dot);
        }
      }
      dot += __shfl_xor(dot, 32, 64);
      const float sc = have ? dot * c2 : -INFINITY;
      const float m_new = fmaxf(m_run, sc);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float corr = __builtin_amdgcn_exp2f(m_run - m_use);
      const float p = have ? __builtin_amdgcn_exp2f(sc - m_use) : 0.f;
      l_run = l_run * corr + p;
      m_run = m_new;
#pragma unroll
      for (int db = 0; db < DB; db++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          const u32x2_t vw = *(const u32x2_t *)(bv + c * L::brow + (db * 32 + 8 * q4 + 4 * g) * 2);
          o[db][4 * q4 + 0] = fmaf(p, lo_f32(vw.x), o[db][4 * q4 + 0] * corr);
          o[db][4 * q4 + 1] = fmaf(p, hi_f32(vw.x), o[db][4 * q4 + 1] * corr);
          o[db][4 * q4 + 2] = fmaf(p, lo_f32(vw.y), o[db][4 * q4 + 2] * corr);
          o[db][4 * q4 + 3] = fmaf(p, hi_f32(vw.y), o[db][4 * q4 + 3] * corr);
        }
      wave_lds_order();                                       // the next stream's rows overwrite the area
    }
  }
  __syncthreads();

  if (nb > 0) {
    prefetch(0);
    stage(0);
    __syncthreads();
    if (nb > 1) prefetch(1);
  }
  for (int blk = 0; blk < nb; blk++) {
    const int cur = blk & 1;
    const unsigned char *k_lds = lds + cur * L::buf, *vt_lds = k_lds + kBlockKeys * L::kstr;
    const bool act = blk * kBlockKeys <= wave_lim;            // wavefront-uniform: some query here sees this block
    // The next block is staged first (into the buffer every wavefront left at the last barrier), from the
    // registers its loads filled during the previous iteration; the loads of the block after it follow.
    if (blk + 1 < nb) {
      stage(cur ^ 1);
      if (blk + 2 < nb) prefetch(blk + 2);
    }
    if (act) {
      f32x16_t s[kKeyTiles];
#pragma unroll
      for (int kt = 0; kt < kKeyTiles; kt++) {
#pragma unroll
        for (int v = 0; v < 16; v++) s[kt][v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; kk++) {
          const u32x4_t kf = *(const u32x4_t *)(k_lds + (kt * 32 + c) * L::kstr + kk * 32 + g * 16);
          s[kt] = mfma16(kf, qf[kk], s[kt]);
        }
      }
      // s[kt][v] = q . k for key blk*kBlockKeys + kt*32 + 8*(v/4) + 4*g + v%4 and query c
      if (blk * kBlockKeys + kBlockKeys - 1 > r0 - (J - 1)) {  // the block reaches past some query's region
        const int key0 = blk * kBlockKeys + 4 * g;
#pragma unroll
        for (int kt = 0; kt < kKeyTiles; kt++)
#pragma unroll
          for (int v = 0; v < 16; v++)
            if (key0 + kt * 32 + 8 * (v >> 2) + (v & 3) > lim) s[kt][v] = -INFINITY;
      }
      float mb = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < kKeyTiles; kt++)
#pragma unroll
        for (int v = 0; v < 16; v++) mb = fmaxf(mb, s[kt][v]);
      mb = fmaxf(mb, __shfl_xor(mb, 32, 64));
      // The reference maximum moves only when the block's maximum exceeds it by more than 2^8: until then
      // the probabilities are taken against the old reference (at most 2^8, harmless in fp32 and bf16, and
      // the final division by the sum cancels the choice), and the 64 output registers are left alone.
      const float mb2 = mb * c2;
      const bool move = mb2 > m_run + 8.f;                     // also the first finite maximum after -inf
      if (__any(move)) {
        const float m_new = move ? mb2 : m_run;
        const float corr = move ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;   // m_new is finite where move
        l_run *= corr;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < DB; db++)
#pragma unroll
          for (int v = 0; v < 16; v++) o[db][v] *= corr;
      }
      const float m_use = m_run == -INFINITY ? 0.f : m_run;    // nothing seen yet: every term below becomes 0
      // Per 32-key tile: probabilities (vector ALU), then O^T += V^T P^T in two 16-key steps (matrix cores);
      // step (kt, h) uses the lane's own values v = 8h .. 8h+7 of tile kt, i.e. keys kt*32 + 16h + 8*(e/4) + 4g
      // + e%4, and V^T supplies the same keys per dim.  The tiles are independent, so the second tile's
      // vector arithmetic can run while the first tile's matrix instructions execute.
      float ls = 0.f;
#pragma unroll
      for (int kt = 0; kt < kKeyTiles; kt++) {
        float p[16];
        uint32_t pk[8];                                       // probabilities, two bf16 per word
#pragma unroll
        for (int v = 0; v < 16; v++) { p[v] = __builtin_amdgcn_exp2f(fmaf(s[kt][v], c2, -m_use)); ls += p[v]; }
#pragma unroll
        for (int e = 0; e < 8; e++) pk[e] = pack_bf16x2(p[2 * e], p[2 * e + 1]);
#pragma unroll
        for (int h = 0; h < 2; h++) {
          const u32x4_t pf = {pk[4 * h], pk[4 * h + 1], pk[4 * h + 2], pk[4 * h + 3]};
#pragma unroll
          for (int db = 0; db < DB; db++) o[db] = mfma16(vread(vt_lds, 2 * kt + h, db), pf, o[db]);
        }
      }
      ls += __shfl_xor(ls, 32, 64);
      l_run += ls;
    }
    __syncthreads();                                          // block blk+1 staged; everyone is done with block blk
  }

  if (t >= T) return;
  const float inv = 1.f / l_run;
  bf16_t *orow = (bf16_t *)a.out + (((size_t)bi * T + t) * a.hq + (size_t)hk * G + gh) * HD;
#pragma unroll
  for (int db = 0; db < DB; db++)
#pragma unroll
    for (int q4 = 0; q4 < 4; q4++) {
      u32x2_t w;
      w.x = pack_bf16x2(o[db][4 * q4 + 0] * inv, o[db][4 * q4 + 1] * inv);
      w.y = pack_bf16x2(o[db][4 * q4 + 2] * inv, o[db][4 * q4 + 3] * inv);
      *(u32x2_t *)(orow + db * 32 + 8 * q4 + 4 * g) = w;
    }
}

template <int HD>
hipError_t launch_hd(const HcaArgs &a, hipStream_t st) {
  static bool attr_done[64] = {};                             // per device: the attribute belongs to the device's copy of the code
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64 || !attr_done[dev]) {
    e = hipFuncSetAttribute((const void *)hca_attention_kernel<HD>, hipFuncAttributeMaxDynamicSharedMemorySize, HcaLds<HD>::total);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64) attr_done[dev] = true;
  }
  const int G = a.hq / a.hkv;
  const int n_qt = (a.seq + kHcaRows - 1) / kHcaRows;
  const long long grid = (long long)a.batch * a.hkv * G * n_qt;
  if (grid > 0x7FFFFFFFll) return hipErrorInvalidValue;
  hipLaunchKernelGGL((hca_attention_kernel<HD>), dim3((unsigned)grid), dim3(kHcaThreads), HcaLds<HD>::total, st, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_hca_attention(const HcaArgs &a, hipStream_t st) {
  if (a.n_streams < 1 || a.n_streams > kMaxStreams || a.batch < 1 || a.seq < 1 || a.hkv < 1 || a.hq < a.hkv || a.hq % a.hkv)
    return hipErrorInvalidValue;
  if (a.hd == 128) return launch_hd<128>(a, st);
  if (a.hd == 64) return launch_hd<64>(a, st);
  return hipErrorInvalidValue;
}

}  // namespace spec
