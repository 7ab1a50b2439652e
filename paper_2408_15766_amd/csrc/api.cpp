// libspec: host side of the speculative-decoding hot path (state machine, workspace layout,
// launch sequences).  Every arithmetic step runs in the gfx950 kernels; this file only orders
// launches on the context's stream and moves a few hundred bytes per cycle across the boundary.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/spec.h"
#include "kernels.h"

using namespace spec;

namespace {

enum State { CREATED = 0, READY = 1, DRAFTED = 2, VERIFIED = 3 };

constexpr int kPrefillChunk = 512;     // prompt rows per target forward during prefill
// A captured forward sizes its attention launches for a bound on the key positions, not for the positions of
// the cycle it was captured in.  The bound is the context rounded up to the next multiple of kGraphBucket, and
// the graph is captured again when the context outgrows it: sizing for max_seq instead costs 2-9 % of the verify
// at a 512-token context (workgroups that find nothing to do still have to be dispatched).
constexpr int kGraphBucket = 256;
constexpr int kDraftNodeStream = 1 << 16;  // random stream of node i's child sampling: (cycle, kDraftNodeStream + i)
constexpr int kMaxGemmEvents = 2048;  // event pairs kept per cycle at profile level 2

struct GemmPlan { int n_split; };

struct RowTables {                    // device index tables describing the rows of one forward
  const int *token, *pos, *slot, *depth, *anc;
};

struct HostStage {                    // pinned host staging, one allocation
  int tree_n;
  int base;                           // committed tokens at the time of the verify (read by replayed kernels)
  int tok[kMaxNodes], par[kMaxNodes], dep[kMaxNodes];
  float sc[kMaxNodes];
  int pos[kMaxNodes], slot[kMaxNodes];
  int anc[kMaxNodes * kAncStride];
  AcceptResult acc;
  int first_token;
};

thread_local std::string g_create_error;   // last spec_create failure of the calling thread

}  // namespace

struct spec_ctx {
  spec_config cfg;
  spec_weights w;
  std::vector<spec_layer_weights> layers;
  hipStream_t stream = nullptr;
  int state = CREATED;
  int n = 0;            // tokens committed to the target cache
  int n_pend = 0;       // pending (feature, token) pairs for the next draft root step
  int root = -1;        // pending root token (host copy)
  uint32_t cycle = 0;
  int last_nodes = 0;
  int esz = 4;
  int m_max = 0;        // largest row count of any forward
  int max_parts = 0;
  int seq_draft = 0;    // draft cache capacity in rows
  std::string err;

  // device buffers (carved from the workspace)
  char *kv_t = nullptr, *kv_d = nullptr;
  size_t t_kv_stride = 0, t_layer_stride = 0, d_kv_stride = 0;   // in elements
  float *h = nullptr, *part = nullptr, *attn_part = nullptr, *logits = nullptr, *dlogits = nullptr;
  void *x = nullptr, *qbuf = nullptr, *attn_out = nullptr, *act = nullptr, *xcat = nullptr, *feats = nullptr,
       *gfeat = nullptr, *pend_feat = nullptr;
  float2 *rope = nullptr, *stats = nullptr, *sc_stat = nullptr;
  float *sc_val = nullptr, *top_lp = nullptr;
  int *sc_idx = nullptr, *top_tok = nullptr;
  int *d_prompt = nullptr, *d_pos = nullptr, *d_slot = nullptr, *d_depth = nullptr;
  int *pend_tok = nullptr, *root_tok = nullptr, *amax_idx = nullptr;
  float *amax_val = nullptr;
  // verify tree on the device: packed exactly like the head of HostStage (tree_n .. anc)
  int *t_n = nullptr, *t_base = nullptr, *t_tok = nullptr, *t_par = nullptr, *t_dep = nullptr, *t_pos = nullptr, *t_slot = nullptr, *t_anc = nullptr;
  float *t_sc = nullptr;
  DraftState ds{};
  AcceptResult *acc = nullptr;
  HostStage *stage = nullptr;
  size_t part_floats = 0;

  // static tree shape (spec_set_static_tree); n_nodes == 0: the dynamic tree of the configuration
  struct StaticHost {
    int n_nodes = 0, max_depth = 0, n_expanded = 0;       // n_expanded: nodes of depth >= 1 that have children
    bool sampled = false;
    int rows[kMaxDepth + 1] = {};                         // expanded nodes per depth (depth 0: the root, 1 if it has children)
    int width[kMaxDepth + 1] = {};                        // proposals needed per node of that depth (max over its nodes)
  } st;
  StaticTables st_tb{};
  int *st_qrow_of = nullptr, *st_enode = nullptr;         // device: node -> row of st_qrows; (depth, row) -> node
  float *st_qrows = nullptr;                              // device: draft logit rows of the expanded nodes (sampled children)

  // HIP graph of the verify forward (replayed every cycle; needs a non-default stream)
  bool graphs = true;
  hipGraphExec_t verify_exec = nullptr;
  int verify_exec_rows = 0;
  int verify_exec_bound = 0;              // largest key position the captured launches are sized for
  hipGraphExec_t expand_exec = nullptr;   // draft expansion steps 2..D + rerank
  int expand_exec_bound = 0;

  // profiling
  int prof_level = 0;
  hipEvent_t ev_phase[4][2] = {};
  bool phase_pending[4] = {};
  std::vector<hipEvent_t> ev_gemm;
  int n_gemm_ev = 0;
  int gemm_bucket = 0;                 // 4: inside verify, 5: inside draft
  std::vector<int> gemm_ev_bucket;
  double prof_ms[8] = {};
  int64_t prof_cnt[8] = {};
};

namespace {

int fail(spec_ctx *c, int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_create_error = buf;
  return code;
}

#define HIPCHK(c, expr)                                                                      \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) return fail((c), SPEC_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// The split count depends on the matrix shape only (never on the number of rows), so a token
// sees the same summation order in plain decoding and inside a tree.
// rows of the packed gate/up matrix: per 16 columns, 16 gate rows and 16 up rows
int gate_up_rows(int f) { return 32 * ((f + 15) / 16); }

GemmPlan plan_gemm(int total_rows, int in, int dtype) {
  const int blocks = (total_rows + 31) / 32;
  const int kslab = gemm_k_per_slab(dtype);
  const int slabs = (in + kslab - 1) / kslab;
  // Every wave streams one (32-row block, K range) unit and the launch spreads its units over all compute units
  // whatever the split count, so the count only trades parallel streams against partial-sum traffic.  Measured on
  // MI355X over the projections of the four benchmark shapes (M = 60):
  //  * at least 4 slabs per split, at most 8 splits;
  //  * the smallest count with 512 units or more (two streaming waves per compute unit): below that the launch is
  //    slower (7B O projection, 256 units 13.3 us, 512 units 9.8 us), above it each further split costs more in partial
  //    sums than it gains (7B down 20.6 us with 4 splits, 21.0 with 8; 70B O 26.0 with 2, 28.8 with 4);
  //  * a count up to twice that which divides the slabs evenly is taken instead (13B down, 54 slabs: 28.5 us with 4
  //    splits, 27.7 with 6; 8B QKV, 16 slabs: 12.5 us with 4);
  //  * streams that stay longer than 24 slabs are halved again while the units fit the chip's 1024 SIMDs (70B down,
  //    112 slabs: 80.8 us with 2 splits, 76.4 with 4).
  int smax = 1;
  while (smax < 8 && slabs / (smax + 1) >= 4) smax++;
  int s = 1;
  while (s < smax && blocks * s < 512) s++;
  for (int c = s; c <= smax && c <= 2 * s; c++)
    if (slabs % c == 0) { s = c; break; }
  while (2 * s <= smax && slabs / (2 * s) >= 24 && blocks * 2 * s <= 1024) s *= 2;
  GemmPlan p;
  p.n_split = s;
  return p;
}

struct Layout {                       // workspace carve-out; all offsets 256-byte aligned
  size_t total = 0;
  size_t take(size_t bytes) { size_t o = total; total = align_up(total + bytes); return o; }
};

bool config_ok(const spec_config *c, std::string *why) {
  auto bad = [&](const char *m) { if (why) *why = m; return false; };
  if (!c) return bad("cfg is NULL");
  if (c->dtype != SPEC_DTYPE_FP32 && c->dtype != SPEC_DTYPE_BF16) return bad("dtype must be 0 (fp32) or 1 (bf16)");
  if (c->n_layers < 1 || c->d_model < 1 || c->d_ffn < 1 || c->vocab < 1) return bad("non-positive model dimension");
  if (c->head_dim != 64 && c->head_dim != 128) return bad("head_dim must be 64 or 128");
  if (c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads != 0) return bad("n_q_heads must be a multiple of n_kv_heads");
  const int g = c->n_q_heads / c->n_kv_heads;
  if (g != 1 && g != 2 && g != 4 && g != 8) return bad("q heads per kv head must be 1, 2, 4 or 8");
  const int epl = c->dtype == SPEC_DTYPE_BF16 ? 8 : 4;
  if (c->d_model % epl || c->d_ffn % epl || (c->n_q_heads * c->head_dim) % epl) return bad("dimensions must be multiples of 16 bytes");
  if (c->tree_total < 1 || c->tree_total > SPEC_MAX_NODES) return bad("tree_total out of range");
  if (c->tree_total > 1) {
    if (c->tree_depth < 1 || c->tree_depth > SPEC_MAX_DEPTH) return bad("tree_depth out of range");
    if (c->tree_topk < 1 || c->tree_topk > SPEC_MAX_TOPK || c->tree_topk > c->vocab) return bad("tree_topk out of range");
  }
  if (c->max_seq < c->tree_total + 1) return bad("max_seq too small");
  if (!(c->temperature >= 0.f)) return bad("temperature must be >= 0");
  if (!(c->rope_theta > 1.f) || !(c->rms_eps >= 0.f)) return bad("rope_theta / rms_eps out of range");
  return true;
}

// Lays out the workspace; with ctx == nullptr only the size is computed.
size_t layout(const spec_config &c, spec_ctx *x, char *base) {
  Layout L;
  const size_t esz = c.dtype == SPEC_DTYPE_BF16 ? 2 : 4;
  const int d = c.d_model, dq = c.n_q_heads * c.head_dim, dkv = c.n_kv_heads * c.head_dim, f = c.d_ffn, v = c.vocab;
  const int m_max = std::max({c.tree_total, kPrefillChunk, kMaxDepth + 1, c.tree_topk});
  const int k = std::max(1, c.tree_topk), D = std::max(1, c.tree_depth);
  const int seq_draft = c.max_seq + D * k;
  const int max_parts = (c.max_seq + D * k) / kAttnPart + 2;   // parts of the longest row + the tail slot
  size_t part_floats = 0;
  {
    struct { int rows, in; } g[5] = {{dq + 2 * dkv, d}, {d, dq}, {gate_up_rows(f), d}, {d, f}, {d, 2 * d}};
    for (auto &e : g) {
      GemmPlan p = plan_gemm(e.rows, e.in, c.dtype);
      part_floats = std::max(part_floats, (size_t)p.n_split * m_max * e.rows);
    }
  }
#define TAKE(field, type, bytes) { size_t o_ = L.take(bytes); if (x) x->field = (type)(base + o_); }
  TAKE(kv_t, char *, (size_t)c.n_layers * 2 * c.max_seq * dkv * esz)
  TAKE(kv_d, char *, (size_t)2 * seq_draft * dkv * esz)
  TAKE(h, float *, (size_t)m_max * d * 4)
  TAKE(x, void *, (size_t)m_max * d * esz)
  TAKE(qbuf, void *, (size_t)m_max * dq * 4)
  TAKE(attn_out, void *, (size_t)m_max * dq * esz)
  TAKE(act, void *, (size_t)m_max * f * esz)
  TAKE(xcat, void *, (size_t)m_max * 2 * d * esz)
  TAKE(feats, void *, (size_t)m_max * d * esz)
  TAKE(gfeat, void *, (size_t)m_max * d * esz)
  TAKE(pend_feat, void *, (size_t)(kMaxDepth + 1) * d * esz)
  TAKE(part, float *, part_floats * 4)
  TAKE(attn_part, float *, (size_t)m_max * c.n_q_heads * max_parts * (c.head_dim + 2) * 4)
  TAKE(logits, float *, (size_t)std::max(c.tree_total, 1) * v * 4)
  TAKE(dlogits, float *, (size_t)kMaxTopK * v * 4)
  TAKE(rope, float2 *, (size_t)m_max * (c.head_dim / 2) * 8)
  TAKE(stats, float2 *, (size_t)kMaxNodes * argmax_slices(c.vocab) * 8)
  const int n_slices = (v + kTopkSlice - 1) / kTopkSlice;
  TAKE(sc_stat, float2 *, (size_t)kMaxTopK * n_slices * 8)
  TAKE(sc_val, float *, (size_t)kMaxTopK * n_slices * kMaxTopK * 4)
  TAKE(sc_idx, int *, (size_t)kMaxTopK * n_slices * kMaxTopK * 4)
  TAKE(top_tok, int *, (size_t)kMaxTopK * kMaxTopK * 4)
  TAKE(top_lp, float *, (size_t)kMaxTopK * kMaxTopK * 4)
  TAKE(d_prompt, int *, (size_t)c.max_seq * 4)
  TAKE(d_pos, int *, (size_t)m_max * 4)
  TAKE(d_slot, int *, (size_t)m_max * 4)
  TAKE(d_depth, int *, (size_t)m_max * 4)
  TAKE(pend_tok, int *, (size_t)(kMaxDepth + 1) * 4)
  TAKE(root_tok, int *, 256)
  TAKE(amax_val, float *, (size_t)kMaxNodes * argmax_slices(c.vocab) * 4)
  TAKE(amax_idx, int *, (size_t)kMaxNodes * argmax_slices(c.vocab) * 4)
  // verify tree: one contiguous block mirroring the head of HostStage, so one copy moves it
  {
    size_t o_ = L.take(offsetof(HostStage, acc));
    if (x) {
      char *b = base + o_;
      x->t_n = (int *)(b + offsetof(HostStage, tree_n));
      x->t_base = (int *)(b + offsetof(HostStage, base));
      x->t_tok = (int *)(b + offsetof(HostStage, tok));
      x->t_par = (int *)(b + offsetof(HostStage, par));
      x->t_dep = (int *)(b + offsetof(HostStage, dep));
      x->t_sc = (float *)(b + offsetof(HostStage, sc));
      x->t_pos = (int *)(b + offsetof(HostStage, pos));
      x->t_slot = (int *)(b + offsetof(HostStage, slot));
      x->t_anc = (int *)(b + offsetof(HostStage, anc));
    }
  }
  const int pool = k + (D - 1) * k * k;
  TAKE(ds.pool_tok, int *, (size_t)pool * 4)
  TAKE(ds.pool_par, int *, (size_t)pool * 4)
  TAKE(ds.pool_dep, int *, (size_t)pool * 4)
  TAKE(ds.pool_sc, float *, (size_t)pool * 4)
  TAKE(ds.n_pool, int *, 256)
  TAKE(ds.front_pool, int *, kMaxTopK * 4)
  TAKE(ds.front_tok, int *, kMaxTopK * 4)
  TAKE(ds.front_src, int *, kMaxTopK * 4)
  TAKE(ds.front_depth, int *, kMaxTopK * 4)
  TAKE(ds.front_anc, int *, kMaxTopK * kAncStride * 4)
  TAKE(ds.front_slot, int *, kMaxTopK * 4)
  TAKE(ds.front_pos, int *, kMaxTopK * 4)
  TAKE(acc, AcceptResult *, sizeof(AcceptResult))
#undef TAKE
  if (x) {
    x->esz = (int)esz; x->m_max = m_max; x->max_parts = max_parts; x->seq_draft = seq_draft;
    x->t_kv_stride = (size_t)c.max_seq * dkv; x->t_layer_stride = 2 * x->t_kv_stride;
    x->d_kv_stride = (size_t)seq_draft * dkv;
    x->part_floats = part_floats;
  }
  return L.total;
}

// ---- profiling helpers -----------------------------------------------------------------------
void phase_begin(spec_ctx *c, int phase) {
  if (c->prof_level >= 1) { (void)hipEventRecord(c->ev_phase[phase][0], c->stream); }
}
void phase_end(spec_ctx *c, int phase) {
  if (c->prof_level >= 1) { (void)hipEventRecord(c->ev_phase[phase][1], c->stream); c->phase_pending[phase] = true; }
}
// Call only after the stream has been synchronised.
void harvest_profile(spec_ctx *c) {
  if (c->prof_level < 1) return;
  for (int p = 0; p < 4; p++)
    if (c->phase_pending[p]) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, c->ev_phase[p][0], c->ev_phase[p][1]) == hipSuccess) { c->prof_ms[p] += ms; c->prof_cnt[p]++; }
      c->phase_pending[p] = false;
    }
  for (int i = 0; i < c->n_gemm_ev; i++) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->ev_gemm[2 * i], c->ev_gemm[2 * i + 1]) == hipSuccess) {
      c->prof_ms[c->gemm_ev_bucket[i]] += ms; c->prof_cnt[c->gemm_ev_bucket[i]]++;
    }
  }
  c->n_gemm_ev = 0;
}

// ---- launch sequences ------------------------------------------------------------------------
struct Seg { const void *w; int rows; };

int run_gemm(spec_ctx *c, const void *x, int ldx, int m, int in, const Seg *segs, int nseg, float *out, int ldp, int m_pad,
             const GemmPlan &p, void *swiglu_act = nullptr) {
  GemmArgs a{};
  a.act = swiglu_act;
  a.x = x; a.ldx = ldx; a.m = m; a.in = in; a.nseg = nseg;
  int col = 0, blocks = 0;
  for (int s = 0; s < 3; s++) {
    a.seg_w[s] = s < nseg ? segs[s].w : segs[0].w;
    a.seg_rows[s] = s < nseg ? segs[s].rows : 0;
    a.seg_blocks[s] = swiglu_act ? (a.seg_rows[s] + 15) / 16 : (a.seg_rows[s] + 31) / 32;   // SwiGLU: rows = columns of act, 16 per block
    a.seg_col0[s] = col;
    col += a.seg_rows[s];
    blocks += a.seg_blocks[s];
  }
  a.total_blocks = blocks;
  a.part = out; a.ldp = ldp; a.m_pad = m_pad;
  a.n_split = p.n_split;
  const bool ev = c->prof_level >= 2 && c->gemm_bucket && c->n_gemm_ev < kMaxGemmEvents;
  if (ev) (void)hipEventRecord(c->ev_gemm[2 * c->n_gemm_ev], c->stream);
  HIPCHK(c, launch_gemm(c->cfg.dtype, a, c->stream));
  if (ev) {
    (void)hipEventRecord(c->ev_gemm[2 * c->n_gemm_ev + 1], c->stream);
    c->gemm_ev_bucket[c->n_gemm_ev] = c->gemm_bucket;
    c->n_gemm_ev++;
  }
  return SPEC_OK;
}

// One decoder layer over m rows.  In: c->h (fp32 residual stream) and c->x (rows normed by the
// layer's attn_norm).  Out: c->h updated; x_out = rmsnorm(h) * next_norm (or h itself, cast).
int layer_forward(spec_ctx *c, const spec_layer_weights &lw, char *kcache, char *vcache, int m, int base,
                  const RowTables &rt, int max_pos, const void *next_norm, void *x_out, const int *base_ptr = nullptr) {
  const spec_config &g = c->cfg;
  const int d = g.d_model, dq = g.n_q_heads * g.head_dim, dkv = g.n_kv_heads * g.head_dim, f = g.d_ffn;
  const int dt = g.dtype;
  {
    const Seg segs[3] = {{lw.wq, dq}, {lw.wk, dkv}, {lw.wv, dkv}};
    const GemmPlan p = plan_gemm(dq + 2 * dkv, d, dt);
    int rc = run_gemm(c, c->x, d, m, d, segs, 3, c->part, dq + 2 * dkv, c->m_max, p);
    if (rc) return rc;
    HIPCHK(c, launch_reduce_rope_kv(dt, c->part, p.n_split, c->m_max, dq + 2 * dkv, m, g.n_q_heads, g.n_kv_heads, g.head_dim,
                                    c->rope, rt.slot, c->qbuf, kcache, vcache, c->stream));
  }
  {
    AttnArgs a{};
    a.q = c->qbuf; a.kcache = kcache; a.vcache = vcache;
    a.rows = m; a.hq = g.n_q_heads; a.hkv = g.n_kv_heads; a.hd = g.head_dim; a.base = base; a.base_ptr = base_ptr;
    a.depth = rt.depth; a.anc = rt.anc;
    a.scale = 1.0f / sqrtf((float)g.head_dim);
    a.part = c->attn_part; a.max_parts = c->max_parts; a.out = c->attn_out;
    HIPCHK(c, launch_attention(dt, a, max_pos, c->stream));
  }
  {
    const Seg segs[1] = {{lw.wo, d}};
    const GemmPlan p = plan_gemm(d, dq, dt);
    int rc = run_gemm(c, c->attn_out, dq, m, dq, segs, 1, c->part, d, c->m_max, p);
    if (rc) return rc;
    HIPCHK(c, launch_reduce_add_norm(dt, c->part, p.n_split, c->m_max, d, m, d, 1, lw.ffn_norm, g.rms_eps, c->h, c->x, c->stream));
  }
  {
    // gate and up projections, one packed matrix.  Without a K split a wavefront owns both sums of a column and
    // applies SwiGLU itself (no partial sums, no extra pass); with a K split the row kernel does it.
    const int gu = gate_up_rows(f);
    const GemmPlan p = plan_gemm(gu, d, dt);
    if (p.n_split == 1) {
      const Seg segs[1] = {{lw.w_gate_up, f}};
      int rc = run_gemm(c, c->x, d, m, d, segs, 1, c->part, gu, c->m_max, p, c->act);
      if (rc) return rc;
    } else {
      const Seg segs[1] = {{lw.w_gate_up, gu}};
      int rc = run_gemm(c, c->x, d, m, d, segs, 1, c->part, gu, c->m_max, p);
      if (rc) return rc;
      HIPCHK(c, launch_reduce_swiglu(dt, c->part, p.n_split, c->m_max, gu, m, f, c->act, c->stream));
    }
  }
  {
    const Seg segs[1] = {{lw.w_down, d}};
    const GemmPlan p = plan_gemm(d, f, dt);
    int rc = run_gemm(c, c->act, f, m, f, segs, 1, c->part, d, c->m_max, p);
    if (rc) return rc;
    HIPCHK(c, launch_reduce_add_norm(dt, c->part, p.n_split, c->m_max, d, m, d, 1, next_norm, g.rms_eps, c->h, x_out, c->stream));
  }
  return SPEC_OK;
}

// LM head over `rows` feature rows starting at `x` -> logits [rows, vocab] fp32.
int lm_head(spec_ctx *c, const void *x, int rows, float *logits) {
  const spec_config &g = c->cfg;
  const Seg segs[1] = {{c->w.lm_head, g.vocab}};
  GemmPlan p;                                    // the vocabulary alone gives enough workgroups: no K split
  p.n_split = 1;
  return run_gemm(c, x, g.d_model, rows, g.d_model, segs, 1, logits, g.vocab, rows, p);
}

// Target model over m rows -> c->feats [m, d] (final-norm output) and the updated target cache.
// With base_ptr set, the base comes from device memory and max_pos is only an upper bound for grid
// sizes: the launch sequence is then independent of the cycle and can be captured into a graph.
int target_forward(spec_ctx *c, int m, int base, const RowTables &rt, int max_pos, const int *base_ptr = nullptr) {
  const spec_config &g = c->cfg;
  // (the launch that opens the forward also fills the rotary table of its rows)
  HIPCHK(c, launch_embed_norm(g.dtype, c->w.embed, rt.token, m, g.d_model, c->layers[0].attn_norm, g.rms_eps, c->h, c->x, c->stream,
                              rt.pos, g.head_dim, g.rope_theta, c->rope));
  for (int l = 0; l < g.n_layers; l++) {
    char *kc = c->kv_t + (size_t)l * c->t_layer_stride * c->esz;
    char *vc = kc + c->t_kv_stride * c->esz;
    const bool last = l + 1 == g.n_layers;
    int rc = layer_forward(c, c->layers[l], kc, vc, m, base, rt, max_pos, last ? c->w.final_norm : c->layers[l + 1].attn_norm,
                           last ? c->feats : c->x, base_ptr);
    if (rc) return rc;
  }
  return SPEC_OK;
}

// Draft model over m rows of (feature, token) -> c->gfeat [m, d] (predicted features, no norm).
int draft_forward(spec_ctx *c, int m, int base, const void *feat, const int *src_row, const RowTables &rt, int max_pos,
                  const int *base_ptr = nullptr) {
  const spec_config &g = c->cfg;
  const int d = g.d_model;
  HIPCHK(c, launch_concat_feat_embed(g.dtype, feat, src_row, c->w.embed, rt.token, m, d, c->xcat, c->stream, rt.pos, g.head_dim,
                                     g.rope_theta, c->rope));
  const Seg segs[1] = {{c->w.draft_fc, d}};
  const GemmPlan p = plan_gemm(d, 2 * d, g.dtype);
  int rc = run_gemm(c, c->xcat, 2 * d, m, 2 * d, segs, 1, c->part, d, c->m_max, p);
  if (rc) return rc;
  HIPCHK(c, launch_reduce_add_norm(g.dtype, c->part, p.n_split, c->m_max, d, m, d, 0, c->w.draft_layer.attn_norm, g.rms_eps, c->h,
                                   c->x, c->stream));
  char *kc = c->kv_d;
  char *vc = kc + c->d_kv_stride * c->esz;
  return layer_forward(c, c->w.draft_layer, kc, vc, m, base, rt, max_pos, nullptr, c->gfeat, base_ptr);
}

int sync(spec_ctx *c) {
  HIPCHK(c, hipStreamSynchronize(c->stream));
  harvest_profile(c);
  return SPEC_OK;
}

// End of a drafting call: the device tree goes to the host arrays of the caller.
int finish_draft(spec_ctx *c, spec_tree *out) {
  c->gemm_bucket = 0;
  HIPCHK(c, hipMemcpyAsync(&c->stage->tree_n, c->t_n, offsetof(HostStage, pos), hipMemcpyDeviceToHost, c->stream));
  phase_end(c, 0);
  int rc = sync(c);
  if (rc) return rc;
  const HostStage &s = *c->stage;
  out->n_nodes = s.tree_n;
  for (int j = 0; j < s.tree_n; j++) {
    out->token[j] = s.tok[j]; out->parent[j] = s.par[j]; out->depth[j] = s.dep[j];
    if (out->score) out->score[j] = s.sc[j];
  }
  c->state = DRAFTED;
  return SPEC_OK;
}

// Proposals of the rows just run through the LM head (c->dlogits, `rows` rows, the nodes of depth `depth`):
// the `width` best tokens per row, or `width` tokens drawn without replacement when children are sampled
// (the rows' logits are then kept for the acceptance).
int static_proposals(spec_ctx *c, int rows, int depth, int width, int first_qrow) {
  const spec_config &g = c->cfg;
  const float *src = c->dlogits;
  if (c->st.sampled) {
    HIPCHK(c, hipMemcpyAsync(c->st_qrows + (size_t)first_qrow * g.vocab, c->dlogits, (size_t)rows * g.vocab * 4, hipMemcpyDeviceToDevice,
                             c->stream));
    HIPCHK(c, launch_perturb_rows(c->dlogits, rows, g.vocab, g.temperature, g.seed, c->cycle, c->st_enode + depth * kMaxTopK, c->logits,
                                  c->stream));
    src = c->logits;                                          // free until the verify forward writes it
  }
  HIPCHK(c, launch_rows_topk_logprob(src, rows, g.vocab, width, c->sc_val, c->sc_idx, c->sc_stat, c->top_tok, c->top_lp, c->stream));
  return SPEC_OK;
}

// Drafting of a static tree shape; the root step's draft forward has run (m1 pending rows, c->dlogits row 0 =
// the draft's logits at the root).  One draft forward per depth over the nodes that have children.
int draft_static(spec_ctx *c, int m1) {
  const spec_ctx::StaticHost &st = c->st;
  const int with_scores = st.sampled ? 0 : 1;
  int qrow = 0;
  if (st.rows[0] > 0) {
    int rc = static_proposals(c, 1, 0, st.width[0], qrow);
    if (rc) return rc;
    qrow += 1;
  }
  HIPCHK(c, launch_static_step(c->st_tb, 1, c->top_tok, c->top_lp, m1 - 1, c->root_tok, c->t_base, with_scores, c->ds, c->t_n, c->t_tok,
                               c->t_par, c->t_dep, c->t_sc, c->stream));
  for (int d = 1; d < st.max_depth; d++) {
    const int rows = st.rows[d];
    if (rows == 0) break;                                     // no node of this depth has children: nothing deeper exists
    RowTables fr{c->ds.front_tok, c->ds.front_pos, c->ds.front_slot, c->ds.front_depth, c->ds.front_anc};
    int rc = draft_forward(c, rows, c->n, c->gfeat, c->ds.front_src, fr, c->n + d - 1);
    if (rc) return rc;
    rc = lm_head(c, c->gfeat, rows, c->dlogits);
    if (rc) return rc;
    rc = static_proposals(c, rows, d, st.width[d], qrow);
    if (rc) return rc;
    qrow += rows;
    HIPCHK(c, launch_static_step(c->st_tb, d + 1, c->top_tok, c->top_lp, m1 - 1, c->root_tok, c->t_base, with_scores, c->ds, c->t_n,
                                 c->t_tok, c->t_par, c->t_dep, c->t_sc, c->stream));
  }
  return SPEC_OK;
}

}  // namespace

// =============================================================================================
extern "C" {

uint64_t spec_packed_bytes(int32_t dtype, int32_t rows, int32_t in) {
  if ((dtype != 0 && dtype != 1) || rows < 1 || in < 1 || in % (dtype == 1 ? 8 : 4)) return 0;
  return packed_weight_bytes(dtype, rows, in);
}

int spec_pack_weight(int32_t dtype, const void *src, int32_t rows, int32_t in, void *dst, void *stream) {
  if (!src || !dst || spec_packed_bytes(dtype, rows, in) == 0 || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return SPEC_EINVAL;
  return launch_pack_weight(dtype, src, rows, in, dst, (hipStream_t)stream) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

uint64_t spec_packed_gate_up_bytes(int32_t dtype, int32_t rows, int32_t in) {
  if ((dtype != 0 && dtype != 1) || rows < 1 || in < 1 || in % (dtype == 1 ? 8 : 4)) return 0;
  return packed_gate_up_bytes(dtype, rows, in);
}

int spec_pack_gate_up(int32_t dtype, const void *gate, const void *up, int32_t rows, int32_t in, void *dst, void *stream) {
  if (!gate || !up || !dst || spec_packed_gate_up_bytes(dtype, rows, in) == 0 || ((uintptr_t)dst & 15) || ((uintptr_t)gate & 15) ||
      ((uintptr_t)up & 15))
    return SPEC_EINVAL;
  return launch_pack_gate_up(dtype, gate, up, rows, in, dst, (hipStream_t)stream) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

uint64_t spec_workspace_bytes(const spec_config *cfg) {
  if (!config_ok(cfg, nullptr)) return 0;
  return layout(*cfg, nullptr, nullptr);
}

int spec_create(const spec_config *cfg, const spec_weights *w, spec_ctx **out) {
  std::string why;
  if (!out) return fail(nullptr, SPEC_EINVAL, "out is NULL");
  *out = nullptr;
  if (!config_ok(cfg, &why)) return fail(nullptr, SPEC_EINVAL, "bad configuration: %s", why.c_str());
  if (!w || !w->embed || !w->lm_head || !w->final_norm || !w->layers || !w->draft_fc) return fail(nullptr, SPEC_EINVAL, "NULL weight pointer");
  auto layer_ok = [](const spec_layer_weights &l) {
    return l.attn_norm && l.wq && l.wk && l.wv && l.wo && l.ffn_norm && l.w_gate_up && l.w_down;
  };
  for (int l = 0; l < cfg->n_layers; l++)
    if (!layer_ok(w->layers[l])) return fail(nullptr, SPEC_EINVAL, "NULL weight pointer in layer %d", l);
  if (!layer_ok(w->draft_layer)) return fail(nullptr, SPEC_EINVAL, "NULL weight pointer in the draft layer");
  const size_t need = layout(*cfg, nullptr, nullptr);
  if (!cfg->workspace || ((uintptr_t)cfg->workspace & 255)) return fail(nullptr, SPEC_EINVAL, "workspace is NULL or not 256-byte aligned");
  if (cfg->workspace_bytes < need) return fail(nullptr, SPEC_ECAP, "workspace too small: %llu < %llu bytes",
                                               (unsigned long long)cfg->workspace_bytes, (unsigned long long)need);
  spec_ctx *c = new (std::nothrow) spec_ctx();
  if (!c) return fail(nullptr, SPEC_EINVAL, "out of host memory");
  c->cfg = *cfg;
  c->w = *w;
  c->layers.assign(w->layers, w->layers + cfg->n_layers);
  c->w.layers = c->layers.data();
  c->stream = (hipStream_t)cfg->stream;
  layout(*cfg, c, (char *)cfg->workspace);
  hipError_t e = hipSetDevice(cfg->device);
  if (e == hipSuccess) e = gemm_init();
  if (e == hipSuccess) e = hipHostMalloc((void **)&c->stage, sizeof(HostStage), hipHostMallocDefault);
  if (e != hipSuccess) {
    int rc = fail(nullptr, SPEC_EHIP, "device %d / pinned staging: %s", cfg->device, hipGetErrorString(e));
    delete c;
    return rc;
  }
  for (int p = 0; p < 4; p++)
    for (int k = 0; k < 2; k++) (void)hipEventCreate(&c->ev_phase[p][k]);
  *out = c;
  return SPEC_OK;
}

void spec_destroy(spec_ctx *c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  for (int p = 0; p < 4; p++)
    for (int k = 0; k < 2; k++) if (c->ev_phase[p][k]) (void)hipEventDestroy(c->ev_phase[p][k]);
  for (hipEvent_t e : c->ev_gemm) (void)hipEventDestroy(e);
  if (c->verify_exec) (void)hipGraphExecDestroy(c->verify_exec);
  if (c->expand_exec) (void)hipGraphExecDestroy(c->expand_exec);
  if (c->stage) (void)hipHostFree(c->stage);
  delete c;
}

const char *spec_last_error(const spec_ctx *c) { return c ? c->err.c_str() : g_create_error.c_str(); }

int spec_committed(const spec_ctx *c) { return c ? c->n : SPEC_EINVAL; }

int spec_prefill(spec_ctx *c, const int32_t *prompt, int32_t n_prompt, int32_t *first_token) {
  if (!c) return SPEC_EINVAL;
  if (!prompt || !first_token || n_prompt < 1) return fail(c, SPEC_EINVAL, "prefill: NULL argument or empty prompt");
  if (c->state != CREATED) return fail(c, SPEC_ESTATE, "prefill: context already prefilled");
  const spec_config &g = c->cfg;
  if (n_prompt + g.tree_total > g.max_seq) return fail(c, SPEC_ECAP, "prefill: prompt %d + tree %d exceeds max_seq %d", n_prompt, g.tree_total, g.max_seq);
  for (int i = 0; i < n_prompt; i++)
    if (prompt[i] < 0 || prompt[i] >= g.vocab) return fail(c, SPEC_EINVAL, "prefill: token %d at %d out of range", prompt[i], i);
  HIPCHK(c, hipSetDevice(g.device));
  phase_begin(c, 3);
  HIPCHK(c, hipMemcpyAsync(c->d_prompt, prompt, (size_t)n_prompt * 4, hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));       // the caller's prompt buffer is pageable: finish the copy now
  const bool draft = g.tree_total > 1;
  for (int c0 = 0; c0 < n_prompt; c0 += kPrefillChunk) {
    const int m = std::min(kPrefillChunk, n_prompt - c0);
    HIPCHK(c, launch_chain_rows(c0, m, 0, c->d_pos, c->d_slot, c->d_depth, c->stream));
    RowTables rt{c->d_prompt + c0, c->d_pos, c->d_slot, c->d_depth, nullptr};
    int rc = target_forward(c, m, c0, rt, c0 + m - 1);
    if (rc) return rc;
    const bool last = c0 + m == n_prompt;
    if (last) {
      rc = lm_head(c, (const char *)c->feats + (size_t)(m - 1) * g.d_model * c->esz, 1, c->logits);
      if (rc) return rc;
      if (g.temperature > 0.f)
        HIPCHK(c, launch_sample_row(c->logits, g.vocab, g.temperature, g.seed, 0, 0, c->root_tok, c->stream));
      else
        HIPCHK(c, launch_rows_argmax(c->logits, 1, g.vocab, c->amax_val, c->amax_idx, c->root_tok, c->stream));
      // pending pair for the first draft root step: (feature of the last prompt position, first token)
      HIPCHK(c, hipMemcpyAsync(c->pend_feat, (const char *)c->feats + (size_t)(m - 1) * g.d_model * c->esz,
                               (size_t)g.d_model * c->esz, hipMemcpyDeviceToDevice, c->stream));
      HIPCHK(c, hipMemcpyAsync(c->pend_tok, c->root_tok, 4, hipMemcpyDeviceToDevice, c->stream));
    }
    // draft over the pairs (feature of position i-1, token at position i), i = c0+1 .. c0+m (the last
    // chunk stops one short: its final pair needs the first generated token and stays pending)
    const int md = last ? m - 1 : m;
    if (draft && md > 0) {
      HIPCHK(c, launch_chain_rows(c0, md, 1, c->d_pos, c->d_slot, c->d_depth, c->stream));
      RowTables dr{c->d_prompt + c0 + 1, c->d_pos, c->d_slot, c->d_depth, nullptr};
      rc = draft_forward(c, md, c0, c->feats, nullptr, dr, c0 + md - 1);
      if (rc) return rc;
    }
  }
  c->stage->base = n_prompt;
  HIPCHK(c, hipMemcpyAsync(c->t_base, &c->stage->base, 4, hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipMemcpyAsync(&c->stage->first_token, c->root_tok, 4, hipMemcpyDeviceToHost, c->stream));
  phase_end(c, 3);
  int rc = sync(c);
  if (rc) return rc;
  c->root = c->stage->first_token;
  *first_token = c->root;
  c->n = n_prompt;
  c->n_pend = 1;
  c->cycle = 0;
  c->state = READY;
  return SPEC_OK;
}

int spec_draft_tree(spec_ctx *c, spec_tree *out) {
  if (!c) return SPEC_EINVAL;
  if (!out || !out->token || !out->parent || !out->depth) return fail(c, SPEC_EINVAL, "draft_tree: NULL argument");
  if (c->state != READY) return fail(c, SPEC_ESTATE, "draft_tree: needs a prefilled context with no tree pending");
  const spec_config &g = c->cfg;
  if (c->n + g.tree_total > g.max_seq) return fail(c, SPEC_ECAP, "draft_tree: committed %d + tree %d exceeds max_seq %d", c->n, g.tree_total, g.max_seq);
  c->cycle++;
  if (g.tree_total == 1) {                          // plain decoding: the tree is the root alone
    out->n_nodes = 1; out->token[0] = c->root; out->parent[0] = -1; out->depth[0] = 0;
    if (out->score) out->score[0] = 0.f;
    c->state = DRAFTED;
    return SPEC_OK;
  }
  HIPCHK(c, hipSetDevice(g.device));
  phase_begin(c, 0);
  c->gemm_bucket = 5;
  const int K = g.tree_topk, D = g.tree_depth, d = g.d_model;
  // root step: the pending pairs occupy draft slots n - n_pend .. n - 1 (rotary positions one higher)
  const int m1 = c->n_pend, base = c->n - m1;
  HIPCHK(c, launch_chain_rows(base, m1, 1, c->d_pos, c->d_slot, c->d_depth, c->stream));
  RowTables rt{c->pend_tok, c->d_pos, c->d_slot, c->d_depth, nullptr};
  int rc = draft_forward(c, m1, base, c->pend_feat, nullptr, rt, base + m1 - 1);
  if (rc) return rc;
  rc = lm_head(c, (const char *)c->gfeat + (size_t)(m1 - 1) * d * c->esz, 1, c->dlogits);
  if (rc) return rc;
  if (c->st.n_nodes > 0) {
    rc = draft_static(c, m1);
    if (rc) return rc;
    return finish_draft(c, out);
  }
  HIPCHK(c, launch_rows_topk_logprob(c->dlogits, 1, g.vocab, K, c->sc_val, c->sc_idx, c->sc_stat, c->top_tok, c->top_lp, c->stream));
  HIPCHK(c, launch_pool_init(c->ds, c->top_tok, c->top_lp, K, m1 - 1, c->t_base, c->stream));
  // expansion steps 2..D (the frontier's k nodes, each fed (parent's predicted feature, own token)) and
  // the rerank.  Every argument is fixed or device-resident (frontier tables, committed count), so the
  // whole sequence is captured once and replayed.
  auto expand_all = [&](const int *base_ptr, int base, int pos_bound) -> int {
    for (int t = 2; t <= D; t++) {
      RowTables fr{c->ds.front_tok, c->ds.front_pos, c->ds.front_slot, c->ds.front_depth, c->ds.front_anc};
      // xcat is built from gfeat before the layer overwrites gfeat, so one buffer serves all steps
      int r = draft_forward(c, K, base, c->gfeat, c->ds.front_src, fr, base_ptr ? pos_bound : base + t - 2, base_ptr);
      if (r) return r;
      r = lm_head(c, c->gfeat, K, c->dlogits);
      if (r) return r;
      HIPCHK(c, launch_rows_topk_logprob(c->dlogits, K, g.vocab, K, c->sc_val, c->sc_idx, c->sc_stat, c->top_tok, c->top_lp, c->stream));
      HIPCHK(c, launch_pool_expand(c->ds, c->top_tok, c->top_lp, K, t, c->t_base, t < D ? 1 : 0, c->stream));
    }
    HIPCHK(c, launch_rerank(c->ds, g.tree_total, c->root_tok, c->t_n, c->t_tok, c->t_par, c->t_dep, c->t_sc, c->stream));
    return SPEC_OK;
  };
  if (c->graphs && c->stream != nullptr && c->prof_level < 2) {
    const int need = c->n + D;                                  // largest key position of a draft row of this cycle
    if (c->expand_exec == nullptr || need > c->expand_exec_bound) {
      if (c->expand_exec) { (void)hipGraphExecDestroy(c->expand_exec); c->expand_exec = nullptr; }
      const int bound = std::min(c->seq_draft - 1, (need / kGraphBucket + 1) * kGraphBucket - 1);
      hipGraph_t graph = nullptr;
      HIPCHK(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
      rc = expand_all(c->t_base, 0, bound);
      hipError_t e = hipStreamEndCapture(c->stream, &graph);
      if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
      if (e != hipSuccess) return fail(c, SPEC_EHIP, "graph capture (draft): %s", hipGetErrorString(e));
      e = hipGraphInstantiate(&c->expand_exec, graph, nullptr, nullptr, 0);
      (void)hipGraphDestroy(graph);
      if (e != hipSuccess) { c->expand_exec = nullptr; return fail(c, SPEC_EHIP, "graph instantiate (draft): %s", hipGetErrorString(e)); }
      c->expand_exec_bound = bound;
    }
    HIPCHK(c, hipGraphLaunch(c->expand_exec, c->stream));
  } else {
    rc = expand_all(nullptr, c->n, 0);
    if (rc) return rc;
  }
  return finish_draft(c, out);
}

int spec_verify(spec_ctx *c, const spec_tree *tree) {
  if (!c) return SPEC_EINVAL;
  if (!tree || !tree->token || !tree->parent || !tree->depth) return fail(c, SPEC_EINVAL, "verify: NULL argument");
  if (c->state != DRAFTED) return fail(c, SPEC_ESTATE, "verify: call spec_draft_tree first");
  const spec_config &g = c->cfg;
  const int N = tree->n_nodes;
  if (N < 1 || N > g.tree_total) return fail(c, SPEC_EINVAL, "verify: n_nodes %d outside 1..%d", N, g.tree_total);
  if (c->n + N > g.max_seq) return fail(c, SPEC_ECAP, "verify: committed %d + nodes %d exceeds max_seq %d", c->n, N, g.max_seq);
  if (tree->token[0] != c->root || tree->parent[0] != -1 || tree->depth[0] != 0)
    return fail(c, SPEC_EINVAL, "verify: node 0 must be the pending root token %d with parent -1 and depth 0", c->root);
  HostStage &s = *c->stage;
  int max_depth = 0;
  for (int j = 0; j < N; j++) {
    const int tok = tree->token[j], par = tree->parent[j], dep = tree->depth[j];
    if (tok < 0 || tok >= g.vocab) return fail(c, SPEC_EINVAL, "verify: node %d token %d out of range", j, tok);
    if (j > 0) {
      if (par < 0 || par >= j) return fail(c, SPEC_EINVAL, "verify: node %d parent %d must precede it", j, par);
      if (dep != tree->depth[par] + 1) return fail(c, SPEC_EINVAL, "verify: node %d depth %d inconsistent with its parent", j, dep);
      if (dep > SPEC_MAX_DEPTH) return fail(c, SPEC_EINVAL, "verify: node %d deeper than %d", j, SPEC_MAX_DEPTH);
    }
    s.tok[j] = tok; s.par[j] = par; s.dep[j] = dep; s.sc[j] = tree->score ? tree->score[j] : 0.f;
    s.pos[j] = c->n + dep; s.slot[j] = c->n + j;
    for (int a = j, q = dep; a >= 0; a = tree->parent[a], q--) s.anc[j * kAncStride + q] = a;   // path, root first
    max_depth = std::max(max_depth, dep);
  }
  s.tree_n = N;
  s.base = c->n;
  HIPCHK(c, hipSetDevice(g.device));
  phase_begin(c, 1);
  c->gemm_bucket = 4;
  HIPCHK(c, hipMemcpyAsync(c->t_n, &s.tree_n, offsetof(HostStage, acc), hipMemcpyHostToDevice, c->stream));
  RowTables rt{c->t_tok, c->t_pos, c->t_slot, c->t_dep, c->t_anc};
  int rc;
  const bool use_graph = c->graphs && c->stream != nullptr && c->prof_level < 2 && N == g.tree_total;
  if (use_graph) {
    // Every launch argument of the forward is either fixed or read from device memory (the tree
    // tables and the base), so the sequence is captured once and replayed each cycle.
    const int need = c->n + kMaxDepth;                          // largest key position a row of this cycle can have
    if (c->verify_exec == nullptr || c->verify_exec_rows != N || need > c->verify_exec_bound) {
      if (c->verify_exec) { (void)hipGraphExecDestroy(c->verify_exec); c->verify_exec = nullptr; }
      const int bound = std::min(g.max_seq - 1, (need / kGraphBucket + 1) * kGraphBucket - 1);
      hipGraph_t graph = nullptr;
      HIPCHK(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
      rc = target_forward(c, N, 0, rt, bound, c->t_base);
      if (!rc) rc = lm_head(c, c->feats, N, c->logits);
      hipError_t e = hipStreamEndCapture(c->stream, &graph);
      if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
      if (e != hipSuccess) return fail(c, SPEC_EHIP, "graph capture: %s", hipGetErrorString(e));
      e = hipGraphInstantiate(&c->verify_exec, graph, nullptr, nullptr, 0);
      (void)hipGraphDestroy(graph);
      if (e != hipSuccess) { c->verify_exec = nullptr; return fail(c, SPEC_EHIP, "graph instantiate: %s", hipGetErrorString(e)); }
      c->verify_exec_rows = N;
      c->verify_exec_bound = bound;
    }
    HIPCHK(c, hipGraphLaunch(c->verify_exec, c->stream));
  } else {
    rc = target_forward(c, N, c->n, rt, c->n + max_depth);
    if (rc) return rc;
    rc = lm_head(c, c->feats, N, c->logits);
    if (rc) return rc;
    if (c->prof_level >= 2 && c->n_gemm_ev < kMaxGemmEvents) {
      // calibration: an event pair with nothing between its records, taken in the flow of the forward (the
      // stream still has queued work, so the interval is the event mechanism's own cost, not host pacing)
      (void)hipEventRecord(c->ev_gemm[2 * c->n_gemm_ev], c->stream);
      (void)hipEventRecord(c->ev_gemm[2 * c->n_gemm_ev + 1], c->stream);
      c->gemm_ev_bucket[c->n_gemm_ev++] = 6;
    }
  }
  c->gemm_bucket = 0;
  phase_end(c, 1);
  c->last_nodes = N;
  c->state = VERIFIED;
  return SPEC_OK;
}

int spec_accept(spec_ctx *c, const spec_tree *tree, int32_t *out_tokens, int32_t *n_out) {
  if (!c) return SPEC_EINVAL;
  if (!tree || !out_tokens || !n_out) return fail(c, SPEC_EINVAL, "accept: NULL argument");
  if (c->state != VERIFIED) return fail(c, SPEC_ESTATE, "accept: call spec_verify first");
  if (tree->n_nodes != c->last_nodes) return fail(c, SPEC_EINVAL, "accept: not the tree that was verified");
  const spec_config &g = c->cfg;
  const int N = c->last_nodes;
  HIPCHK(c, hipSetDevice(g.device));
  phase_begin(c, 2);
  if (g.temperature > 0.f && c->st.n_nodes > 0 && c->st.sampled) {
    // sampled children: the ratio rule against the draft rows kept while drafting (c->part serves as its scratch)
    HIPCHK(c, launch_accept_qratio(c->logits, c->st_qrows, c->st_qrow_of, g.vocab, g.temperature, c->t_tok, c->t_par, N, g.seed, c->cycle,
                                   c->part, c->acc, c->stream));
  } else if (g.temperature > 0.f) {
    HIPCHK(c, launch_rows_softmax_stats(c->logits, N, g.vocab, g.temperature, c->stats, c->stream));
    HIPCHK(c, launch_accept_sample(c->logits, g.vocab, c->stats, g.temperature, c->t_tok, c->t_par, N, g.seed, c->cycle, c->acc, c->stream));
  } else {
    HIPCHK(c, launch_rows_argmax(c->logits, N, g.vocab, c->amax_val, c->amax_idx, nullptr, c->stream));
    HIPCHK(c, launch_accept_greedy(c->amax_val, c->amax_idx, argmax_slices(g.vocab), c->t_tok, c->t_par, N, c->acc, c->stream));
  }
  HIPCHK(c, launch_commit(g.dtype, c->acc, c->kv_t, c->t_layer_stride, c->t_kv_stride, g.n_layers, g.n_kv_heads * g.head_dim,
                          c->n, c->feats, g.d_model, c->pend_feat, c->pend_tok, c->root_tok, c->t_base, c->stream));
  HIPCHK(c, hipMemcpyAsync(&c->stage->acc, c->acc, sizeof(AcceptResult), hipMemcpyDeviceToHost, c->stream));
  phase_end(c, 2);
  int rc = sync(c);
  if (rc) return rc;
  const AcceptResult &r = c->stage->acc;
  const int m = r.n_acc;
  if (m < 0 || m > kMaxDepth) return fail(c, SPEC_EHIP, "accept: device returned an invalid accepted count %d", m);
  for (int i = 0; i <= m; i++) out_tokens[i] = r.token[i];
  *n_out = m + 1;
  c->n += 1 + m;
  c->n_pend = m + 1;
  c->root = r.token[m];
  c->state = READY;
  return SPEC_OK;
}

// ---- inspection ------------------------------------------------------------------------------
int64_t spec_get_logits(spec_ctx *c, float *dst, int64_t cap) {
  if (!c || !dst) return SPEC_EINVAL;
  if (c->last_nodes < 1) return fail(c, SPEC_ESTATE, "get_logits: nothing verified yet");
  const int64_t n = (int64_t)c->last_nodes * c->cfg.vocab;
  if (cap < n) return fail(c, SPEC_ECAP, "get_logits: capacity %lld < %lld", (long long)cap, (long long)n);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(dst, c->logits, (size_t)n * 4, hipMemcpyDeviceToHost));
  return n;
}

static int64_t copy_widen(spec_ctx *c, const void *src, int64_t n, float *dst) {
  if (c->cfg.dtype == SPEC_DTYPE_FP32) {
    HIPCHK(c, hipMemcpy(dst, src, (size_t)n * 4, hipMemcpyDeviceToHost));
    return n;
  }
  std::vector<uint16_t> tmp((size_t)n);
  HIPCHK(c, hipMemcpy(tmp.data(), src, (size_t)n * 2, hipMemcpyDeviceToHost));
  for (int64_t i = 0; i < n; i++) {
    const uint32_t u = (uint32_t)tmp[(size_t)i] << 16;
    memcpy(&dst[i], &u, 4);
  }
  return n;
}

int64_t spec_get_features(spec_ctx *c, float *dst, int64_t cap) {
  if (!c || !dst) return SPEC_EINVAL;
  if (c->last_nodes < 1) return fail(c, SPEC_ESTATE, "get_features: nothing verified yet");
  const int64_t n = (int64_t)c->last_nodes * c->cfg.d_model;
  if (cap < n) return fail(c, SPEC_ECAP, "get_features: capacity %lld < %lld", (long long)cap, (long long)n);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return copy_widen(c, c->feats, n, dst);
}

int64_t spec_get_kv(spec_ctx *c, int32_t which, int32_t layer, int32_t n_rows, float *k_dst, float *v_dst, int64_t cap) {
  if (!c || !k_dst || !v_dst) return SPEC_EINVAL;
  const spec_config &g = c->cfg;
  const int dkv = g.n_kv_heads * g.head_dim;
  const int64_t n = (int64_t)n_rows * dkv;
  if (n_rows < 1 || cap < n) return fail(c, SPEC_ECAP, "get_kv: bad row count or capacity");
  const char *k, *v;
  if (which == 0) {
    if (layer < 0 || layer >= g.n_layers || n_rows > g.max_seq) return fail(c, SPEC_EINVAL, "get_kv: layer/rows out of range");
    k = c->kv_t + (size_t)layer * c->t_layer_stride * c->esz;
    v = k + c->t_kv_stride * c->esz;
  } else if (which == 1) {
    if (n_rows > c->seq_draft) return fail(c, SPEC_EINVAL, "get_kv: rows out of range");
    k = c->kv_d;
    v = k + c->d_kv_stride * c->esz;
  } else {
    return fail(c, SPEC_EINVAL, "get_kv: which must be 0 or 1");
  }
  HIPCHK(c, hipStreamSynchronize(c->stream));
  int64_t r = copy_widen(c, k, n, k_dst);
  if (r < 0) return r;
  return copy_widen(c, v, n, v_dst);
}

namespace {
struct StaticPlan {                   // host-side analysis of a static shape
  int depth[kMaxNodes], erow[kMaxNodes], eoff[kMaxNodes], qrow_of[kMaxNodes], enode[(kMaxDepth + 1) * kMaxTopK];
  spec_ctx::StaticHost h;
};
// Validates a shape and derives its tables; returns nullptr or the reason it is not accepted.
const char *plan_static(int n, const int32_t *parent, const int32_t *rank, bool sampled, StaticPlan *p) {
  if (n < 1 || n > kMaxNodes || !parent || !rank) return "n_nodes outside 1..128 or NULL arrays";
  if (parent[0] != -1) return "node 0 must be the root (parent -1)";
  int kids[kMaxNodes] = {}, last_rank[kMaxNodes];
  for (int i = 0; i < n; i++) { last_rank[i] = -1; p->erow[i] = p->eoff[i] = p->qrow_of[i] = -1; }
  for (int i = 0; i < (kMaxDepth + 1) * kMaxTopK; i++) p->enode[i] = 0;
  p->depth[0] = 0;
  p->h = spec_ctx::StaticHost{};
  for (int i = 1; i < n; i++) {
    const int u = parent[i];
    if (u < 0 || u >= i) return "a parent must precede its children";
    p->depth[i] = p->depth[u] + 1;
    if (p->depth[i] < p->depth[i - 1]) return "nodes must be in order of depth";
    if (p->depth[i] > kMaxDepth) return "deeper than 15";
    if (rank[i] < 0 || rank[i] >= kMaxTopK) return "rank outside 0..15";
    if (rank[i] <= last_rank[u]) return "the children of a node must be listed in increasing rank";
    // The ratio rule tries a node's children as successive draws without replacement, each against the draft
    // distribution renormalised over the tokens not listed before it: that is the law of a child only if every
    // earlier draw is in the tree, so sampled children must carry ranks 0, 1, ..., c-1.
    if (sampled && rank[i] != last_rank[u] + 1) return "sampled children of a node must carry ranks 0, 1, ... without gaps";
    last_rank[u] = rank[i];
    kids[u]++;
    p->h.width[p->depth[u]] = std::max(p->h.width[p->depth[u]], rank[i] + 1);
    p->h.max_depth = std::max(p->h.max_depth, p->depth[i]);
  }
  int qrow = 0, off = 0;
  for (int i = 0; i < n; i++) {
    if (!kids[i]) continue;
    const int d = p->depth[i];
    if (p->h.rows[d] >= kMaxTopK) return "more than 16 nodes with children at one depth";
    p->erow[i] = p->h.rows[d];
    p->enode[d * kMaxTopK + p->h.rows[d]] = kDraftNodeStream + i;
    p->h.rows[d]++;
    p->qrow_of[i] = qrow++;
    if (i > 0) { p->eoff[i] = off++; p->h.n_expanded++; }
  }
  for (int d = 1; d < p->h.max_depth; d++)
    if (p->h.rows[d] == 0) return "a depth without expanded nodes below a deeper node";   // cannot happen for a tree; defensive
  p->h.n_nodes = n;
  return nullptr;
}
size_t static_table_ints() { return (size_t)6 * kMaxNodes + (kMaxDepth + 1) * kMaxTopK; }
}  // namespace

uint64_t spec_static_tree_bytes(const spec_config *cfg, int32_t n_nodes, const int32_t *parent, const int32_t *rank, int32_t sampled) {
  StaticPlan p;
  if (!cfg || plan_static(n_nodes, parent, rank, sampled != 0, &p) != nullptr) return 0;
  size_t bytes = align_up(static_table_ints() * 4);
  if (sampled) bytes += align_up((size_t)(p.h.n_expanded + (p.h.rows[0] ? 1 : 0)) * cfg->vocab * 4);
  return bytes;
}

int spec_set_static_tree(spec_ctx *c, int32_t n_nodes, const int32_t *parent, const int32_t *rank, int32_t sampled, void *buffer,
                         uint64_t buffer_bytes) {
  if (!c) return SPEC_EINVAL;
  if (c->state != CREATED && c->state != READY) return fail(c, SPEC_ESTATE, "set_static_tree: a drafted tree is pending");
  if (n_nodes == 0) { c->st = spec_ctx::StaticHost{}; return SPEC_OK; }          // back to the dynamic tree
  const spec_config &g = c->cfg;
  StaticPlan p;
  const char *why = plan_static(n_nodes, parent, rank, sampled != 0, &p);
  if (why) return fail(c, SPEC_EINVAL, "set_static_tree: %s", why);
  if (n_nodes > g.tree_total) return fail(c, SPEC_ECAP, "set_static_tree: %d nodes exceed the configured tree_total %d", n_nodes, g.tree_total);
  if (p.h.n_expanded > g.tree_depth * g.tree_topk)
    return fail(c, SPEC_ECAP, "set_static_tree: %d expanded nodes exceed the draft scratch of tree_depth * tree_topk = %d", p.h.n_expanded,
                g.tree_depth * g.tree_topk);
  if (sampled && !(g.temperature > 0.f)) return fail(c, SPEC_EINVAL, "set_static_tree: sampled children need temperature > 0");
  if (sampled && (c->part_floats < (size_t)g.vocab || n_nodes > g.tree_total))
    return fail(c, SPEC_ECAP, "set_static_tree: workspace too small for the ratio rule's scratch");
  const uint64_t need = spec_static_tree_bytes(&g, n_nodes, parent, rank, sampled);
  if (!buffer || ((uintptr_t)buffer & 255) || buffer_bytes < need)
    return fail(c, SPEC_EINVAL, "set_static_tree: buffer NULL, not 256-byte aligned or smaller than %llu bytes", (unsigned long long)need);
  HIPCHK(c, hipSetDevice(g.device));
  std::vector<int> host(static_table_ints(), 0);
  int *hp = host.data();
  int *h_parent = hp, *h_rank = hp + kMaxNodes, *h_depth = hp + 2 * kMaxNodes, *h_erow = hp + 3 * kMaxNodes, *h_eoff = hp + 4 * kMaxNodes,
      *h_qrow = hp + 5 * kMaxNodes, *h_enode = hp + 6 * kMaxNodes;
  for (int i = 0; i < n_nodes; i++) {
    h_parent[i] = parent[i]; h_rank[i] = rank[i]; h_depth[i] = p.depth[i]; h_erow[i] = p.erow[i]; h_eoff[i] = p.eoff[i]; h_qrow[i] = p.qrow_of[i];
  }
  memcpy(h_enode, p.enode, sizeof(p.enode));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(buffer, host.data(), host.size() * 4, hipMemcpyHostToDevice));
  int *dp = (int *)buffer;
  c->st_tb.n_nodes = n_nodes;
  c->st_tb.parent = dp; c->st_tb.rank = dp + kMaxNodes; c->st_tb.depth = dp + 2 * kMaxNodes;
  c->st_tb.erow = dp + 3 * kMaxNodes; c->st_tb.eoff = dp + 4 * kMaxNodes;
  c->st_qrow_of = dp + 5 * kMaxNodes; c->st_enode = dp + 6 * kMaxNodes;
  c->st_qrows = sampled ? (float *)((char *)buffer + align_up(static_table_ints() * 4)) : nullptr;
  c->st = p.h;
  c->st.sampled = sampled != 0;
  return SPEC_OK;
}

int spec_set_graphs(spec_ctx *c, int32_t enable) {
  if (!c) return SPEC_EINVAL;
  c->graphs = enable != 0;
  return SPEC_OK;
}

int spec_set_profile(spec_ctx *c, int32_t level) {
  if (!c || level < 0 || level > 2) return SPEC_EINVAL;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  harvest_profile(c);
  if (level >= 2 && c->ev_gemm.empty()) {
    c->ev_gemm.resize(2 * kMaxGemmEvents);
    c->gemm_ev_bucket.assign(kMaxGemmEvents, 0);
    for (auto &e : c->ev_gemm) HIPCHK(c, hipEventCreate(&e));
  }
  c->prof_level = level;
  return SPEC_OK;
}

int spec_get_profile(spec_ctx *c, double *ms, int64_t *counts) {
  if (!c || !ms || !counts) return SPEC_EINVAL;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  harvest_profile(c);
  for (int i = 0; i < 8; i++) { ms[i] = c->prof_ms[i]; counts[i] = c->prof_cnt[i]; c->prof_ms[i] = 0; c->prof_cnt[i] = 0; }
  return SPEC_OK;
}

}  // extern "C"

// ---- kernel-level entry points (spec_kernels.h) ------------------------------------------------
#include "../../include/spec_kernels.h"
extern "C" {

int spec_k_gemm(int32_t dtype, const void *x, int32_t ldx, int32_t m, int32_t in, const void *w0, int32_t rows0,
                const void *w1, int32_t rows1, const void *w2, int32_t rows2, float *part, int32_t ldp, int32_t m_pad,
                int32_t n_split, void *stream) {
  if (!x || !w0 || !part || rows0 < 1 || (dtype != 0 && dtype != 1)) return SPEC_EINVAL;
  const int epl = dtype == 1 ? 8 : 4;
  if (in < 1 || in % epl || ldx % epl || m < 1 || m > 4096 || m_pad < m) return SPEC_EINVAL;
  const void *ws[3] = {w0, w1, w2};
  const int rs[3] = {rows0, w1 ? rows1 : 0, (w1 && w2) ? rows2 : 0};
  GemmArgs a{};
  a.x = x; a.ldx = ldx; a.m = m; a.in = in;
  int col = 0, blocks = 0, nseg = 0;
  for (int s = 0; s < 3; s++) {
    a.seg_w[s] = rs[s] > 0 ? ws[s] : w0;
    a.seg_rows[s] = rs[s];
    a.seg_blocks[s] = (rs[s] + 31) / 32;
    a.seg_col0[s] = col;
    col += rs[s]; blocks += a.seg_blocks[s];
    if (rs[s] > 0) nseg = s + 1;
  }
  if (ldp < col) return SPEC_EINVAL;
  a.nseg = nseg; a.total_blocks = blocks; a.part = part; a.ldp = ldp; a.m_pad = m_pad; a.n_split = n_split;
  return launch_gemm(dtype, a, (hipStream_t)stream) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

int spec_k_gemm_swiglu(int32_t dtype, const void *x, int32_t ldx, int32_t m, int32_t in, const void *w_gate_up, int32_t rows, void *act,
                       void *stream) {
  if (!x || !w_gate_up || !act || ((uintptr_t)act & 3) || rows < 1 || (dtype != 0 && dtype != 1)) return SPEC_EINVAL;
  const int epl = dtype == 1 ? 8 : 4;
  if (in < 1 || in % epl || ldx % epl || m < 1 || m > 4096) return SPEC_EINVAL;
  GemmArgs a{};
  a.x = x; a.ldx = ldx; a.m = m; a.in = in;
  for (int s = 0; s < 3; s++) {
    a.seg_w[s] = w_gate_up;
    a.seg_rows[s] = s == 0 ? rows : 0;
    a.seg_blocks[s] = s == 0 ? (rows + 15) / 16 : 0;
    a.seg_col0[s] = 0;
  }
  a.nseg = 1; a.total_blocks = a.seg_blocks[0];
  a.part = nullptr; a.ldp = gate_up_rows(rows); a.m_pad = m; a.n_split = 1;
  a.act = act;
  return launch_gemm(dtype, a, (hipStream_t)stream) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

int spec_k_attention(int32_t dtype, const void *q, const void *kcache, const void *vcache, int32_t rows, int32_t hq,
                     int32_t hkv, int32_t hd, int32_t base, const int32_t *depth, const int32_t *anc, int32_t max_depth,
                     float *scratch, int32_t max_parts, void *out, void *stream) {
  if (!q || !kcache || !vcache || !depth || !scratch || !out || rows < 1 || base < 0 || max_depth < 0) return SPEC_EINVAL;
  if (anc && max_depth > kMaxDepth) return SPEC_EINVAL;
  AttnArgs a{};
  a.q = q; a.kcache = kcache; a.vcache = vcache; a.rows = rows; a.hq = hq; a.hkv = hkv; a.hd = hd; a.base = base;
  a.depth = depth; a.anc = anc; a.scale = 1.0f / sqrtf((float)hd); a.part = scratch; a.max_parts = max_parts; a.out = out;
  return launch_attention(dtype, a, base + max_depth, (hipStream_t)stream) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

int spec_k_topk_logprob(const float *logits, int32_t rows, int32_t vocab, int32_t k, float *scratch_f, int32_t *scratch_i,
                        int32_t *top_tok, float *top_lp, void *stream) {
  if (!logits || !scratch_f || !scratch_i || !top_tok || !top_lp || rows < 1 || rows > kMaxTopK) return SPEC_EINVAL;
  const int n_slices = (vocab + kTopkSlice - 1) / kTopkSlice;
  float *sc_val = scratch_f;
  float2 *sc_stat = (float2 *)(scratch_f + (size_t)kMaxTopK * n_slices * kMaxTopK);
  return launch_rows_topk_logprob(logits, rows, vocab, k, sc_val, scratch_i, sc_stat, top_tok, top_lp, (hipStream_t)stream) == hipSuccess
             ? SPEC_OK : SPEC_EHIP;
}

int spec_k_accept_qratio(const float *p_logits, const float *q_logits, int32_t n_nodes, int32_t vocab, float temperature,
                         const int32_t *tree_tok, const int32_t *tree_par, uint64_t seed, uint32_t cycle, float *work,
                         int32_t *result, void *stream) {
  static_assert(sizeof(AcceptResult) == 33 * sizeof(int32_t), "result layout documented in spec_kernels.h");
  if (!p_logits || !q_logits || !tree_tok || !tree_par || !work || !result || n_nodes < 1 || n_nodes > kMaxNodes || vocab < 1 ||
      !(temperature > 0.f))
    return SPEC_EINVAL;
  return launch_accept_qratio(p_logits, q_logits, nullptr, vocab, temperature, tree_tok, tree_par, n_nodes, seed, cycle, work,
                              (AcceptResult *)result, (hipStream_t)stream) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

int spec_k_sample_children(const float *logits, int32_t vocab, float temperature, int32_t m, uint64_t seed, uint32_t cycle,
                           uint32_t node_stream, float *scratch_f, int32_t *scratch_i, int32_t *out, void *stream) {
  if (!logits || !out || !scratch_f || !scratch_i || vocab < 1 || m < 1 || m > kMaxTopK || m > vocab || !(temperature > 0.f))
    return SPEC_EINVAL;
  const int n_slices = (vocab + kTopkSlice - 1) / kTopkSlice;
  float *z = scratch_f;                                       // [vocab], then the top-k scratch of one row (as spec_k_topk_logprob)
  float *sc_val = z + (size_t)(vocab + 3) / 4 * 4;
  float2 *sc_stat = (float2 *)(sc_val + (size_t)kMaxTopK * n_slices * kMaxTopK);
  float *top_lp = (float *)(sc_stat + (size_t)kMaxTopK * n_slices);
  int *sc_idx = scratch_i, *top_tok = scratch_i + (size_t)kMaxTopK * n_slices * kMaxTopK;
  return launch_sample_children(logits, vocab, temperature, m, seed, cycle, node_stream, z, sc_val, sc_idx, sc_stat, top_tok, top_lp,
                                out, (hipStream_t)stream) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

}  // extern "C"

// ---- training-side entry points (spec_train.h) -----------------------------------------------
#include "../../include/spec_train.h"
extern "C" {

int spec_hca_attention(int32_t n_streams, const void *q, const void *const *k, const void *const *v, int32_t batch,
                       int32_t seq, int32_t hq, int32_t hkv, int32_t hd, void *out, void *stream) {
  if (!q || !k || !v || !out || n_streams < 1 || n_streams > SPEC_HCA_MAX_STREAMS || batch < 1 || seq < 1) return SPEC_EINVAL;
  if ((hd != 64 && hd != 128) || hkv < 1 || hq < hkv || hq % hkv) return SPEC_EINVAL;
  static_assert(SPEC_HCA_MAX_STREAMS == kMaxStreams, "header and kernel agree on the stream limit");
  HcaArgs a{};
  a.q = q; a.out = out; a.n_streams = n_streams; a.batch = batch; a.seq = seq; a.hq = hq; a.hkv = hkv; a.hd = hd;
  a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)hd));
  if (((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return SPEC_EINVAL;
  for (int m = 0; m < n_streams; m++) {
    if (!k[m] || !v[m] || ((uintptr_t)k[m] & 15) || ((uintptr_t)v[m] & 15)) return SPEC_EINVAL;
    a.k[m] = k[m]; a.v[m] = v[m];
  }
  return launch_hca_attention(a, (hipStream_t)stream) == hipSuccess ? SPEC_OK : SPEC_EHIP;
}

namespace {
constexpr int kLossChunk = 512;                               // positions whose logits are live at a time
struct LossLayout { int chunk, ldz; size_t zq, zp, cand, rows_topk, rows_ce, total; };   // offsets in floats
LossLayout loss_layout(int rows, int vocab, int k) {
  LossLayout l{};
  l.chunk = rows < kLossChunk ? rows : kLossChunk;
  l.ldz = (vocab + 63) / 64 * 64;
  auto up = [](size_t x) { return (x + 63) / 64 * 64; };
  size_t o = 0;
  l.zq = o; o += up((size_t)l.chunk * l.ldz);
  l.zp = o; o += up((size_t)l.chunk * l.ldz);
  l.cand = o; o += up(topk_loss_scratch_floats(l.chunk, vocab, k));
  l.rows_topk = o; o += up((size_t)rows);                     // used when the caller does not want the per-row losses
  l.rows_ce = o; o += up((size_t)rows);
  l.total = o;
  return l;
}
bool loss_args_ok(int rows, int vocab, int k) {
  return rows >= 1 && vocab >= 1 && k >= 1 && k <= SPEC_LOSS_MAX_K && k <= vocab && (int64_t)((vocab + kTopkSlice - 1) / kTopkSlice) * k <= 4096;
}
}  // namespace

uint64_t spec_topk_loss_scratch_bytes(int32_t rows, int32_t vocab, int32_t k) {
  if (!loss_args_ok(rows, vocab, k)) return 0;
  return (uint64_t)loss_layout(rows, vocab, k).total * sizeof(float);
}

int spec_topk_loss(int32_t dtype, const void *feat_target, const void *feat_draft, int32_t rows, int32_t d,
                   const void *lm_head, int32_t vocab, int32_t k, void *scratch, uint64_t scratch_bytes, float *loss_topk,
                   float *loss_ce, float *loss_sum, void *stream) {
  static_assert(SPEC_LOSS_MAX_K == kLossMaxK, "header and kernel agree on the K limit");
  if (!feat_target || !feat_draft || !lm_head || !scratch || (dtype != 0 && dtype != 1) || !loss_args_ok(rows, vocab, k))
    return SPEC_EINVAL;
  const int epl = dtype == 1 ? 8 : 4;
  if (d < 1 || d % epl || ((uintptr_t)scratch & 255)) return SPEC_EINVAL;
  const LossLayout l = loss_layout(rows, vocab, k);
  if (scratch_bytes < (uint64_t)l.total * sizeof(float)) return SPEC_EINVAL;
  float *sf = (float *)scratch;
  float *out_topk = loss_topk ? loss_topk : sf + l.rows_topk, *out_ce = loss_ce ? loss_ce : sf + l.rows_ce;
  const size_t esz = dtype == 1 ? 2 : 4;
  hipStream_t st = (hipStream_t)stream;
  for (int r0 = 0; r0 < rows; r0 += l.chunk) {
    const int m = rows - r0 < l.chunk ? rows - r0 : l.chunk;
    const void *xs[2] = {(const char *)feat_target + (size_t)r0 * d * esz, (const char *)feat_draft + (size_t)r0 * d * esz};
    float *zs[2] = {sf + l.zq, sf + l.zp};
    for (int side = 0; side < 2; side++) {                    // the LM head over the chunk's rows: fp32 logits
      GemmArgs a{};
      a.x = xs[side]; a.ldx = d; a.m = m; a.in = d;
      for (int s = 0; s < 3; s++) { a.seg_w[s] = lm_head; a.seg_rows[s] = 0; a.seg_blocks[s] = 0; a.seg_col0[s] = 0; }
      a.seg_rows[0] = vocab; a.seg_blocks[0] = (vocab + 31) / 32;
      a.nseg = 1; a.total_blocks = a.seg_blocks[0];
      a.part = zs[side]; a.ldp = l.ldz; a.m_pad = l.chunk; a.n_split = 1;
      if (launch_gemm(dtype, a, st) != hipSuccess) return SPEC_EHIP;
    }
    if (launch_topk_loss_rows(zs[0], zs[1], l.ldz, m, vocab, k, sf + l.cand, out_topk + r0, out_ce + r0, st) != hipSuccess)
      return SPEC_EHIP;
  }
  if (loss_sum && launch_loss_total(out_topk, out_ce, rows, loss_sum, st) != hipSuccess) return SPEC_EHIP;
  return SPEC_OK;
}

}  // extern "C"
