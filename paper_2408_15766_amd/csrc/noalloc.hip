// spec_k_topk_logprob_static: the per-row top-k log-probability call for callers that cannot allocate device memory
// and have no workspace to hand over (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  The two selection kernels are those of spec_k_topk_logprob; their scratch (per-slice candidates and
// softmax statistics) lives in a file-scope device array instead of caller memory.
//
// The array's name is only a host-side handle: its device address is looked up once per device with
// hipGetSymbolAddress (with that device current: every GPU holds its own copy at its own address) and only that
// address is ever passed to a kernel.
#include <mutex>

#include "../../include/spec.h"
#include "../../include/spec_kernels.h"
#include "common.h"
#include "kernels.h"

namespace {

constexpr int kStaticSlices = SPEC_STATIC_TOPK_MAX_VOCAB / spec::kTopkSlice;      // 64 slices of 4096 tokens
static_assert(SPEC_STATIC_TOPK_MAX_VOCAB % spec::kTopkSlice == 0, "the limit is a whole number of slices");
constexpr size_t kValBytes = (size_t)spec::kMaxTopK * kStaticSlices * spec::kMaxTopK * sizeof(float);   // candidates' values
constexpr size_t kStatBytes = (size_t)spec::kMaxTopK * kStaticSlices * sizeof(float2);                  // (max, sum exp) per slice
constexpr size_t kIdxBytes = (size_t)spec::kMaxTopK * kStaticSlices * spec::kMaxTopK * sizeof(int);     // candidates' tokens
constexpr size_t kScratchBytes = kValBytes + kStatBytes + kIdxBytes;                                    // 136 KiB
static_assert(kValBytes % 256 == 0 && kStatBytes % 256 == 0, "the three regions stay 256-byte aligned");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices] = {};           // device address of `scratch` on each device, once looked up

// Device address of this device's copy of the array (the current device must be `dev`).
hipError_t scratch_address(int dev, void **out) {
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void *p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" int spec_k_topk_logprob_static(const float *logits, int32_t rows, int32_t vocab, int32_t k, int32_t *top_tok,
                                          float *top_lp, void *stream) {
  if (!logits || !top_tok || !top_lp || rows < 1 || rows > spec::kMaxTopK || vocab < 1 || k < 1 || k > spec::kMaxTopK || k > vocab)
    return SPEC_EINVAL;
  if (vocab > SPEC_STATIC_TOPK_MAX_VOCAB) return SPEC_ECAP;   // beyond what the static scratch holds
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPEC_EHIP;
  void *base = nullptr;
  if (scratch_address(dev, &base) != hipSuccess) return SPEC_EHIP;
  char *b = (char *)base;
  float *sc_val = (float *)b;
  float2 *sc_stat = (float2 *)(b + kValBytes);
  int *sc_idx = (int *)(b + kValBytes + kStatBytes);
  // Nothing has to be cleared: the first kernel writes every candidate and statistic the second one reads.
  return spec::launch_rows_topk_logprob(logits, rows, vocab, k, sc_val, sc_idx, sc_stat, top_tok, top_lp, (hipStream_t)stream) ==
                 hipSuccess
             ? SPEC_OK
             : SPEC_EHIP;
}
