// zo_score for callers that cannot allocate device memory (code under HIP graph capture, tight serving
// loops, harnesses that forbid hipMalloc): the scratch of the scoring kernels lives in a static device
// array of this library instead of a caller workspace.
#include <stdio.h>

#include <mutex>

#include "zo_host.hpp"
#include "zo_internal.hpp"

namespace {

constexpr size_t kScratchBytes = (size_t)32 << 20;   // held by every GPU the library runs on until the process ends
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Device address of this device's copy of the array.  The array's name is a host-side stand-in, not a
// device address: each GPU holds its own copy at its own address, looked up once per device.
std::mutex g_mu;
void* g_scratch_ptr[zo::kMaxDevices];

int32_t scratch_for_current_device(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return zo::fail_status(ZO_ERR_HIP, hipGetErrorString(e));
  if (dev < 0 || dev >= zo::kMaxDevices) return zo::fail_status(ZO_ERR_UNSUPPORTED, "device index beyond the per-device table");
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return zo::fail_status(ZO_ERR_HIP, e != hipSuccess ? hipGetErrorString(e) : "hipGetSymbolAddress returned NULL");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return ZO_OK;
}

}  // namespace

extern "C" {

size_t zo_score_static_capacity(void) { return kScratchBytes; }

int32_t zo_score_static(const zo_batch* batch, const void* H, int64_t ldh, const void* W_head, int64_t ldw,
                        int32_t vocab, int32_t d, zo_dtype dtype, const int32_t* targets, float* tok_nll,
                        float* seq_nll, float* cand_sum, int32_t* cand_cnt, void* stream) {
  // all validation before the first HIP call, as in zo_score
  if (int32_t st = zo::score_validate(batch, H, ldh, W_head, ldw, vocab, d, dtype, targets, seq_nll, cand_sum, cand_cnt))
    return st;
  const size_t need = zo_score_workspace_bytes(batch->n_tokens, batch->n_seqs, vocab, d, dtype);
  if (need > kScratchBytes) {
    char msg[256];
    snprintf(msg, sizeof msg,
             "zo_score_static: %d tokens x vocabulary %d need %zu bytes of scratch, the static array holds %zu; "
             "use zo_score with a caller workspace",
             batch->n_tokens, vocab, need, kScratchBytes);
    return zo::fail_status(ZO_ERR_WORKSPACE, msg);
  }
  if (batch->n_seqs == 0 && batch->n_cands == 0) return ZO_OK;
  void* ptr = nullptr;
  if (int32_t st = scratch_for_current_device(&ptr)) return st;
  // Every scratch region the kernels read is written by an earlier kernel of the same call (the list of scored
  // tokens and its count, the per-tile partial maxima and sums, the target logits), so nothing has to be
  // cleared although the array keeps the previous call's contents.
  return zo_score(batch, H, ldh, W_head, ldw, vocab, d, dtype, targets, tok_nll, seq_nll, cand_sum, cand_cnt, ptr,
                  kScratchBytes, stream);
}

}  // extern "C"
