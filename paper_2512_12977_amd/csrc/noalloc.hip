// vlc_first_token_noalloc: the first-token head for callers that cannot allocate device memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// The scratch the head needs - the normed rows and the partial choices of the greedy pick - lives in a
// file-scope device array instead of a caller-provided workspace; everything else is vlc_first_token.
#include <hip/hip_runtime.h>

#include <mutex>

#include "vlc_internal.h"

namespace {

constexpr int64_t kScratchBytes = (int64_t)1 << 20;   // 1 MiB per GPU, held until the process ends
constexpr int kMaxDevices = 64;

// Each GPU the library runs on holds its own copy of this array at its own address.  In host code the
// name below is only a handle for hipGetSymbolAddress: kernels and copies get the address that call
// returns for the current device, never the name.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
int scratch_of_current_device(void** out) {
  int dev = 0;
  VLC_CHECK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices)
    return vlc::fail(VLC_ERR_SHAPE, "vlc_first_token_noalloc: device %d beyond the %d this entry point keeps scratch for",
                     dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    VLC_CHECK_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return vlc::fail(VLC_ERR_HIP, "vlc_first_token_noalloc: hipGetSymbolAddress returned NULL");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return VLC_OK;
}

}  // namespace

extern "C" int64_t vlc_first_token_noalloc_max_bytes(void) { return kScratchBytes; }

extern "C" int vlc_first_token_noalloc(const void* h, const int32_t* rows, int64_t n_req, int H, int64_t vocab,
                                       float eps, const void* w_norm, const void* w_out, float* logits,
                                       int32_t* token, int dtype, void* stream) {
  if (dtype != VLC_F32 && dtype != VLC_BF16) return vlc::fail(VLC_ERR_DTYPE, "vlc_first_token_noalloc: dtype=%d", dtype);
  if (n_req < 0 || H <= 0) return vlc::fail(VLC_ERR_SHAPE, "vlc_first_token_noalloc: n_req=%lld H=%d", (long long)n_req, H);
  if (n_req == 0) return VLC_OK;
  const int64_t need = vlc_first_token_workspace_bytes(H, n_req, dtype);
  if (need <= 0) return VLC_ERR_SHAPE;   // message already set
  if (need > kScratchBytes)
    return vlc::fail(VLC_ERR_WORKSPACE,
                     "vlc_first_token_noalloc: %lld requests of H=%d need %lld bytes of scratch, the built-in array "
                     "holds %lld; use vlc_first_token with a workspace of your own",
                     (long long)n_req, H, (long long)need, (long long)kScratchBytes);
  void* ptr = nullptr;
  if (int rc = scratch_of_current_device(&ptr)) return rc;
  // Nothing in the scratch has to start at zero: the norm kernel writes every normed row and the first pass of
  // the greedy choice writes every partial (value, index) before the kernels that read them run.
  return vlc_first_token(h, rows, n_req, H, vocab, eps, w_norm, w_out, logits, token, ptr, kScratchBytes, dtype,
                         stream);
}
