// cls_scores_static: the standalone importance scoring for callers that cannot allocate device
// memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// It is cls_scores with the workspace taken from a device array of this library instead of from
// the caller.  The array's address on a device is looked up once per device with
// hipGetSymbolAddress; host code never uses the array's name as an address.
#include <mutex>

#include "ns_common.h"

namespace ns {
namespace {

constexpr size_t kScratchBytes = 8u << 20;   // 8 MiB per GPU, held until the process ends
constexpr int kMaxDevices = 64;

__device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices];            // per device: the array's device address, once known

// The array's address on the current device (nullptr and an error message on failure).
void *scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(NS_ERR_HIP, "cls_scores_static: cannot identify the current device");
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      fail(NS_ERR_HIP, "cls_scores_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace
}  // namespace ns

using namespace ns;

extern "C" {

size_t cls_scores_static_max_bytes(void) { return kScratchBytes; }

ns_status cls_scores_static(const ns_attn_desc *desc, const void *q, const void *k, float *scores, void *stream) {
  const size_t need = cls_scores_workspace_bytes(desc);   // 0 for an invalid descriptor: reported below
  if (need > kScratchBytes)
    return fail(NS_ERR_WORKSPACE,
                "cls_scores_static: this problem needs %zu bytes of scratch memory, the built-in buffer has %zu; "
                "use cls_scores with a workspace of your own", need, kScratchBytes);
  void *ptr = scratch_on_current_device();
  if (!ptr) return NS_ERR_HIP;
  // every float of the logits and partial records that the scoring kernel reads is written by the
  // row kernel of the same call first, so nothing has to be cleared
  return cls_scores_impl(desc, q, k, scores, ptr, kScratchBytes, stream);
}

}  // extern "C"
