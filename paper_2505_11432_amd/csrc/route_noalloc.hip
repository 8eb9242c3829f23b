// moe_route_noalloc: moe_route for callers that cannot allocate and have no workspace to pass (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  The per-chunk expert histograms that
// moe_route keeps in the caller's workspace live in a file-scope device array instead.  Every GPU the library runs
// on holds its own copy of the array, at its own address, until the process ends; the address is looked up once per
// device with hipGetSymbolAddress and only that pointer is ever handed to kernels (the array's name is a host-side
// stand-in, not a device address).
#include <mutex>

#include "moe_common.h"

namespace moe {
namespace {

constexpr size_t kScratchBytes = MOE_ROUTE_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Address of this device's copy of `scratch` (looked up on the first call with that device current).
int scratch_address(void** out) {
  int dev = 0;
  MOE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    MOE_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return MOE_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MOE_OK;
}

}  // namespace

int route_noalloc_prepare() {
  void* p = nullptr;
  return scratch_address(&p);
}

}  // namespace moe

using namespace moe;

extern "C" int moe_route_noalloc(const float* logits, int T, int E, int k, int renorm, int32_t* topk_idx,
                                 float* topk_w, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                                 void* stream) {
  if (T < 0 || E < 1 || E > MOE_MAX_EXPERTS || k < 1 || k > E || k > MOE_MAX_TOPK || (long)T * k > 0x7fffffffL)
    return MOE_ERR_INVALID;
  if (route_ws_bytes(T, E) > kScratchBytes) return MOE_ERR_UNSUPPORTED;     // beyond the static scratch: use moe_route
  if (T == 0) return MOE_OK;
  if (!logits || !topk_idx || !topk_w || !counts || !offsets || !perm || !inv_perm) return MOE_ERR_INVALID;
  void* ws = nullptr;
  const int rc = scratch_address(&ws);
  if (rc != MOE_OK) return rc;
  // Every histogram entry the later kernels read is written by the first kernel of this call, so nothing in the
  // scratch has to start at zero and the previous call's contents do not matter.
  return launch_route(logits, T, E, k, renorm != 0, 0, E, 0, 0, topk_idx, topk_w, nullptr, counts, offsets, perm, inv_perm,
                      ws, as_stream(stream));
}
