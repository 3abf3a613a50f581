// ccq_gemm_static: ccq_gemm for callers that cannot allocate device memory (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc).  The fp32 partial tiles of the K shares, which ccq_gemm keeps in
// the caller's workspace, live here in a file-scope device array that every GPU the library runs on holds for
// the life of the process.  The kernels are the same; they receive the array's device address as their workspace.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

#include "ccq_internal.h"

namespace ccq {

constexpr int64_t kStaticScratchBytes = (int64_t)8 << 20;
constexpr int kMaxDevices = 64;

// In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on each GPU (every GPU holds its own copy at its own address), looked up once per
// device with that device current.  A racing first call on two host threads looks the same address up twice.
static std::atomic<void*> scratch_addr[kMaxDevices];

static int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return CCQ_ERR_HIP;
  }
  void* p = scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return CCQ_ERR_HIP;
    }
    scratch_addr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return CCQ_OK;
}

}  // namespace ccq

using namespace ccq;

extern "C" int64_t ccq_gemm_static_max_workspace(void) { return kStaticScratchBytes; }

extern "C" int ccq_gemm_static(const ccq_weight* w, const void* x, int32_t M, int64_t ldx, void* y, int64_t ldy, void* hip_stream) {
  const int64_t need = gemm_workspace_need(w, M);
  if (need > kStaticScratchBytes) return CCQ_ERR_WORKSPACE;  // an invalid descriptor (-1) is reported by the dispatcher below
  void* ws = nullptr;
  if (need > 0) {
    const int rc = scratch_of_current_device(&ws);
    if (rc != CCQ_OK) return rc;
  }
  // The partial tiles are written in full by the multiply kernel before the reduction reads them: nothing in the
  // array has to start at zero, whatever the previous call left there.
  return gemm_dispatch(w, x, M, ldx, y, ldy, ws, need > 0 ? kStaticScratchBytes : 0, hip_stream, nullptr);
}
