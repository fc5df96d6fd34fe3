// sbp_backward_linear_static: the linear backward for callers that cannot allocate device memory and have no
// workspace to hand over (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// Same kernels as sbp_backward_linear; the workspace (fp32 partial sums of the dW splits, db slices, the inverse
// row map) is a fixed array in device memory that belongs to the library.
#include <mutex>

#include "sbp_internal.h"

namespace sbp {

// One copy of this array exists on every GPU the library is loaded on, from the first use of the library on that
// GPU until the process ends.  In host code the name is only a handle: the device address comes from
// hipGetSymbolAddress, once per device, with that device current.
static __device__ __align__(256) unsigned char scratch[SBP_STATIC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (NULL + error text on failure).
static void* static_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(SBP_ERR_HIP, "no current device (or device number beyond %d)", kMaxDevices - 1);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      fail(SBP_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace sbp

using namespace sbp;

extern "C" {

size_t sbp_static_scratch_bytes(void) { return (size_t)SBP_STATIC_SCRATCH_BYTES; }

int32_t sbp_backward_linear_static(const void* dY, const int32_t* idx, const int32_t* inv, const void* Xk, const void* W,
                                   int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype, void* dW, float* db,
                                   void* dX, uint32_t flags, void* stream) {
  // the host-side checks of sbp_backward_linear, then the size limit, then (first HIP call) the scratch address
  int32_t st = check_linear_args(dY, idx, Xk, W, M, K, Cin, Cout, dtype, dW, dX, flags);
  if (st != SBP_OK) return st;
  const size_t need = sbp_backward_linear_workspace(M, K, Cin, Cout, dtype, flags);
  if (need > (size_t)SBP_STATIC_SCRATCH_BYTES)
    return fail(SBP_ERR_CAPACITY, "these sizes need %zu bytes of scratch, the static buffer holds %zu: use sbp_backward_linear "
                "with a workspace of the caller's", need, (size_t)SBP_STATIC_SCRATCH_BYTES);
  if (!dW && !db && !dX) return SBP_OK;
  void* ws = static_scratch_ptr();
  if (!ws) return SBP_ERR_HIP;
  const LinearPlan p = plan_linear(M, K, Cin, Cout, dtype, flags);
  return launch_backward_linear(p, dY, idx, inv, Xk, W, M, K, Cin, Cout, dtype, dW, db, dX, ws, flags,
                                (hipStream_t)stream);
}

}  // extern "C"
