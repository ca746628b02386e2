// rtc_minplus_conv_static: the min-plus convolution for callers that cannot allocate device
// memory.  The workspace that rtc_minplus_conv takes from its caller lives here, in a device
// array that is part of the library's code object; nothing in this file allocates or frees.
#include <hip/hip_runtime.h>

#include <mutex>

#include "rtc_internal.h"

namespace {

// The workspace itself.  In host code this name is only a handle for hipGetSymbolAddress; the
// device address, which differs per GPU, is looked up once per device and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[RTC_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (nullptr with *status set on failure).
void* scratch_address(int* status) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *status = RTC_ERR_HIP;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      *status = RTC_ERR_HIP;
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int rtc_minplus_conv_static(const void* f, const void* g, void* out, int64_t batch, int64_t n,
                                       int64_t stride_f, int64_t stride_g, rtc_dtype dt, int32_t* dev_flags,
                                       void* hip_stream) {
  // the shape decides the workspace; rtc_workspace_bytes returns 0 for an invalid shape or dtype,
  // which rtc_minplus_conv then reports with its own status
  const size_t need = rtc_workspace_bytes(RTC_OP_CONV, batch, n, dt);
  if (need > (size_t)RTC_STATIC_SCRATCH_BYTES) return RTC_ERR_WORKSPACE;
  int status = RTC_OK;
  void* ws = scratch_address(&status);
  if (ws == nullptr) return status;
  // Every array of the workspace is written by the call's own kernels before it is read, so what
  // the previous call left in it needs no clearing.
  return rtc_minplus_conv(f, g, out, batch, n, stride_f, stride_g, dt, ws, (size_t)RTC_STATIC_SCRATCH_BYTES, dev_flags,
                          hip_stream);
}
