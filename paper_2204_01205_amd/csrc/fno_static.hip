// fno_spectral_conv_fwd_static: the spectral convolution for callers that cannot allocate.
//
// Same kernels and kernel sequence as fno_spectral_conv_fwd; the workspace (pruned
// intermediates, twiddle tables, table blobs) is a fixed array in device memory that belongs to
// the library instead of a buffer the caller brings.  Each GPU the library runs on holds its
// own copy of the array, at its own address, until the process ends.
#include "../../include/fno.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdio>
#include <mutex>

namespace fno {
// last detail text of the calling thread, shared with fno_status_string (fno_api.cpp)
void set_status_detail(const char* text);
}  // namespace fno

namespace {

constexpr size_t kScratchBytes = FNO_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

// In host code this name is only a handle for hipGetSymbolAddress; the device address it
// stands for is looked up once per device and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_mutex;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (looked up on the first call there).
int scratch_on_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fno::set_status_detail(e != hipSuccess ? hipGetErrorString(e) : "device ordinal outside the table");
    return FNO_EHIP;
  }
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    std::lock_guard<std::mutex> lock(g_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (p == nullptr) {
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || p == nullptr) {
        fno::set_status_detail(e != hipSuccess ? hipGetErrorString(e) : "scratch symbol has no device address");
        return FNO_EHIP;
      }
      g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return FNO_OK;
}

}  // namespace

extern "C" int fno_spectral_conv_fwd_static(const fno_desc* desc, const float* x, const float* R, float* y,
                                            float* xhat_save, void* stream) {
  size_t need = 0;
  int rc = fno_workspace_bytes(desc, FNO_OP_SPECTRAL_CONV_FWD, &need);
  if (rc != FNO_OK) return rc;
  if (need > kScratchBytes) {
    char msg[160];
    std::snprintf(msg, sizeof(msg), "this shape needs %zu bytes of scratch; the static array holds %zu", need,
                  kScratchBytes);
    fno::set_status_detail(msg);
    return FNO_ENOSPC;
  }
  void* ws = nullptr;
  rc = scratch_on_current_device(&ws);
  if (rc != FNO_OK) return rc;
  // every byte of the workspace a call reads is written earlier in the same call (tables first,
  // then each intermediate by its producer), so nothing left by the previous call is ever read
  return fno_spectral_conv_fwd(desc, x, R, y, xhat_save, ws, kScratchBytes, stream);
}
