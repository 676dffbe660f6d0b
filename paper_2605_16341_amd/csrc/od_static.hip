// orthdion_step_static: the optimizer step for callers that cannot allocate device memory (code
// under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The step's
// workspace - everything orthdion_step keeps in the caller's `workspace` argument: the factors
// P and R, split-reduction partials, Gram and triangular matrices, fp16 operand copies, scale,
// flag and diagnostic words - lives in a file-scope device array of this library instead.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until
// the process ends.  The array's name is only a host-side stand-in: the device address is
// looked up once per device with hipGetSymbolAddress and kept; only that address is handed to
// kernels.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/orthdion.h"
#include "od_internal.h"

namespace {

constexpr size_t kStaticScratchBytes = ORTHDION_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call there).
int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ORTHDION_E_HIP;
  std::lock_guard<std::mutex> guard(g_lock);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return ORTHDION_E_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return ORTHDION_OK;
}

}  // namespace

extern "C" size_t orthdion_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int orthdion_step_static(orthdion_handle h, void* const* X, const void* const* G, float* const* M,
                                    float* const* Q, void* stream) {
  if (!h) return ORTHDION_E_NULL_PTR;
  if (orthdion_workspace_bytes(h) > kStaticScratchBytes) return ORTHDION_E_WORKSPACE_TOO_SMALL;
  void* ws = nullptr;
  const int rc = scratch_of_current_device(&ws);
  if (rc != ORTHDION_OK) return rc;
  // orthdion_step clears the words of the workspace that must start at zero (scale, flag and
  // accumulator words) itself, every step, so the contents a previous call left are harmless.
  return orthdion_step_impl(h, X, G, M, Q, ws, kStaticScratchBytes, stream, 0);
}
