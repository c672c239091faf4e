// llc_couple_static: llc_couple for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  The partial results of
// the scan live in an array that is part of this code object instead of a caller's workspace.
#include <mutex>

#include "common.hpp"

using namespace llc;

// One array per GPU (every device that loads this code object holds its own copy at its own
// address).  In host code the array's name is only a handle: the device address comes from
// hipGetSymbolAddress, once per device, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[LLC_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once known

int static_scratch(void **ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LLC_E_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return LLC_E_LAUNCH;
    if (((uintptr_t)p & 255) != 0) return LLC_E_LAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return LLC_OK;
}
}  // namespace

extern "C" int llc_couple_static(const llc_couple_args *a) {
  if (a == nullptr) return LLC_E_NULL;
  // plan the call against the array's size first: a shape that does not fit is refused before
  // the device is touched (the placeholder address is never dereferenced by a dry run)
  llc_couple_args c = *a;
  c.flags |= LLC_FLAG_DRY_RUN;
  int rc = couple_on(&c, (void *)(uintptr_t)256, LLC_STATIC_SCRATCH_BYTES);
  if (rc == LLC_E_WORKSPACE) return LLC_E_SCRATCH;
  if (rc != LLC_OK || (a->flags & LLC_FLAG_DRY_RUN) != 0 || a->B == 0) return rc;
  void *ptr = nullptr;
  rc = static_scratch(&ptr);
  if (rc != LLC_OK) return rc;
  // every cell of the partial results that is read is written by this call's scan first, and
  // the shared running bests are preset by a fill kernel: nothing of an earlier call is seen
  return couple_on(a, ptr, LLC_STATIC_SCRATCH_BYTES);
}

