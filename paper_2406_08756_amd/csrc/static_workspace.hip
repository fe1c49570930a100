// A workspace that needs no allocation call: a fixed block of device memory that lives in
// the library's code object, for callers that cannot call hipMalloc (code under HIP graph
// capture, serving loops, harnesses that forbid it).  Every GPU the library runs on holds
// its own copy of the array, at its own address, from the moment the code object is loaded
// there until the process ends.
//
// In host code the array's name is only a handle for the symbol, never a device address:
// the address is asked for once per device (hipGetSymbolAddress, with that device current)
// and from then on only that pointer is used - for kernel arguments and copies alike.
#include <hip/hip_runtime.h>

#include <mutex>

#include "static_workspace.h"

namespace lynx {
namespace {

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticWorkspaceBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mutex;
void* g_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once known
bool g_busy[kMaxDevices] = {};   // a layer currently lives in it

}  // namespace

hipError_t static_workspace_acquire(void** ptr, int* device) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mutex);
  if (g_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 255u) != 0) return hipErrorInvalidSymbol;
    g_ptr[dev] = p;
  }
  if (g_busy[dev]) return hipErrorContextAlreadyInUse;
  g_busy[dev] = true;
  *ptr = g_ptr[dev];
  *device = dev;
  return hipSuccess;
}

void static_workspace_release(int device) {
  if (device < 0 || device >= kMaxDevices) return;
  std::lock_guard<std::mutex> lock(g_mutex);
  g_busy[device] = false;
}

}  // namespace lynx
