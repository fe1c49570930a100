// The library's built-in workspace (see static_workspace.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace lynx {

constexpr size_t kStaticWorkspaceBytes = static_cast<size_t>(64) << 20;

// Device address of the current device's copy of the built-in workspace, and that device's
// index; marks it taken.  hipErrorContextAlreadyInUse while another layer holds it.  Calls
// no allocation routine.
hipError_t static_workspace_acquire(void** ptr, int* device);
void static_workspace_release(int device);

}  // namespace lynx
