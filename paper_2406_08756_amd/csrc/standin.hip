// A rate-limited device copy that stands in, in single-GPU measurements, for the
// tensor-parallel all-reduce this build omits (the communication that the paper's
// schedule overlaps regeneration with).  A fixed, small number of workgroups walk the
// buffer, so like a collective's copy engines or reduction kernels it occupies a few
// compute units and a bounded share of the memory bandwidth for a while, instead of
// the whole chip for an instant.  Measurement aid only: nothing on the layer's path uses it.
#include <hip/hip_runtime.h>

#include "../../include/lynx.h"

namespace {

__global__ void __launch_bounds__(256)
standin_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t nvec) {
  for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < nvec;
       i += static_cast<size_t>(gridDim.x) * 256)
    dst[i] = src[i];
}

}  // namespace

extern "C" lynx_status lynx_comm_standin(void* dst_device, const void* src_device, size_t bytes, int workgroups,
                                         void* hip_stream) {
  if (dst_device == nullptr || src_device == nullptr || bytes % 16 != 0 || workgroups < 1 || workgroups > 4096 ||
      ((reinterpret_cast<uintptr_t>(dst_device) | reinterpret_cast<uintptr_t>(src_device)) & 15u))
    return LYNX_ERR_INVALID_ARG;
  if (bytes == 0) return LYNX_OK;
  hipLaunchKernelGGL(standin_copy_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint4*>(src_device), static_cast<uint4*>(dst_device), bytes / 16);
  return hipGetLastError() == hipSuccess ? LYNX_OK : LYNX_ERR_HIP;
}
