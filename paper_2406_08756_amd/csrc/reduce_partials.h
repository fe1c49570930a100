// Second stage of the deterministic column reductions: out[c] = sum over the
// per-workgroup partial rows part[r][c], always added in the same order.
#pragma once
#include "device_common.h"

namespace lynx {

// Workgroup = 64 columns x 16 row groups; group g adds rows g, g+16, ... and
// the 16 group sums are then added in order.  blockIdx.y selects one of up to
// two (partials, output) pairs so LayerNorm's dgamma and dbeta share a launch.
template <typename T>
__global__ void __launch_bounds__(1024)
reduce_partials_kernel(const float* __restrict__ part0, T* __restrict__ out0,
                       const float* __restrict__ part1, T* __restrict__ out1, int nparts, int cols) {
  __shared__ float sm[16][64];
  const float* part = blockIdx.y == 0 ? part0 : part1;
  T* out = blockIdx.y == 0 ? out0 : out1;
  const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float s = 0.f;
  if (c < cols) {
#pragma unroll 8
    for (int r = grp; r < nparts; r += 16) s += part[static_cast<size_t>(r) * cols + c];
  }
  sm[grp][lane] = s;
  __syncthreads();
  if (grp == 0 && c < cols) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += sm[i][lane];
    store1(out + c, t);
  }
}

template <typename T>
inline void launch_reduce_partials(const float* part0, T* out0, const float* part1, T* out1,
                                   int nparts, int cols, hipStream_t st) {
  const dim3 grid((cols + 63) / 64, part1 != nullptr ? 2 : 1);
  hipLaunchKernelGGL((reduce_partials_kernel<T>), grid, dim3(1024), 0, st, part0, out0, part1, out1,
                     nparts, cols);
}

}  // namespace lynx
