// LayerNorm forward (operators 1 and 9) and backward.  Forward: one wavefront
// per token row, the row held in registers, two-pass mean / variance in fp32,
// statistics written for backward.  Backward: one workgroup of four
// wavefronts per row stream; each lane owns fixed columns so the per-column
// sums for dgamma / dbeta accumulate in registers over the rows the workgroup
// visits, and are then reduced over workgroups in a second fixed-order stage.
#include "device_common.h"
#include "kernels.h"
#include "reduce_partials.h"

namespace lynx {
namespace {

constexpr int kFwdRowsPerBlock = 4;
constexpr int kBwdThreads = 256;
constexpr int kBwdMaxBlocks = 1024;

template <typename T, int NC>
__global__ void __launch_bounds__(kFwdRowsPerBlock* kWave)
layernorm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                     const T* __restrict__ beta, T* __restrict__ y, float* __restrict__ mean,
                     float* __restrict__ rstd, int rows, int cols, float eps) {
  const int lane = threadIdx.x & (kWave - 1);
  const int r = blockIdx.x * kFwdRowsPerBlock + (threadIdx.x >> 6);
  if (r >= rows) return;
  const size_t base = static_cast<size_t>(r) * cols;
  float v[NC][8];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (lane + c * kWave) * 8;
    if (j0 < cols) {
      load8(x + base + j0, v[c]);
#pragma unroll
      for (int k = 0; k < 8; ++k) sum += v[c][k];
    }
  }
  const float inv_n = 1.0f / static_cast<float>(cols);
  const float mu = wave_sum(sum) * inv_n;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (lane + c * kWave) * 8;
    if (j0 < cols) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        v[c][k] -= mu;
        sq += v[c][k] * v[c][k];
      }
    }
  }
  const float rs = rsqrtf(wave_sum(sq) * inv_n + eps);
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (lane + c * kWave) * 8;
    if (j0 < cols) {
      float g[8], b[8];
      load8(gamma + j0, g);
      load8(beta + j0, b);
#pragma unroll
      for (int k = 0; k < 8; ++k) v[c][k] = g[k] * (v[c][k] * rs) + b[k];
      store8(y + base + j0, v[c]);
    }
  }
  if (lane == 0) {
    mean[r] = mu;
    rstd[r] = rs;
  }
}

// Block-wide sums of four values; every thread gets all totals.  The combination
// order is fixed.
__device__ __forceinline__ void block_sum4(float (&v)[4], float* smem) {
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = wave_sum(v[i]);
  const int w = threadIdx.x >> 6;
  __syncthreads();  // previous use of smem is over
  if ((threadIdx.x & (kWave - 1)) == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) smem[4 * i + w] = v[i];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i)
    v[i] = (smem[4 * i] + smem[4 * i + 1]) + (smem[4 * i + 2] + smem[4 * i + 3]);
}

// Two rows per iteration: all loads of both rows (dy, x, residual gradient) are
// issued before the reductions, which doubles the bytes in flight per workgroup
// and halves the number of workgroup barriers per row.
template <typename T, int NC>
__global__ void __launch_bounds__(kBwdThreads)
layernorm_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                     const float* __restrict__ mean, const float* __restrict__ rstd,
                     const T* __restrict__ gamma, const T* dres, T* dx_out,
                     float* __restrict__ part_dg, float* __restrict__ part_db, int rows, int cols) {
  __shared__ float smem[16];
  float g[NC][8], adg[NC][8], adb[NC][8];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (threadIdx.x + c * kBwdThreads) * 8;
    if (j0 < cols) load8(gamma + j0, g[c]);
#pragma unroll
    for (int k = 0; k < 8; ++k) { adg[c][k] = 0.f; adb[c][k] = 0.f; }
  }
  const float inv_n = 1.0f / static_cast<float>(cols);
  for (int r0 = 2 * blockIdx.x; r0 < rows; r0 += 2 * gridDim.x) {
    const bool two = r0 + 1 < rows;
    const int rr[2] = {r0, two ? r0 + 1 : r0};
    float gd[2][NC][8], xh[2][NC][8], dr[2][NC][8];
    float mu[2], rs[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      mu[q] = mean[rr[q]];
      rs[q] = rstd[rr[q]];
      const size_t base = static_cast<size_t>(rr[q]) * cols;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int j0 = (threadIdx.x + c * kBwdThreads) * 8;
        if (j0 < cols) {
          load8(dy + base + j0, gd[q][c]);
          load8(x + base + j0, xh[q][c]);
          load8(dres + base + j0, dr[q][c]);
        }
      }
    }
    float sums[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const float live = (q == 0 || two) ? 1.0f : 0.0f;  // a lone last row is not counted twice
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int j0 = (threadIdx.x + c * kBwdThreads) * 8;
        if (j0 < cols) {
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            xh[q][c][k] = (xh[q][c][k] - mu[q]) * rs[q];
            adg[c][k] += live * gd[q][c][k] * xh[q][c][k];
            adb[c][k] += live * gd[q][c][k];
            gd[q][c][k] *= g[c][k];
            sums[2 * q] += gd[q][c][k];
            sums[2 * q + 1] += gd[q][c][k] * xh[q][c][k];
          }
        }
      }
    }
    block_sum4(sums, smem);
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      if (q == 1 && !two) break;
      const size_t base = static_cast<size_t>(rr[q]) * cols;
      const float m1 = sums[2 * q] * inv_n, m2 = sums[2 * q + 1] * inv_n;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int j0 = (threadIdx.x + c * kBwdThreads) * 8;
        if (j0 < cols) {
          float o[8];
#pragma unroll
          for (int k = 0; k < 8; ++k)
            o[k] = dr[q][c][k] + rs[q] * (gd[q][c][k] - m1 - xh[q][c][k] * m2);
          store8(dx_out + base + j0, o);
        }
      }
    }
  }
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (threadIdx.x + c * kBwdThreads) * 8;
    if (j0 < cols) {
      store8(part_dg + static_cast<size_t>(blockIdx.x) * cols + j0, adg[c]);
      store8(part_db + static_cast<size_t>(blockIdx.x) * cols + j0, adb[c]);
    }
  }
}

int bwd_blocks(int rows) {
  const int pairs = (rows + 1) / 2;
  return pairs < kBwdMaxBlocks ? pairs : kBwdMaxBlocks;
}

}  // namespace

hipError_t layernorm_fwd(int dtype, const void* x, const void* gamma, const void* beta, void* y,
                         float* mean, float* rstd, int rows, int cols, float eps, hipStream_t st) {
  if (cols > 8192 || cols % 8) return hipErrorInvalidValue;
  const dim3 grid((rows + kFwdRowsPerBlock - 1) / kFwdRowsPerBlock);
  const dim3 block(kFwdRowsPerBlock * kWave);
  const int nc = (cols / 8 + kWave - 1) / kWave;
#define CALL(NC)                                                                                   \
  if (dtype == 1)                                                                                  \
    hipLaunchKernelGGL((layernorm_fwd_kernel<bf16_t, NC>), grid, block, 0, st,                     \
                       static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(gamma),           \
                       static_cast<const bf16_t*>(beta), static_cast<bf16_t*>(y), mean, rstd,      \
                       rows, cols, eps);                                                           \
  else                                                                                             \
    hipLaunchKernelGGL((layernorm_fwd_kernel<float, NC>), grid, block, 0, st,                      \
                       static_cast<const float*>(x), static_cast<const float*>(gamma),             \
                       static_cast<const float*>(beta), static_cast<float*>(y), mean, rstd, rows,  \
                       cols, eps)
  if (nc <= 1) { CALL(1); }
  else if (nc <= 2) { CALL(2); }
  else if (nc <= 4) { CALL(4); }
  else if (nc <= 6) { CALL(6); }
  else if (nc <= 8) { CALL(8); }
  else if (nc <= 10) { CALL(10); }
  else if (nc <= 12) { CALL(12); }
  else { CALL(16); }
#undef CALL
  return hipGetLastError();
}

size_t layernorm_bwd_scratch_bytes(int rows, int cols) {
  return 2 * static_cast<size_t>(bwd_blocks(rows)) * cols * sizeof(float);
}

hipError_t layernorm_bwd(int dtype, const void* dy, const void* x, const float* mean,
                         const float* rstd, const void* gamma, const void* dres, void* dx_out,
                         void* dgamma, void* dbeta, float* scratch, int rows, int cols,
                         hipStream_t st) {
  if (cols > 8192 || cols % 8) return hipErrorInvalidValue;
  const int nb = bwd_blocks(rows);
  float* part_dg = scratch;
  float* part_db = scratch + static_cast<size_t>(nb) * cols;
  const int nc = (cols / 8 + kBwdThreads - 1) / kBwdThreads;
#define CALL(NC)                                                                                   \
  if (dtype == 1)                                                                                  \
    hipLaunchKernelGGL((layernorm_bwd_kernel<bf16_t, NC>), dim3(nb), dim3(kBwdThreads), 0, st,     \
                       static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(x), mean, rstd,  \
                       static_cast<const bf16_t*>(gamma), static_cast<const bf16_t*>(dres),        \
                       static_cast<bf16_t*>(dx_out), part_dg, part_db, rows, cols);                \
  else                                                                                             \
    hipLaunchKernelGGL((layernorm_bwd_kernel<float, NC>), dim3(nb), dim3(kBwdThreads), 0, st,      \
                       static_cast<const float*>(dy), static_cast<const float*>(x), mean, rstd,    \
                       static_cast<const float*>(gamma), static_cast<const float*>(dres),          \
                       static_cast<float*>(dx_out), part_dg, part_db, rows, cols)
  if (nc <= 1) { CALL(1); }
  else if (nc <= 2) { CALL(2); }
  else if (nc <= 3) { CALL(3); }
  else { CALL(4); }
#undef CALL
  if (dtype == 1)
    launch_reduce_partials<bf16_t>(part_dg, static_cast<bf16_t*>(dgamma), part_db,
                                   static_cast<bf16_t*>(dbeta), nb, cols, st);
  else
    launch_reduce_partials<float>(part_dg, static_cast<float*>(dgamma), part_db,
                                  static_cast<float*>(dbeta), nb, cols, st);
  return hipGetLastError();
}

}  // namespace lynx
