// Shape-agnostic strided matrix product on the vector ALUs: the correctness
// path for fp32 storage and for shapes the MFMA kernels do not tile.  64x64
// output tile per workgroup, 4x4 outputs per thread, operands staged through
// LDS in K-slabs of 16; every access is bounds-checked, so any M, N, K works.
// Causal modes restrict the outputs (n <= m) or the contraction (k <= m or
// k >= m) exactly, without relying on zero padding in the operands.
#include "device_common.h"
#include "kernels.h"

namespace lynx {
namespace {

constexpr int BM = 64, BN = 64, BK = 16, kThreads = 256;

template <typename T>
__global__ void __launch_bounds__(kThreads) gemm_generic_kernel(GemmDesc d) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  if (d.causal == kCausalOutLower && n0 > m0 + BM - 1) return;
  const int z1 = blockIdx.z / d.nz2, z2 = blockIdx.z - z1 * d.nz2;
  const T* A = static_cast<const T*>(d.A) + z1 * d.a_sz1 + z2 * d.a_sz2;
  const T* B = static_cast<const T*>(d.B) + z1 * d.b_sz1 + z2 * d.b_sz2;
  T* C = static_cast<T*>(d.C) + z1 * d.c_sz1 + z2 * d.c_sz2;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;

  int k_begin = 0, k_end = d.K;
  if (d.causal == kCausalKLeM) k_end = min(d.K, m0 + BM);
  if (d.causal == kCausalKGeM) k_begin = (m0 / BK) * BK;

  float acc[4][4] = {};
  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
    // A slab [BM x BK]: walk along whichever dimension is contiguous
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int mm, kk;
      if (d.a_sk == 1) { kk = tid & 15; mm = (tid >> 4) + 16 * r; }
      else { mm = tid & 63; kk = (tid >> 6) + 4 * r; }
      const int m = m0 + mm, k = k0 + kk;
      bool ok = m < d.M && k < d.K;
      if (d.causal == kCausalKLeM) ok = ok && k <= m;
      if (d.causal == kCausalKGeM) ok = ok && k >= m;
      As[kk][mm] = ok ? load1(A + m * d.a_sm + k * d.a_sk) : 0.0f;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int nn, kk;
      if (d.b_sk == 1) { kk = tid & 15; nn = (tid >> 4) + 16 * r; }
      else { nn = tid & 63; kk = (tid >> 6) + 4 * r; }
      const int n = n0 + nn, k = k0 + kk;
      const bool ok = n < d.N && k < d.K;
      Bs[kk][nn] = ok ? load1(B + k * d.b_sk + n * d.b_sn) : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
  const T* bias = static_cast<const T*>(d.bias);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= d.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= d.N) continue;
      if (d.causal == kCausalOutLower && n > m) continue;
      float v = acc[i][j];
      if (bias != nullptr) v += load1(bias + n);
      store1(C + m * d.c_sm + n, v);
    }
  }
}

}  // namespace

hipError_t gemm_generic(int dtype, const GemmDesc& d, hipStream_t st) {
  const dim3 grid((d.N + BN - 1) / BN, (d.M + BM - 1) / BM, d.nz1 * d.nz2);
  if (dtype == 1)
    hipLaunchKernelGGL((gemm_generic_kernel<bf16_t>), grid, dim3(kThreads), 0, st, d);
  else
    hipLaunchKernelGGL((gemm_generic_kernel<float>), grid, dim3(kThreads), 0, st, d);
  return hipGetLastError();
}

}  // namespace lynx
