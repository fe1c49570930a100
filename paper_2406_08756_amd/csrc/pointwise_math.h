// Per-element arithmetic that more than one kernel must perform bit-identically: the
// stand-alone elementwise kernels and the matrix-product epilogues that absorb them.
// Floating-point contraction is off inside these functions and every fused multiply-add is written
// out, so the instruction sequence, and with it every rounding, is the same wherever
// these functions are inlined.
#pragma once
#include "device_common.h"

namespace lynx {

// tanh-form GeLU (operator 11) and its derivative.
constexpr float kGeluKappa = 0.7978845608028654f;  // sqrt(2/pi)
constexpr float kGeluC = 0.044715f;

__device__ __forceinline__ float tanh_fast(float x) {
#pragma clang fp contract(off)
  // 1 - 2/(1+e^{2x}); saturates correctly at both ends
  return 1.0f - __fdividef(2.0f, 1.0f + __expf(2.0f * x));
}
// kappa (u + c u^3) = u (kappa + kappa c u^2)
__device__ __forceinline__ float gelu_inner(float u) {
#pragma clang fp contract(off)
  return u * __builtin_fmaf(kGeluKappa * kGeluC, u * u, kGeluKappa);
}
__device__ __forceinline__ float gelu_f(float u) {
#pragma clang fp contract(off)
  const float th = tanh_fast(gelu_inner(u));
  return 0.5f * u * (1.0f + th);
}
__device__ __forceinline__ float gelu_grad_f(float u) {
#pragma clang fp contract(off)
  const float th = tanh_fast(gelu_inner(u));
  const float dinner = __builtin_fmaf(3.0f * kGeluKappa * kGeluC, u * u, kGeluKappa);
  const float sech2 = __builtin_fmaf(-th, th, 1.0f);
  return __builtin_fmaf(0.5f * u * sech2, dinner, 0.5f * (1.0f + th));
}

// du = round(dg gelu'(u)) for 8 elements.
template <typename T>
__device__ __forceinline__ void gelu_bwd8(const float (&dg)[8], const float (&u)[8], float (&du)[8]) {
#pragma clang fp contract(off)
#pragma unroll
  for (int i = 0; i < 8; ++i) du[i] = round_to_storage(dg[i] * gelu_grad_f(u[i]), static_cast<T*>(nullptr));
}

// out = res + keep (in + bias) c for the 8 elements of dropout group `group` (operators
// 8 and 13); `in` is the storage-rounded product of the preceding linear layer.
__device__ __forceinline__ void bias_dropout_add8(const float (&in)[8], const float (&bias)[8],
                                                  const float (&res)[8], const DropoutKey& key,
                                                  uint64_t group, float (&out)[8]) {
#pragma clang fp contract(off)
  float a[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = in[i] + bias[i];
  dropout_apply8(key, group, a);
#pragma unroll
  for (int i = 0; i < 8; ++i) out[i] = res[i] + a[i];
}

}  // namespace lynx
