// Arithmetic of the attention softmax (operators 4 and 5) that more than one kernel must
// perform bit-identically: the row kernel of softmax.hip and the fused attention kernels
// that never store S, P or Pd.  A regenerated or fused result may not differ from the
// forward's in a single bit, so everything whose rounding depends on evaluation order is
// fixed here: floating-point contraction is off, and the row sum of the exponentials has
// one canonical order that both a row-per-wavefront layout and a matrix-core accumulator
// layout can follow cheaply.
//
// Canonical row sum.  Columns are taken in vectors of 8 (the 16-byte vector of bf16
// storage).  Of vector v, g_h(v) = (e[4h] + e[4h+1]) + (e[4h+2] + e[4h+3]) for h = 0, 1.
// Over the 8 vectors of an aligned block of 64 columns,
//   T_h = ((g_h(v0) + g_h(v1)) + (g_h(v2) + g_h(v3))) + ((g_h(v4) + g_h(v5)) + (g_h(v6) + g_h(v7)))
// and the block's sum is T_0 + T_1.  Blocks of 64 columns alternate between two running
// sums, A_w += block(2 t + w) for t = 0, 1, ... in ascending order (w = 0, 1: the first and
// second half of every 128 columns), and the row sum is A_0 + A_1.  Columns beyond the
// causal limit contribute exact zeros, so how many blocks a kernel visits is immaterial.
#pragma once
#include "device_common.h"

namespace lynx {

// z = scale * S, from the storage-rounded score.
__device__ __forceinline__ float softmax_logit(float s_stored, float scale) {
#pragma clang fp contract(off)
  return s_stored * scale;
}
// e = exp(z - m); exp(-inf) = 0 for excluded entries.
__device__ __forceinline__ float softmax_exp(float z, float m) {
#pragma clang fp contract(off)
  return __expf(z - m);
}
__device__ __forceinline__ float softmax_group4(float a, float b, float c, float d) {
#pragma clang fp contract(off)
  return (a + b) + (c + d);
}
__device__ __forceinline__ float softmax_tree8(float x0, float x1, float x2, float x3, float x4, float x5,
                                               float x6, float x7) {
#pragma clang fp contract(off)
  return ((x0 + x1) + (x2 + x3)) + ((x4 + x5) + (x6 + x7));
}
// P = round(e * inv), inv = 1 / row sum.
__device__ __forceinline__ float softmax_inverse(float sum) {
#pragma clang fp contract(off)
  return 1.0f / sum;
}
template <typename T>
__device__ __forceinline__ float softmax_prob(float e, float inv) {
#pragma clang fp contract(off)
  return round_to_storage(e * inv, static_cast<T*>(nullptr));
}
// dS = scale P (dP - dot) (B4 with the scale of B3 folded in), dP already masked and scaled.
__device__ __forceinline__ float softmax_bwd(float p, float dp, float dot, float scale) {
#pragma clang fp contract(off)
  return scale * (p * (dp - dot));
}

}  // namespace lynx
