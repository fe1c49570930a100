// Fused scaled, causally masked softmax with attention dropout (operators 4
// and 5) and its backward.  One wavefront owns one row i of one (batch, head)
// slice: the row's i+1 valid scores live in registers (16-byte vectors, lane l
// holds vectors l, l+64, ...), reductions are wavefront butterflies, and the
// dropout decisions are regenerated from the Philox counter, never read.
// Written rows are zero-filled up to the next multiple of 128 columns so the
// tensor-core attention products can read whole tiles of the diagonal blocks.
#include "attn_math.h"
#include "dropout_host.h"

namespace lynx {
namespace {

constexpr int kRowsPerBlock = 4;  // wavefronts per workgroup
constexpr int kPad = 128;

template <typename T, int NC>
__global__ void __launch_bounds__(kRowsPerBlock* kWave)
softmax_dropout_fwd_kernel(const T* __restrict__ S, T* __restrict__ P, T* __restrict__ Pd, int s,
                           int a, int global_heads, int head0, float scale, DropoutKey key) {
  const int lane = threadIdx.x & (kWave - 1);
  const int i = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (i >= s) return;
  const int bh = blockIdx.y;
  const int bi = bh / a, hd = bh - bi * a;
  const size_t row = (static_cast<size_t>(bh) * s + i) * s;
  const uint64_t gidx = ((static_cast<uint64_t>(bi) * global_heads + head0 + hd) * s + i) *
                        static_cast<uint64_t>(s);
  // (uniform over the wavefront: passes c whose 512 columns lie beyond the row are skipped as a
  // whole; they would contribute exact zeros to the sum and nothing to the output)
  const int nvalid = __builtin_amdgcn_readfirstlane(i + 1);
  const int npad = min(s, (nvalid + kPad - 1) / kPad * kPad);

  float z[NC][8];
  float m = -INFINITY;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    if (c * kWave * 8 >= nvalid) break;
    const int j0 = (lane + c * kWave) * 8;
    if (j0 < nvalid) {
      load8_streaming(S + row + j0, z[c]);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        z[c][k] = (j0 + k < nvalid) ? softmax_logit(z[c][k], scale) : -INFINITY;
        m = fmaxf(m, z[c][k]);
      }
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) z[c][k] = -INFINITY;
    }
  }
  m = wave_max(m);
  // the row sum in its canonical order (attn_math.h): lane l of pass c holds vector l + 64 c,
  // so an aligned block of 64 columns is 8 consecutive lanes
  float a0 = 0.f, a1 = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    if (c * kWave * 8 >= nvalid) break;
#pragma unroll
    for (int k = 0; k < 8; ++k) z[c][k] = softmax_exp(z[c][k], m);
    float t0 = softmax_group4(z[c][0], z[c][1], z[c][2], z[c][3]);
    float t1 = softmax_group4(z[c][4], z[c][5], z[c][6], z[c][7]);
    t0 = group8_sum(t0);
    t1 = group8_sum(t1);
    const float blk = t0 + t1;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      a0 += __int_as_float(__builtin_amdgcn_readlane(__float_as_int(blk), 16 * b));
      a1 += __int_as_float(__builtin_amdgcn_readlane(__float_as_int(blk), 16 * b + 8));
    }
  }
  const float inv = softmax_inverse(a0 + a1);
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    if (c * kWave * 8 >= nvalid) break;
    const int j0 = (lane + c * kWave) * 8;
    if (j0 < npad) {
      float pr[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) pr[k] = softmax_prob<T>(z[c][k], inv);
      if (P != nullptr) {
        // with Pd also written, the next kernel (Pd V) reads Pd; P waits for backward
        if (Pd != nullptr) store8_streaming(P + row + j0, pr);
        else store8(P + row + j0, pr);
      }
      if (Pd != nullptr) {
        // entries beyond the diagonal are exactly 0 already; the zero padding needs no draw
        if (j0 < nvalid) dropout_apply8(key, (gidx + j0) >> 3, pr);
        store8(Pd + row + j0, pr);
      }
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(kRowsPerBlock* kWave)
attn_dropout_fwd_kernel(const T* __restrict__ P, T* __restrict__ Pd, int s, int a, int global_heads,
                        int head0, DropoutKey key) {
  const int lane = threadIdx.x & (kWave - 1);
  const int i = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (i >= s) return;
  const int bh = blockIdx.y;
  const int bi = bh / a, hd = bh - bi * a;
  const size_t row = (static_cast<size_t>(bh) * s + i) * s;
  const uint64_t gidx = ((static_cast<uint64_t>(bi) * global_heads + head0 + hd) * s + i) *
                        static_cast<uint64_t>(s);
  const int nvalid = i + 1;
  const int npad = min(s, (nvalid + kPad - 1) / kPad * kPad);
  for (int j0 = lane * 8; j0 < npad; j0 += kWave * 8) {
    float pr[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (j0 < nvalid) {
      load8(P + row + j0, pr);
#pragma unroll
      for (int k = 0; k < 8; ++k) pr[k] = (j0 + k < nvalid) ? pr[k] : 0.0f;
      dropout_apply8(key, (gidx + j0) >> 3, pr);
    }
    store8(Pd + row + j0, pr);
  }
}

template <typename T, int NC>
__global__ void __launch_bounds__(kRowsPerBlock* kWave)
softmax_dropout_bwd_kernel(const T* dPd, const T* __restrict__ P, T* dS,  // dS may alias dPd
                           int s, int a, int global_heads, int head0, float scale, DropoutKey key) {
  const int lane = threadIdx.x & (kWave - 1);
  const int i = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (i >= s) return;
  const int bh = blockIdx.y;
  const int bi = bh / a, hd = bh - bi * a;
  const size_t row = (static_cast<size_t>(bh) * s + i) * s;
  const uint64_t gidx = ((static_cast<uint64_t>(bi) * global_heads + head0 + hd) * s + i) *
                        static_cast<uint64_t>(s);
  const int nvalid = i + 1;
  const int npad = min(s, (nvalid + kPad - 1) / kPad * kPad);

  float dp[NC][8], p[NC][8];
  float dot = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (lane + c * kWave) * 8;
    if (j0 < nvalid) {
      load8(dPd + row + j0, dp[c]);
      load8(P + row + j0, p[c]);
#pragma unroll
      for (int k = 0; k < 8; ++k) {  // beyond the diagonal dPd holds whatever the product left
        dp[c][k] = (j0 + k < nvalid) ? dp[c][k] : 0.0f;
        p[c][k] = (j0 + k < nvalid) ? p[c][k] : 0.0f;
      }
      dropout_apply8(key, (gidx + j0) >> 3, dp[c]);
#pragma unroll
      for (int k = 0; k < 8; ++k) dot += dp[c][k] * p[c][k];
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) { dp[c][k] = 0.f; p[c][k] = 0.f; }
    }
  }
  dot = wave_sum(dot);
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (lane + c * kWave) * 8;
    if (j0 < npad) {
      float ds[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) ds[k] = scale * (p[c][k] * (dp[c][k] - dot));
      store8(dS + row + j0, ds);
    }
  }
}

// Row dot products over the head dimension: 16 lanes per (token, head) pair.
template <typename T>
__global__ void __launch_bounds__(256)
attn_rowdot_kernel(const T* __restrict__ x, const T* __restrict__ y, float* __restrict__ out, int a, int s,
                   int d, long long ld, long long pairs) {
  const long long q = static_cast<long long>(blockIdx.x) * 16 + (threadIdx.x >> 4);
  const int l = threadIdx.x & 15;
  float acc = 0.f;
  long long t = 0;
  int hd = 0;
  if (q < pairs) {
    t = q / a;
    hd = static_cast<int>(q - t * a);
    const size_t base = static_cast<size_t>(t) * ld + static_cast<size_t>(hd) * d;
    for (int v = l; v * 8 < d; v += 16) {
      float xv[8], yv[8];
      load8(x + base + v * 8, xv);            // dC: the kernels that follow read it again
      load8_streaming(y + base + v * 8, yv);  // C: its last use
#pragma unroll
      for (int k = 0; k < 8; ++k) acc += xv[k] * yv[k];
    }
  }
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 16);
  if (q < pairs && l == 0) {
    const long long bi = t / s, i = t - bi * s;
    out[(bi * a + hd) * s + i] = acc;
  }
}

// registers hold ceil(s / 512) vectors per lane
#define LYNX_DISPATCH_NC(s, CALL)            \
  if ((s) <= 512) { CALL(1); }               \
  else if ((s) <= 1024) { CALL(2); }         \
  else if ((s) <= 2048) { CALL(4); }         \
  else if ((s) <= 4096) { CALL(8); }         \
  else { CALL(16); }

}  // namespace

hipError_t softmax_dropout_fwd(int dtype, const void* S, void* P, void* Pd, AttnShape sh, float scale,
                               DropoutParams dp, hipStream_t st) {
  if (sh.s > 8192) return hipErrorInvalidValue;
  const dim3 grid((sh.s + kRowsPerBlock - 1) / kRowsPerBlock, sh.b * sh.a);
  const dim3 block(kRowsPerBlock * kWave);
  const DropoutKey key = make_dropout_key(dp, 0);
#define CALL(NC)                                                                                  \
  if (dtype == 1)                                                                                 \
    hipLaunchKernelGGL((softmax_dropout_fwd_kernel<bf16_t, NC>), grid, block, 0, st,              \
                       static_cast<const bf16_t*>(S), static_cast<bf16_t*>(P),                    \
                       static_cast<bf16_t*>(Pd), sh.s, sh.a, sh.global_heads, sh.head0, scale,    \
                       key);                                                                      \
  else                                                                                            \
    hipLaunchKernelGGL((softmax_dropout_fwd_kernel<float, NC>), grid, block, 0, st,               \
                       static_cast<const float*>(S), static_cast<float*>(P),                      \
                       static_cast<float*>(Pd), sh.s, sh.a, sh.global_heads, sh.head0, scale, key)
  LYNX_DISPATCH_NC(sh.s, CALL)
#undef CALL
  return hipGetLastError();
}

hipError_t attn_dropout_fwd(int dtype, const void* P, void* Pd, AttnShape sh, DropoutParams dp,
                            hipStream_t st) {
  const dim3 grid((sh.s + kRowsPerBlock - 1) / kRowsPerBlock, sh.b * sh.a);
  const dim3 block(kRowsPerBlock * kWave);
  const DropoutKey key = make_dropout_key(dp, 0);
  if (dtype == 1)
    hipLaunchKernelGGL((attn_dropout_fwd_kernel<bf16_t>), grid, block, 0, st,
                       static_cast<const bf16_t*>(P), static_cast<bf16_t*>(Pd), sh.s, sh.a,
                       sh.global_heads, sh.head0, key);
  else
    hipLaunchKernelGGL((attn_dropout_fwd_kernel<float>), grid, block, 0, st,
                       static_cast<const float*>(P), static_cast<float*>(Pd), sh.s, sh.a,
                       sh.global_heads, sh.head0, key);
  return hipGetLastError();
}

hipError_t attn_rowdot(int dtype, const void* x, const void* y, float* out, int b, int a, int s, int d,
                       long long ld, hipStream_t st) {
  if (d % 8 || ld % 8) return hipErrorInvalidValue;
  const long long pairs = static_cast<long long>(b) * s * a;
  const dim3 grid(static_cast<unsigned>((pairs + 15) / 16));
  if (dtype == 1)
    hipLaunchKernelGGL((attn_rowdot_kernel<bf16_t>), grid, dim3(256), 0, st, static_cast<const bf16_t*>(x),
                       static_cast<const bf16_t*>(y), out, a, s, d, ld, pairs);
  else
    hipLaunchKernelGGL((attn_rowdot_kernel<float>), grid, dim3(256), 0, st, static_cast<const float*>(x),
                       static_cast<const float*>(y), out, a, s, d, ld, pairs);
  return hipGetLastError();
}

hipError_t softmax_dropout_bwd(int dtype, const void* dPd, const void* P, void* dS, AttnShape sh,
                               float scale, DropoutParams dp, hipStream_t st) {
  if (sh.s > 8192) return hipErrorInvalidValue;
  const dim3 grid((sh.s + kRowsPerBlock - 1) / kRowsPerBlock, sh.b * sh.a);
  const dim3 block(kRowsPerBlock * kWave);
  const DropoutKey key = make_dropout_key(dp, 0);
#define CALL(NC)                                                                                  \
  if (dtype == 1)                                                                                 \
    hipLaunchKernelGGL((softmax_dropout_bwd_kernel<bf16_t, NC>), grid, block, 0, st,              \
                       static_cast<const bf16_t*>(dPd), static_cast<const bf16_t*>(P),            \
                       static_cast<bf16_t*>(dS), sh.s, sh.a, sh.global_heads, sh.head0, scale,    \
                       key);                                                                      \
  else                                                                                            \
    hipLaunchKernelGGL((softmax_dropout_bwd_kernel<float, NC>), grid, block, 0, st,               \
                       static_cast<const float*>(dPd), static_cast<const float*>(P),              \
                       static_cast<float*>(dS), sh.s, sh.a, sh.global_heads, sh.head0, scale, key)
  LYNX_DISPATCH_NC(sh.s, CALL)
#undef CALL
  return hipGetLastError();
}

}  // namespace lynx
