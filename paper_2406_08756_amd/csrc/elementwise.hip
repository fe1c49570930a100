// HBM-bound elementwise kernels: GeLU forward/backward, bias+dropout+residual,
// dropout backward, column sums (bias gradients) and the dropout-mask dump.
// Every thread moves 16-byte vectors of 8 elements; consecutive lanes touch
// consecutive vectors.  Column sums are two fixed-order stages (per row-block
// partials, then a serial sum over row-blocks), so results are deterministic.
#include "dropout_host.h"
#include "reduce_partials.h"

namespace lynx {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = 64;  // rows folded into one column-sum partial

// tanh-form GeLU (operator 11) and its derivative.
constexpr float kKappa = 0.7978845608028654f;  // sqrt(2/pi)
constexpr float kGeluC = 0.044715f;

__device__ __forceinline__ float tanh_fast(float x) {
  // 1 - 2/(1+e^{2x}); saturates correctly at both ends
  return 1.0f - __fdividef(2.0f, 1.0f + __expf(2.0f * x));
}
__device__ __forceinline__ float gelu_f(float u) {
  const float th = tanh_fast(kKappa * (u + kGeluC * u * u * u));
  return 0.5f * u * (1.0f + th);
}
__device__ __forceinline__ float gelu_grad_f(float u) {
  const float th = tanh_fast(kKappa * (u + kGeluC * u * u * u));
  return 0.5f * (1.0f + th) + 0.5f * u * (1.0f - th * th) * kKappa * (1.0f + 3.0f * kGeluC * u * u);
}

template <typename T>
__global__ void __launch_bounds__(kThreads) gelu_fwd_kernel(const T* __restrict__ u,
                                                            T* __restrict__ g, size_t nvec) {
  const size_t v = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (v >= nvec) return;
  float x[8];
  load8(u + v * 8, x);
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = gelu_f(x[i]);
  store8(g + v * 8, x);
}

// ---- per-element functors used with the column-sum frame ------------------
template <typename T>
struct GeluBwdOp {
  const T* dg; const T* u; T* du;
  __device__ __forceinline__ void operator()(size_t off, size_t, float (&out)[8]) const {
    float a[8], b[8];
    load8(dg + off, a);
    load8(u + off, b);
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = round_to_storage(a[i] * gelu_grad_f(b[i]), du);
    store8(du + off, out);
  }
};

template <typename T>
struct DropoutBwdOp {
  const T* dout; T* din; DropoutKey key;
  __device__ __forceinline__ void operator()(size_t off, size_t group, float (&out)[8]) const {
    float a[8];
    load8(dout + off, a);
    const uint32_t keep = dropout_keep8(key, group);
#pragma unroll
    for (int i = 0; i < 8; ++i)
      out[i] = round_to_storage(((keep >> i) & 1u) ? a[i] * key.scale : 0.0f, din);
    store8(din + off, out);
  }
};

template <typename T>
struct IdentityOp {
  const T* x;
  __device__ __forceinline__ void operator()(size_t off, size_t, float (&out)[8]) const {
    load8(x + off, out);
  }
};

// Frame: block (bx, by) covers vectors [bx*256, +256) of rows [by*64, +64);
// thread applies op to its vector in each row and accumulates the 8 columns.
template <typename Op>
__global__ void __launch_bounds__(kThreads) rows_colsum_kernel(Op op, int rows, int cols,
                                                               float* __restrict__ partial) {
  const int vec = blockIdx.x * kThreads + threadIdx.x;
  const int nvec = cols >> 3;
  if (vec >= nvec) return;
  const int r0 = blockIdx.y * kRowsPerBlock;
  const int r1 = min(rows, r0 + kRowsPerBlock);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int r = r0; r < r1; ++r) {
    const size_t off = static_cast<size_t>(r) * cols + static_cast<size_t>(vec) * 8;
    float v[8];
    op(off, off >> 3, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += v[i];
  }
  float* p = partial + static_cast<size_t>(blockIdx.y) * cols + static_cast<size_t>(vec) * 8;
  store8(p, acc);
}

template <typename T, typename Op>
hipError_t launch_rows_colsum(Op op, T* dbias, float* scratch, int rows, int cols, hipStream_t st) {
  const int nvec = cols / 8;
  const int nrb = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
  dim3 grid((nvec + kThreads - 1) / kThreads, nrb);
  hipLaunchKernelGGL((rows_colsum_kernel<Op>), grid, dim3(kThreads), 0, st, op, rows, cols, scratch);
  launch_reduce_partials<T>(scratch, dbias, nullptr, nullptr, nrb, cols, st);
  return hipGetLastError();
}

template <typename T>
__global__ void __launch_bounds__(kThreads)
bias_dropout_add_kernel(const T* __restrict__ in, const T* __restrict__ bias,
                        const T* __restrict__ res, T* __restrict__ out, size_t nvec, int cols,
                        DropoutKey key) {
  const size_t v = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (v >= nvec) return;
  const size_t off = v * 8;
  const int c = static_cast<int>(off % static_cast<size_t>(cols));
  float a[8], b[8], r[8];
  load8(in + off, a);
  load8(bias + c, b);
  load8(res + off, r);
  const uint32_t keep = dropout_keep8(key, v);
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] += ((keep >> i) & 1u) ? (a[i] + b[i]) * key.scale : 0.0f;
  store8(out + off, r);
}

__global__ void __launch_bounds__(kThreads)
mask_bytes_kernel(uint8_t* __restrict__ out, size_t ngroups, uint64_t group0, DropoutKey key) {
  const size_t g = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (g >= ngroups) return;
  const uint32_t keep = dropout_keep8(key, group0 + g);
  uint2 w;
  w.x = (keep & 1u) | ((keep & 2u) << 7) | ((keep & 4u) << 14) | ((keep & 8u) << 21);
  const uint32_t k2 = keep >> 4;
  w.y = (k2 & 1u) | ((k2 & 2u) << 7) | ((k2 & 4u) << 14) | ((k2 & 8u) << 21);
  *reinterpret_cast<uint2*>(out + g * 8) = w;
}

}  // namespace

size_t colsum_scratch_bytes(int rows, int cols) {
  const size_t nrb = (static_cast<size_t>(rows) + kRowsPerBlock - 1) / kRowsPerBlock;
  return nrb * static_cast<size_t>(cols) * sizeof(float);
}

hipError_t gelu_fwd(int dtype, const void* u, void* g, size_t n, hipStream_t st) {
  const size_t nvec = n / 8;
  const dim3 grid(static_cast<unsigned>((nvec + kThreads - 1) / kThreads));
  if (dtype == 1)
    hipLaunchKernelGGL((gelu_fwd_kernel<bf16_t>), grid, dim3(kThreads), 0, st,
                       static_cast<const bf16_t*>(u), static_cast<bf16_t*>(g), nvec);
  else
    hipLaunchKernelGGL((gelu_fwd_kernel<float>), grid, dim3(kThreads), 0, st,
                       static_cast<const float*>(u), static_cast<float*>(g), nvec);
  return hipGetLastError();
}

hipError_t gelu_bwd(int dtype, const void* dg, const void* u, void* du, void* dbias, float* scratch,
                    int rows, int cols, hipStream_t st) {
  if (dtype == 1) {
    GeluBwdOp<bf16_t> op{static_cast<const bf16_t*>(dg), static_cast<const bf16_t*>(u),
                         static_cast<bf16_t*>(du)};
    return launch_rows_colsum(op, static_cast<bf16_t*>(dbias), scratch, rows, cols, st);
  }
  GeluBwdOp<float> op{static_cast<const float*>(dg), static_cast<const float*>(u),
                      static_cast<float*>(du)};
  return launch_rows_colsum(op, static_cast<float*>(dbias), scratch, rows, cols, st);
}

hipError_t bias_dropout_add_fwd(int dtype, const void* in, const void* bias, const void* res,
                                void* out, int rows, int cols, int site, DropoutParams dp,
                                hipStream_t st) {
  const size_t nvec = static_cast<size_t>(rows) * cols / 8;
  const dim3 grid(static_cast<unsigned>((nvec + kThreads - 1) / kThreads));
  const DropoutKey key = make_dropout_key(dp, site);
  if (dtype == 1)
    hipLaunchKernelGGL((bias_dropout_add_kernel<bf16_t>), grid, dim3(kThreads), 0, st,
                       static_cast<const bf16_t*>(in), static_cast<const bf16_t*>(bias),
                       static_cast<const bf16_t*>(res), static_cast<bf16_t*>(out), nvec, cols, key);
  else
    hipLaunchKernelGGL((bias_dropout_add_kernel<float>), grid, dim3(kThreads), 0, st,
                       static_cast<const float*>(in), static_cast<const float*>(bias),
                       static_cast<const float*>(res), static_cast<float*>(out), nvec, cols, key);
  return hipGetLastError();
}

hipError_t dropout_bwd(int dtype, const void* dout, void* din, void* dbias, float* scratch, int rows,
                       int cols, int site, DropoutParams dp, hipStream_t st) {
  const DropoutKey key = make_dropout_key(dp, site);
  if (dtype == 1) {
    DropoutBwdOp<bf16_t> op{static_cast<const bf16_t*>(dout), static_cast<bf16_t*>(din), key};
    return launch_rows_colsum(op, static_cast<bf16_t*>(dbias), scratch, rows, cols, st);
  }
  DropoutBwdOp<float> op{static_cast<const float*>(dout), static_cast<float*>(din), key};
  return launch_rows_colsum(op, static_cast<float*>(dbias), scratch, rows, cols, st);
}

hipError_t column_sum(int dtype, const void* x, void* dbias, float* scratch, int rows, int cols,
                      hipStream_t st) {
  if (dtype == 1) {
    IdentityOp<bf16_t> op{static_cast<const bf16_t*>(x)};
    return launch_rows_colsum(op, static_cast<bf16_t*>(dbias), scratch, rows, cols, st);
  }
  IdentityOp<float> op{static_cast<const float*>(x)};
  return launch_rows_colsum(op, static_cast<float*>(dbias), scratch, rows, cols, st);
}

hipError_t dropout_mask_hidden(uint8_t* out, size_t n, int site, DropoutParams dp, hipStream_t st) {
  const size_t ng = n / 8;
  hipLaunchKernelGGL(mask_bytes_kernel, dim3(static_cast<unsigned>((ng + kThreads - 1) / kThreads)),
                     dim3(kThreads), 0, st, out, ng, static_cast<uint64_t>(0), make_dropout_key(dp, site));
  return hipGetLastError();
}

hipError_t dropout_mask_attn(uint8_t* out, AttnShape sh, DropoutParams dp, hipStream_t st) {
  // one launch per (bi, hd) slice: slices are contiguous in the output but
  // strided in the global index space when the shard holds a subset of heads
  const size_t slice = static_cast<size_t>(sh.s) * sh.s;
  const size_t ng = slice / 8;
  const DropoutKey key = make_dropout_key(dp, 0);
  for (int bi = 0; bi < sh.b; ++bi)
    for (int hd = 0; hd < sh.a; ++hd) {
      const uint64_t first = (static_cast<uint64_t>(bi) * sh.global_heads + sh.head0 + hd) * slice;
      hipLaunchKernelGGL(mask_bytes_kernel,
                         dim3(static_cast<unsigned>((ng + kThreads - 1) / kThreads)), dim3(kThreads),
                         0, st, out + (static_cast<size_t>(bi) * sh.a + hd) * slice, ng, first / 8,
                         key);
    }
  return hipGetLastError();
}

}  // namespace lynx
