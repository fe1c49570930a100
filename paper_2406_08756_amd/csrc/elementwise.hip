// HBM-bound elementwise kernels: GeLU forward/backward, bias+dropout+residual,
// dropout backward, column sums (bias gradients) and the dropout-mask dump.
// Every thread moves 16-byte vectors of 8 elements; consecutive lanes touch
// consecutive vectors.  Column sums are two fixed-order stages (per row-block
// partials, then a serial sum over row-blocks), so results are deterministic.
#include "dropout_host.h"
#include "pointwise_math.h"
#include "reduce_partials.h"

namespace lynx {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerBlock = 32;  // rows folded into one column-sum partial

template <typename T>
__global__ void __launch_bounds__(kThreads) gelu_fwd_kernel(const T* __restrict__ u,
                                                            T* __restrict__ g, size_t nvec) {
  const size_t v = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (v >= nvec) return;
  float x[8];
  load8_streaming(u + v * 8, x);
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = gelu_f(x[i]);
  store8(g + v * 8, x);
}

// ---- per-element functors used with the column-sum frame ------------------
// apply(a, b, group, out): a, b = 8 elements of the one or two inputs, group =
// flat element index / 8; out = the 8 results, already rounded to storage.
template <typename T>
struct GeluBwdOp {  // du = dg * gelu'(u)
  static constexpr int kInputs = 2;
  static constexpr bool kStores = true;
  __device__ __forceinline__ void apply(const float (&a)[8], const float (&b)[8], size_t,
                                        float (&out)[8]) const {
    gelu_bwd8<T>(a, b, out);
  }
};

template <typename T>
struct DropoutBwdOp {  // din = keep * dout / (1 - p)
  static constexpr int kInputs = 1;
  static constexpr bool kStores = true;
  DropoutKey key;
  __device__ __forceinline__ void apply(const float (&a)[8], const float (&)[8], size_t group,
                                        float (&out)[8]) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = a[i];
    dropout_apply8(key, group, out);
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = round_to_storage(out[i], static_cast<T*>(nullptr));
  }
};

template <typename T>
struct IdentityOp {
  static constexpr int kInputs = 1;
  static constexpr bool kStores = false;
  __device__ __forceinline__ void apply(const float (&a)[8], const float (&)[8], size_t,
                                        float (&out)[8]) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = a[i];
  }
};

// Frame: a workgroup owns a tile of kRowsPerBlock rows x 64 vectors (512 columns):
// wavefront w takes rows w, w + 4, ... of the tile, lane l the l-th vector, so every
// wavefront access is 1 KB contiguous and a thread's column stays fixed.  All of a
// thread's loads are issued before its first store; the four wavefronts' column sums
// are added in a fixed order through LDS.  Many small workgroups keep enough
// wavefronts resident to overlap the Philox / GeLU arithmetic with the memory traffic.
constexpr int kRowsPerThread = kRowsPerBlock / (kThreads / kWave);
template <typename T, typename Op>
__global__ void __launch_bounds__(kThreads)
rows_colsum_kernel(Op op, const T* __restrict__ in0, const T* __restrict__ in1, T* __restrict__ outp,
                   int rows, int cols, float* __restrict__ partial) {
  __shared__ float sm[kThreads / kWave][kWave][8];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
  const int vec = blockIdx.x * kWave + lane;
  const bool active = vec < (cols >> 3);
  const int r0 = blockIdx.y * kRowsPerBlock + w;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (active) {
    Raw8<T> ra[kRowsPerThread], rb[Op::kInputs == 2 ? kRowsPerThread : 1];
#pragma unroll
    for (int k = 0; k < kRowsPerThread; ++k) {
      const int r = r0 + k * (kThreads / kWave);
      if (r < rows) {
        const size_t off = static_cast<size_t>(r) * cols + static_cast<size_t>(vec) * 8;
        load_raw_streaming(in0 + off, ra[k]);
        if (Op::kInputs == 2) load_raw_streaming(in1 + off, rb[Op::kInputs == 2 ? k : 0]);
      }
    }
#pragma unroll
    for (int k = 0; k < kRowsPerThread; ++k) {
      const int r = r0 + k * (kThreads / kWave);
      if (r < rows) {
        const size_t off = static_cast<size_t>(r) * cols + static_cast<size_t>(vec) * 8;
        float a[8], b[8] = {}, v[8];
        unpack(ra[k], a);
        if (Op::kInputs == 2) unpack(rb[Op::kInputs == 2 ? k : 0], b);
        op.apply(a, b, off >> 3, v);
        if (Op::kStores) store8(outp + off, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] += v[i];
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) sm[w][lane][i] = acc[i];
  __syncthreads();
  if (w == 0 && active) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = (sm[0][lane][i] + sm[1][lane][i]) + (sm[2][lane][i] + sm[3][lane][i]);
    store8(partial + static_cast<size_t>(blockIdx.y) * cols + static_cast<size_t>(vec) * 8, acc);
  }
}

template <typename T, typename Op>
hipError_t launch_rows_colsum(Op op, const T* in0, const T* in1, T* outp, T* dbias, float* scratch,
                              int rows, int cols, hipStream_t st) {
  const int nvec = cols / 8;
  const int nrb = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
  const dim3 grid((nvec + kWave - 1) / kWave, nrb);
  hipLaunchKernelGGL((rows_colsum_kernel<T, Op>), grid, dim3(kThreads), 0, st, op, in0, in1, outp,
                     rows, cols, scratch);
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
  float o[8];
  bias_dropout_add8(a, b, r, key, v, o);
  store8(out + off, o);
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
    return launch_rows_colsum(GeluBwdOp<bf16_t>{}, static_cast<const bf16_t*>(dg),
                              static_cast<const bf16_t*>(u), static_cast<bf16_t*>(du),
                              static_cast<bf16_t*>(dbias), scratch, rows, cols, st);
  }
  return launch_rows_colsum(GeluBwdOp<float>{}, static_cast<const float*>(dg),
                            static_cast<const float*>(u), static_cast<float*>(du),
                            static_cast<float*>(dbias), scratch, rows, cols, st);
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
    return launch_rows_colsum(DropoutBwdOp<bf16_t>{key}, static_cast<const bf16_t*>(dout),
                              static_cast<const bf16_t*>(nullptr), static_cast<bf16_t*>(din),
                              static_cast<bf16_t*>(dbias), scratch, rows, cols, st);
  }
  return launch_rows_colsum(DropoutBwdOp<float>{key}, static_cast<const float*>(dout),
                            static_cast<const float*>(nullptr), static_cast<float*>(din),
                            static_cast<float*>(dbias), scratch, rows, cols, st);
}

hipError_t column_sum(int dtype, const void* x, void* dbias, float* scratch, int rows, int cols,
                      hipStream_t st) {
  if (dtype == 1) {
    return launch_rows_colsum(IdentityOp<bf16_t>{}, static_cast<const bf16_t*>(x),
                              static_cast<const bf16_t*>(nullptr), static_cast<bf16_t*>(nullptr),
                              static_cast<bf16_t*>(dbias), scratch, rows, cols, st);
  }
  return launch_rows_colsum(IdentityOp<float>{}, static_cast<const float*>(x),
                            static_cast<const float*>(nullptr), static_cast<float*>(nullptr),
                            static_cast<float*>(dbias), scratch, rows, cols, st);
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
