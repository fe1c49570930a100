// LayerNorm forward (operators 1 and 9) and backward.  Forward: one workgroup
// per token row, the row held in registers (a few 16-byte vectors per thread),
// two-pass mean / variance in fp32, statistics written for backward.  Backward: one workgroup of four
// wavefronts per row stream; each lane owns fixed columns so the per-column
// sums for dgamma / dbeta accumulate in registers over the rows the workgroup
// visits, and are then reduced over workgroups in a second fixed-order stage.
#include "dropout_host.h"
#include "reduce_partials.h"

namespace lynx {
namespace {

constexpr int kBwdThreads = 256;
constexpr int kBwdMaxBlocks = 512;
constexpr int kFwdStreamBlocks = 1024;

// Sum over the BS threads of a workgroup, every thread gets the total; `slot` is this
// call's own LDS row, so two calls need no barrier between them.  Fixed combination order.
template <int BS>
__device__ __forceinline__ float block_sum(float v, float* slot) {
  v = wave_sum(v);
  if (BS == kWave) return v;
  if ((threadIdx.x & (kWave - 1)) == 0) slot[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = slot[0];
#pragma unroll
  for (int w = 1; w < BS / kWave; ++w) t += slot[w];
  return t;
}

// One workgroup of BS threads per row, NC 16-byte vectors per thread: few loads per
// thread and many rows in flight stream from HBM markedly faster than a whole row per
// wavefront.  Workgroup b takes row (b % 8) (rows / 8) + b / 8, so that each XCD (which
// receives every eighth workgroup) walks its own contiguous eighth of the tensor.
template <typename T, int BS, int NC>
__global__ void __launch_bounds__(BS)
layernorm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                     const T* __restrict__ beta, T* __restrict__ y, float* __restrict__ mean,
                     float* __restrict__ rstd, int rows, int cols, float eps) {
  __shared__ float red[2][BS / kWave];
  int r = blockIdx.x;
  if ((rows & 7) == 0) r = (r & 7) * (rows >> 3) + (r >> 3);
  const size_t base = static_cast<size_t>(r) * cols;
  // Threads past the end of the row load column 0 again and count for nothing, so the
  // loads and the arithmetic are straight-line code; only the stores are predicated.
  float v[NC][8];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (threadIdx.x + c * BS) * 8;
    const bool on = j0 < cols;
    load8(x + base + (on ? j0 : 0), v[c]);
    const float w = on ? 1.0f : 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) sum += w * v[c][k];
  }
  const float inv_n = 1.0f / static_cast<float>(cols);
  const float mu = block_sum<BS>(sum, red[0]) * inv_n;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const float w = (threadIdx.x + c * BS) * 8 < cols ? 1.0f : 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      v[c][k] -= mu;
      sq += w * (v[c][k] * v[c][k]);
    }
  }
  const float rs = rsqrtf(block_sum<BS>(sq, red[1]) * inv_n + eps);
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (threadIdx.x + c * BS) * 8;
    if (j0 < cols) {
      float g[8], b[8];
      load8(gamma + j0, g);
      load8(beta + j0, b);
#pragma unroll
      for (int k = 0; k < 8; ++k) v[c][k] = g[k] * (v[c][k] * rs) + b[k];
      store8(y + base + j0, v[c]);
    }
  }
  if (threadIdx.x == 0) {
    mean[r] = mu;
    rstd[r] = rs;
  }
}

// The same operator for many rows: a resident set of workgroups, each walking rows of its
// XCD's eighth of the tensor, with the next row's vectors requested before the current
// row is reduced and stored, so a workgroup always has a row in flight (a second row ahead
// and other workgroup counts from 512 to 4096 measure the same or worse).
template <typename T, int BS, int NC>
__global__ void __launch_bounds__(BS)
layernorm_fwd_stream_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                            const T* __restrict__ beta, T* __restrict__ y, float* __restrict__ mean,
                            float* __restrict__ rstd, int rows, int cols, float eps) {
  __shared__ float red[2][BS / kWave];
  const int per_xcd = rows >> 3, groups = gridDim.x >> 3;  // rows % 8 == 0, gridDim.x % 8 == 0
  const int first = blockIdx.x >> 3, xcd_row0 = (blockIdx.x & 7) * per_xcd;
  const float inv_n = 1.0f / static_cast<float>(cols);
  bool on[NC];
  int j0[NC];
  Raw8<T> graw[NC], braw[NC], cur[NC], nxt[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    j0[c] = (threadIdx.x + c * BS) * 8;
    on[c] = j0[c] < cols;
    if (!on[c]) j0[c] = 0;  // counts for nothing, stores nothing
    load_raw(gamma + j0[c], graw[c]);
    load_raw(beta + j0[c], braw[c]);
  }
  if (first < per_xcd) {
    const size_t base = static_cast<size_t>(xcd_row0 + first) * cols;
#pragma unroll
    for (int c = 0; c < NC; ++c) load_raw_streaming(x + base + j0[c], cur[c]);
  }
  for (int i = first; i < per_xcd; i += groups) {
    const int r = xcd_row0 + i;
    const bool more = i + groups < per_xcd;
    if (more) {
      const size_t nbase = static_cast<size_t>(r + groups) * cols;
#pragma unroll
      for (int c = 0; c < NC; ++c) load_raw_streaming(x + nbase + j0[c], nxt[c]);
    }
    float v[NC][8];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      unpack(cur[c], v[c]);
      const float w = on[c] ? 1.0f : 0.0f;
#pragma unroll
      for (int k = 0; k < 8; ++k) sum += w * v[c][k];
    }
    const float mu = block_sum<BS>(sum, red[0]) * inv_n;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const float w = on[c] ? 1.0f : 0.0f;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        v[c][k] -= mu;
        sq += w * (v[c][k] * v[c][k]);
      }
    }
    const float rs = rsqrtf(block_sum<BS>(sq, red[1]) * inv_n + eps);
    const size_t base = static_cast<size_t>(r) * cols;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (on[c]) {
        float g[8], b[8];
        unpack(graw[c], g);
        unpack(braw[c], b);
#pragma unroll
        for (int k = 0; k < 8; ++k) v[c][k] = g[k] * (v[c][k] * rs) + b[k];
        store8(y + base + j0[c], v[c]);
      }
    }
    if (threadIdx.x == 0) {
      mean[r] = mu;
      rstd[r] = rs;
    }
    if (more) {
#pragma unroll
      for (int c = 0; c < NC; ++c) cur[c] = nxt[c];
    }
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

// RPI rows per iteration: all loads of those rows (dy, x, residual gradient) are issued
// before the reductions.  Loaded vectors stay in storage format (half the registers for
// bf16) and are unpacked where used, once for the sums and once for the output, which
// buys the occupancy that hides the load latency.
//
// DROP: the row gradient just formed is also the output gradient of a bias + dropout +
// residual operator (dx_out = d(X + keep (O + b) c)): the same pass writes
// dO = keep c round(dx_out) to `dropped` and accumulates its column sums (the bias
// gradient), which saves the separate pass that would read dx_out again.
template <typename T, int NC, int RPI, bool DROP>
__global__ void __launch_bounds__(kBwdThreads)
layernorm_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                     const float* __restrict__ mean, const float* __restrict__ rstd,
                     const T* __restrict__ gamma, const T* dres, T* dx_out,
                     float* __restrict__ part_dg, float* __restrict__ part_db, int rows, int cols,
                     T* __restrict__ dropped, float* __restrict__ part_dbias, DropoutKey key) {
  __shared__ float smem[16];
  Raw8<T> graw[NC];
  float adg[NC][8], adb[NC][8], adbias[DROP ? NC : 1][8];
#pragma unroll
  for (int c = 0; c < (DROP ? NC : 1); ++c)
#pragma unroll
    for (int k = 0; k < 8; ++k) adbias[c][k] = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int j0 = (threadIdx.x + c * kBwdThreads) * 8;
    if (j0 < cols) load_raw(gamma + j0, graw[c]);
#pragma unroll
    for (int k = 0; k < 8; ++k) { adg[c][k] = 0.f; adb[c][k] = 0.f; }
  }
  const float inv_n = 1.0f / static_cast<float>(cols);
  for (int r0 = RPI * blockIdx.x; r0 < rows; r0 += RPI * gridDim.x) {
    int rr[RPI];
    float mu[RPI], rs[RPI];
    Raw8<T> rdy[RPI][NC], rx[RPI][NC], rdr[RPI][NC];
#pragma unroll
    for (int q = 0; q < RPI; ++q) {
      rr[q] = r0 + q < rows ? r0 + q : r0;  // a missing row re-reads the first, uncounted
      mu[q] = mean[rr[q]];
      rs[q] = rstd[rr[q]];
      const size_t base = static_cast<size_t>(rr[q]) * cols;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int j0 = (threadIdx.x + c * kBwdThreads) * 8;
        if (j0 < cols) {
          if (DROP) {
            load_raw(dy + base + j0, rdy[q][c]);
            load_raw_streaming(x + base + j0, rx[q][c]);
            load_raw_streaming(dres + base + j0, rdr[q][c]);
          } else {
            load_raw_streaming(dy + base + j0, rdy[q][c]);
            load_raw_streaming(x + base + j0, rx[q][c]);
            load_raw_streaming(dres + base + j0, rdr[q][c]);
          }
        }
      }
    }
    float sums[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < RPI; ++q) {
      const float live = r0 + q < rows ? 1.0f : 0.0f;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int j0 = (threadIdx.x + c * kBwdThreads) * 8;
        if (j0 < cols) {
          float gd[8], xh[8], g[8];
          unpack(rdy[q][c], gd);
          unpack(rx[q][c], xh);
          unpack(graw[c], g);
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            xh[k] = (xh[k] - mu[q]) * rs[q];
            adg[c][k] += live * gd[k] * xh[k];
            adb[c][k] += live * gd[k];
            gd[k] *= g[k];
            sums[2 * q] += gd[k];
            sums[2 * q + 1] += gd[k] * xh[k];
          }
        }
      }
    }
    block_sum4(sums, smem);
#pragma unroll
    for (int q = 0; q < RPI; ++q)
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        forget(rdy[q][c]);
        forget(rx[q][c]);
      }
#pragma unroll
    for (int q = 0; q < RPI; ++q) {
      if (r0 + q >= rows) break;
      const size_t base = static_cast<size_t>(rr[q]) * cols;
      const float m1 = sums[2 * q] * inv_n, m2 = sums[2 * q + 1] * inv_n;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int j0 = (threadIdx.x + c * kBwdThreads) * 8;
        if (j0 < cols) {
          float gd[8], xh[8], g[8], dr[8], o[8];
          unpack(rdy[q][c], gd);
          unpack(rx[q][c], xh);
          unpack(graw[c], g);
          unpack(rdr[q][c], dr);
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            xh[k] = (xh[k] - mu[q]) * rs[q];
            o[k] = dr[k] + rs[q] * (gd[k] * g[k] - m1 - xh[k] * m2);
          }
          store8(dx_out + base + j0, o);
          if (DROP) {
            float d[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) d[k] = round_to_storage(o[k], static_cast<T*>(nullptr));
            dropout_apply8(key, (base + j0) >> 3, d);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              d[k] = round_to_storage(d[k], static_cast<T*>(nullptr));
              adbias[DROP ? c : 0][k] += d[k];
            }
            store8(dropped + base + j0, d);
          }
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
      if (DROP) store8(part_dbias + static_cast<size_t>(blockIdx.x) * cols + j0, adbias[DROP ? c : 0]);
    }
  }
}

constexpr int kBwdRowsPerIter = 2;

int bwd_blocks(int rows) {
  const int groups = (rows + kBwdRowsPerIter - 1) / kBwdRowsPerIter;
  return groups < kBwdMaxBlocks ? groups : kBwdMaxBlocks;
}

}  // namespace

hipError_t layernorm_fwd(int dtype, const void* x, const void* gamma, const void* beta, void* y,
                         float* mean, float* rstd, int rows, int cols, float eps, hipStream_t st) {
  if (cols > 8192 || cols % 8 || rows <= 0) return hipErrorInvalidValue;
  const int vecs = cols / 8;
#define CALL(BS, NC)                                                                               \
  if (dtype == 1)                                                                                  \
    hipLaunchKernelGGL((layernorm_fwd_kernel<bf16_t, BS, NC>), dim3(rows), dim3(BS), 0, st,        \
                       static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(gamma),           \
                       static_cast<const bf16_t*>(beta), static_cast<bf16_t*>(y), mean, rstd,      \
                       rows, cols, eps);                                                           \
  else                                                                                             \
    hipLaunchKernelGGL((layernorm_fwd_kernel<float, BS, NC>), dim3(rows), dim3(BS), 0, st,         \
                       static_cast<const float*>(x), static_cast<const float*>(gamma),             \
                       static_cast<const float*>(beta), static_cast<float*>(y), mean, rstd, rows,  \
                       cols, eps)
  // many rows: the streaming form, 1024 resident workgroups (must give the same bits as the
  // one-row form: same per-thread columns, same reduction order)
  if (rows % 8 == 0 && rows >= 4 * kFwdStreamBlocks && vecs > 512) {
#define CALLS(BS, NC)                                                                              \
  if (dtype == 1)                                                                                  \
    hipLaunchKernelGGL((layernorm_fwd_stream_kernel<bf16_t, BS, NC>), dim3(kFwdStreamBlocks),      \
                       dim3(BS), 0, st, static_cast<const bf16_t*>(x),                             \
                       static_cast<const bf16_t*>(gamma), static_cast<const bf16_t*>(beta),        \
                       static_cast<bf16_t*>(y), mean, rstd, rows, cols, eps);                      \
  else                                                                                             \
    hipLaunchKernelGGL((layernorm_fwd_stream_kernel<float, BS, NC>), dim3(kFwdStreamBlocks),       \
                       dim3(BS), 0, st, static_cast<const float*>(x),                              \
                       static_cast<const float*>(gamma), static_cast<const float*>(beta),          \
                       static_cast<float*>(y), mean, rstd, rows, cols, eps)
    if (vecs <= 768) { CALLS(256, 3); }
    else { CALLS(256, 4); }
#undef CALLS
    return hipGetLastError();
  }
  // up to four vectors per thread
  if (vecs <= 64) { CALL(64, 1); }
  else if (vecs <= 128) { CALL(64, 2); }
  else if (vecs <= 256) { CALL(64, 4); }
  else if (vecs <= 512) { CALL(128, 4); }
  else if (vecs <= 768) { CALL(256, 3); }
  else { CALL(256, 4); }
#undef CALL
  return hipGetLastError();
}

size_t layernorm_bwd_scratch_bytes(int rows, int cols) {
  return 3 * static_cast<size_t>(bwd_blocks(rows)) * cols * sizeof(float);
}

namespace {

template <typename T, bool DROP>
hipError_t launch_bwd(const T* dy, const T* x, const float* mean, const float* rstd, const T* gamma,
                      const T* dres, T* dx_out, T* dgamma, T* dbeta, float* scratch, int rows, int cols,
                      T* dropped, T* dbias, DropoutKey key, hipStream_t st) {
  const int nb = bwd_blocks(rows);
  float* part_dg = scratch;
  float* part_db = scratch + static_cast<size_t>(nb) * cols;
  float* part_dbias = scratch + 2 * static_cast<size_t>(nb) * cols;
  const int nc = (cols / 8 + kBwdThreads - 1) / kBwdThreads;
#define CALL(NC)                                                                                     \
  hipLaunchKernelGGL((layernorm_bwd_kernel<T, NC, kBwdRowsPerIter, DROP>), dim3(nb), dim3(kBwdThreads), 0, st, \
                     dy, x, mean, rstd, gamma, dres, dx_out, part_dg, part_db, rows, cols, dropped,   \
                     part_dbias, key)
  if (nc <= 1) { CALL(1); }
  else if (nc <= 2) { CALL(2); }
  else if (nc <= 3) { CALL(3); }
  else { CALL(4); }
#undef CALL
  launch_reduce_partials<T>(part_dg, dgamma, part_db, dbeta, nb, cols, st);
  if (DROP) launch_reduce_partials<T>(part_dbias, dbias, nullptr, nullptr, nb, cols, st);
  return hipGetLastError();
}

}  // namespace

hipError_t layernorm_bwd(int dtype, const void* dy, const void* x, const float* mean,
                         const float* rstd, const void* gamma, const void* dres, void* dx_out,
                         void* dgamma, void* dbeta, float* scratch, int rows, int cols,
                         hipStream_t st) {
  if (cols > 8192 || cols % 8) return hipErrorInvalidValue;
  const DropoutKey none{};
  if (dtype == 1)
    return launch_bwd<bf16_t, false>(static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(x), mean, rstd,
                                     static_cast<const bf16_t*>(gamma), static_cast<const bf16_t*>(dres),
                                     static_cast<bf16_t*>(dx_out), static_cast<bf16_t*>(dgamma),
                                     static_cast<bf16_t*>(dbeta), scratch, rows, cols, nullptr, nullptr, none, st);
  return launch_bwd<float, false>(static_cast<const float*>(dy), static_cast<const float*>(x), mean, rstd,
                                  static_cast<const float*>(gamma), static_cast<const float*>(dres),
                                  static_cast<float*>(dx_out), static_cast<float*>(dgamma),
                                  static_cast<float*>(dbeta), scratch, rows, cols, nullptr, nullptr, none, st);
}

hipError_t layernorm_bwd_dropout_bwd(int dtype, const void* dy, const void* x, const float* mean,
                                     const float* rstd, const void* gamma, const void* dres, void* dx_out,
                                     void* dgamma, void* dbeta, void* dropped, void* dbias, float* scratch,
                                     int rows, int cols, int site, DropoutParams dp, hipStream_t st) {
  if (cols > 8192 || cols % 8) return hipErrorInvalidValue;
  const DropoutKey key = make_dropout_key(dp, site);
  if (dtype == 1)
    return launch_bwd<bf16_t, true>(static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(x), mean, rstd,
                                    static_cast<const bf16_t*>(gamma), static_cast<const bf16_t*>(dres),
                                    static_cast<bf16_t*>(dx_out), static_cast<bf16_t*>(dgamma),
                                    static_cast<bf16_t*>(dbeta), scratch, rows, cols,
                                    static_cast<bf16_t*>(dropped), static_cast<bf16_t*>(dbias), key, st);
  return launch_bwd<float, true>(static_cast<const float*>(dy), static_cast<const float*>(x), mean, rstd,
                                 static_cast<const float*>(gamma), static_cast<const float*>(dres),
                                 static_cast<float*>(dx_out), static_cast<float*>(dgamma),
                                 static_cast<float*>(dbeta), scratch, rows, cols,
                                 static_cast<float*>(dropped), static_cast<float*>(dbias), key, st);
}

}  // namespace lynx
