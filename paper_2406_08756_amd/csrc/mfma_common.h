// Building blocks of the matrix-core kernels: MFMA operand fragments, the LDS slab layouts
// that direct global -> LDS loads fill and fragment reads drain without bank conflicts, and
// the hand-counted waits those loads need.  Shared by the dense products (gemm_mfma.hip) and
// the fused attention kernels (attn_fused.hip); everything here is device code in an
// anonymous namespace of the including file.
#pragma once
#include "device_common.h"

namespace lynx {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4_t __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2_t __attribute__((ext_vector_type(2)));
typedef short short8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

constexpr int kBK = 32;        // K slab
constexpr int kThreads = 256;  // 4 wavefronts
constexpr int kWaves = kThreads / kWave;

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding:
// vmcnt = bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
// Workgroup barrier that neither the optimiser nor the scheduler moves memory
// accesses across (and that, unlike __syncthreads, does not drain the loads
// still in flight).
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}
__device__ __forceinline__ void wait_lgkmcnt0() {
  __builtin_amdgcn_s_waitcnt(15 | (3 << 14) | (7 << 4) | (0 << 8));
}

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

// An MFMA operand fragment as it arrives from LDS.  K-major slabs are read with plain
// 16-byte loads, which the compiler tracks.  MN-major slabs are read with the transposing
// LDS read, issued as inline assembly: the compiler's hazard tracking takes that read, as
// a builtin, to alias every direct-to-LDS load in flight and waits for all of them
// (vmcnt(0)) before it, which empties the prefetch ring once per slab.  The kernel's own
// lgkmcnt waits cover these reads; settle(), called after such a wait, makes every later
// use of the registers depend on a point after it.
template <bool KMAJOR> struct Frag;
template <> struct Frag<true> {
  bf16x8_t v;
  __device__ __forceinline__ bf16x8_t operand() const { return v; }
  __device__ __forceinline__ void settle() {}
};
template <> struct Frag<false> {
  short4_t lo, hi;
  __device__ __forceinline__ bf16x8_t operand() const {
    const short8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8_t, v);
  }
  __device__ __forceinline__ void settle() { asm volatile("" : "+v"(lo), "+v"(hi)); }
};

// One slab (ROWS x 32 elements) of an operand.
template <int ROWS, bool KMAJOR>
struct Slab {
  static constexpr int kElems = ROWS * kBK;
  static constexpr int kLoadsPerWave = ROWS / 16 / kWaves;  // 1 KB direct loads per wavefront
  static_assert(ROWS % (16 * kWaves) == 0, "slab must split over the wavefronts");
  // 16-byte chunk permutation of row `row` of a K-major slab (see the file comment of gemm_mfma.hip)
  __device__ static __forceinline__ int kswz(int row) { return (row >> 2) & 3; }

  // Global element offset, relative to the slab origin (row0, k0), that lane
  // `lane` fetches in this wavefront's j-th load; and that load's LDS offset.
  __device__ static __forceinline__ long long global_offset(int wave, int j, int lane, long long ld) {
    const int q = wave + kWaves * j;  // which 1 KB piece of the slab
    if (KMAJOR) {
      const int row = 16 * q + (lane >> 2);
      const int chunk = (lane & 3) ^ kswz(row);
      return static_cast<long long>(row) * ld + chunk * 8;
    } else {
      constexpr int kRowChunks = ROWS / 8;          // 16-byte chunks per k-row
      constexpr int kRowsPerLoad = 64 / kRowChunks; // k-rows per 1 KB
      const int k = kRowsPerLoad * q + lane / kRowChunks;
      const int chunk = (lane % kRowChunks) ^ ((k & 3) << 2);
      return static_cast<long long>(k) * ld + chunk * 8;
    }
  }
  __device__ static __forceinline__ int lds_offset(int wave, int j) { return (wave + kWaves * j) * 512; }

  // MFMA operand fragment: 8 consecutive k (at 16 ks + 8 (lane / 32)) of slab
  // row tile_row0 + lane % 32.
  __device__ static __forceinline__ Frag<KMAJOR> fragment(const bf16_t* slab, int tile_row0, int ks, int lane) {
    Frag<KMAJOR> f;
    if constexpr (KMAJOR) {
      const int r = tile_row0 + (lane & 31);
      const int chunk = (2 * ks + (lane >> 5)) ^ kswz(r);
      f.v = *reinterpret_cast<const bf16x8_t*>(slab + r * kBK + chunk * 8);
    } else {
      // four blocks of 16 lanes: block b holds rows (b & 1) * 16.. of k-group b >> 1; in a
      // block, lane i points at k-row i / 4, columns 4 (i % 4)..+3 and receives column i.
      const int b = lane >> 4, i = lane & 15;
      const int k = ks * 16 + (b >> 1) * 8 + (i >> 2);
      const int col = tile_row0 + (b & 1) * 16 + ((i & 3) << 2);
      const int sw = (k & 3) << 2;  // same for k and k + 4
      const bf16_t* p = slab + k * ROWS + (((col >> 3) ^ sw) << 3) + (col & 7);
      typedef const __attribute__((address_space(3))) bf16_t* lds_ptr_t;
      const uint32_t addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)(p)));
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(f.lo) : "v"(addr));
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(addr), "n"(4 * ROWS * 2));
    }
    return f;
  }
};

}  // namespace
}  // namespace lynx
