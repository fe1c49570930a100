// Attention without the seq x seq tensors (operators 3-6 and their backward as three
// kernels) for policies that retain none of S, P and Pd: the scores are formed on the matrix
// cores, turned into probabilities and dropped-out probabilities in registers and LDS, and
// consumed by the next product at once, so no s^2 tensor ever reaches HBM.
//
// Every number produced here has to be the one the unfused chain (attn_outer_kernel ->
// softmax_dropout_fwd_kernel -> the causal products of gemm_mfma.hip) produces, bit for bit:
// a policy that keeps S, P or Pd runs that chain, and gradients may not depend on the policy.
// So the kernels below follow the same rounding points and the same accumulation orders:
//   S   = round(sum_dd q k), 8 MFMA steps of 16 in ascending dd              (operator 3)
//   P   = round(exp(scale S - m) / l), m the row maximum of scale S, l the row sum of the
//         exponentials in the canonical order of attn_math.h                  (operator 4)
//   Pd  = round(keep c P)                                                     (operator 5)
//   C   = round(sum_j Pd v), MFMA steps of 16 in ascending j                  (operator 6)
//   dPd = round(sum_dd dC v); dS = round(scale P (keep c dPd - dot))          (B6, B5, B4)
//   dV  = round(sum_i Pd dC), dK = round(sum_i dS q), ascending i;  dQ = round(sum_j dS k)
// The row statistics (m, 1 / l) that the forward kernel leaves next to C let the backward
// kernels rebuild P without a reduction.
//
// Work decomposition: a workgroup of 4 wavefronts (2 x 2, 64 x 64 each) owns a block of 128
// query rows (forward, dQ) or 128 key rows (dK, dV) of one (batch element, head) and walks
// the 128 x 128 tiles of its causal range; operand tiles travel global -> LDS directly.
#include "attn_math.h"
#include "dropout_host.h"
#include "kernels.h"
#include "mfma_common.h"

#include <mutex>
#include <type_traits>

namespace lynx {
namespace {

constexpr int kD = 128;                      // head dimension these kernels are built for
constexpr int kTile = 128;                   // rows / columns of a score tile
using SLK = Slab<kTile, true>;               // a [128][32] K-major slab: Q, K (over dd), Pd, dS (over j)
using SLM = Slab<kTile, false>;              // a [32][128] MN-major slab: V, dC, Q, K as "k-rows"
constexpr int kSlabs = kD / kBK;             // slabs per 128 x 128 operand tile
constexpr int kOpElems = kSlabs * SLK::kElems;                  // 128 x 128 elements
constexpr int kTileLoads = kSlabs * SLK::kLoadsPerWave;         // direct loads per wavefront per tile
static_assert(SLK::kLoadsPerWave == SLM::kLoadsPerWave, "tile loads");

struct AttnFusedArgs {
  const bf16_t* qkv; long long ld;   // [T, 3 p] activations, row stride
  int p;                             // a * d: distance between the q | k | v column blocks
  bf16_t* c; long long ldc;          // [T, p] context (forward: written; backward: unused)
  float* stats;                      // [b * a][s][2]: row maximum of the logits, 1 / row sum
  const bf16_t* dc; long long lddc;  // backward: [T, p] gradient of the context
  const float* rowdot;               // backward: [b * a][s] sum_dd dC C
  bf16_t* dqkv; long long lddq;      // backward: [T, 3 p] gradients, same layout as qkv
  int s, a, nz;                      // sequence length, local heads, b * a
  float scale;
  DropoutKey key;
  int global_heads, head0;
};

typedef __attribute__((address_space(3))) bf16_t* lds_bf16_ptr;
typedef const __attribute__((address_space(3))) bf16_t* lds_cbf16_ptr;
__device__ __forceinline__ uint32_t lds_addr(const bf16_t* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_cbf16_ptr)(p)));
}

// Direct loads of one 128 x 128 operand tile.  K-major: `src` points at (row0, k0 = 0) of a
// [128 rows][128 k] block with row stride ld.  MN-major: `src` points at (k-row 0, col 0) of
// a [128 k-rows][128] block.
template <typename SL>
__device__ __forceinline__ void load_tile(const bf16_t* src, long long ld, bf16_t* dst, int wave, int lane) {
#pragma unroll
  for (int sl = 0; sl < kSlabs; ++sl)
#pragma unroll
    for (int j = 0; j < SL::kLoadsPerWave; ++j) {
      const bf16_t* from = std::is_same<SL, SLK>::value
                               ? src + SL::global_offset(wave, j, lane, ld) + sl * kBK
                               : src + SL::global_offset(wave, j, lane, ld) + static_cast<long long>(sl) * kBK * ld;
      __builtin_amdgcn_global_load_lds((global_void_ptr)(from),
                                       (lds_void_ptr)(dst + sl * SL::kElems + SL::lds_offset(wave, j)), 16, 0, 0);
    }
}

// acc += X Y^T over the head dimension: X, Y K-major tiles in LDS, 64 x 64 per wavefront.
// acc[i][j][r]: column wn0 + 32 i + 8 (r / 4) + 4 (lane / 32) + r % 4, row wm0 + 32 j + lane % 32.
__device__ __forceinline__ void product_kmajor(const bf16_t* sX, const bf16_t* sY, int wm0, int wn0, int lane,
                                               floatx16_t (&acc)[2][2]) {
#pragma unroll
  for (int kk = 0; kk < kD / 16; ++kk) {
    Frag<true> fa[2], fb[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) fa[j] = SLK::fragment(sX + (kk >> 1) * SLK::kElems, wm0 + 32 * j, kk & 1, lane);
#pragma unroll
    for (int i = 0; i < 2; ++i) fb[i] = SLK::fragment(sY + (kk >> 1) * SLK::kElems, wn0 + 32 * i, kk & 1, lane);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i].operand(), fa[j].operand(), acc[i][j], 0, 0, 0);
  }
}

// acc += X Y over the 128 contraction rows of this tile: X K-major (rows x k), Y MN-major
// (k-rows x columns), both in LDS.
__device__ __forceinline__ void product_mixed(const bf16_t* sX, const bf16_t* sY, int wm0, int wn0, int lane,
                                              floatx16_t (&acc)[2][2]) {
#pragma unroll
  for (int kk = 0; kk < kTile / 16; ++kk) {
    Frag<true> fa[2];
    Frag<false> fb[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) fa[j] = SLK::fragment(sX + (kk >> 1) * SLK::kElems, wm0 + 32 * j, kk & 1, lane);
#pragma unroll
    for (int i = 0; i < 2; ++i) fb[i] = SLM::fragment(sY + (kk >> 1) * SLM::kElems, wn0 + 32 * i, kk & 1, lane);
    wait_lgkmcnt0();
#pragma unroll
    for (int i = 0; i < 2; ++i) fb[i].settle();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i].operand(), fa[j].operand(), acc[i][j], 0, 0, 0);
  }
}

// acc += X^T Y over the 128 contraction rows of this tile: X and Y MN-major (k-rows x
// columns), i.e. both are read through the transposing LDS read.
__device__ __forceinline__ void product_tn(const bf16_t* sX, const bf16_t* sY, int wm0, int wn0, int lane,
                                           floatx16_t (&acc)[2][2]) {
#pragma unroll
  for (int kk = 0; kk < kTile / 16; ++kk) {
    Frag<false> fa[2], fb[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) fa[j] = SLM::fragment(sX + (kk >> 1) * SLM::kElems, wm0 + 32 * j, kk & 1, lane);
#pragma unroll
    for (int i = 0; i < 2; ++i) fb[i] = SLM::fragment(sY + (kk >> 1) * SLM::kElems, wn0 + 32 * i, kk & 1, lane);
    wait_lgkmcnt0();
#pragma unroll
    for (int j = 0; j < 2; ++j) fa[j].settle();
#pragma unroll
    for (int i = 0; i < 2; ++i) fb[i].settle();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i].operand(), fa[j].operand(), acc[i][j], 0, 0, 0);
  }
}

__device__ __forceinline__ void clear(floatx16_t (&acc)[2][2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
}

// The storage-rounded value of an accumulator element, as a float.
__device__ __forceinline__ float stored(float v) { return bf16_lo(pack_bf16(v, 0.f)); }

// A wavefront's 64 x 64 quadrant of accumulators, rounded to storage, through its own 8 KB
// of LDS and back as whole rows: afterwards rows[u] holds 8 consecutive columns (8 lc ..) of
// quadrant row 8 u + lr, lr = lane / 8, lc = lane % 8.  LDS executes a wavefront's accesses
// in order, so no barrier is needed between the writes and the reads.
__device__ __forceinline__ void quadrant_to_rows(const floatx16_t (&acc)[2][2], bf16_t* stage, int lane,
                                                 uintx4_t (&rows)[8]) {
  constexpr int WN = 64, kRowChunks = 8;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int nl = 32 * i + 8 * q + 4 * (lane >> 5);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int ml = 32 * j + (lane & 31);
        uintx2_t o;
        o[0] = pack_bf16(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1]);
        o[1] = pack_bf16(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        const int chunk = (nl >> 3) ^ (ml & (kRowChunks - 1));
        asm volatile("ds_write_b64 %0, %1" : : "v"(lds_addr(stage + ml * WN + chunk * 8 + (nl & 7))), "v"(o) : "memory");
      }
    }
  const int lr = lane >> 3, lc = lane & 7;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int r = u * 8 + lr;
    asm volatile("ds_read_b128 %0, %1" : "=v"(rows[u]) : "v"(lds_addr(stage + r * WN + ((lc ^ (r & (kRowChunks - 1))) << 3))) : "memory");
  }
  wait_lgkmcnt0();
#pragma unroll
  for (int u = 0; u < 8; ++u) asm volatile("" : "+v"(rows[u]));
}

// 8 storage values of tile row R, tile columns col0 .. col0 + 7, into a K-major operand tile
// in LDS (the layout SLK::fragment reads).
__device__ __forceinline__ void rows_to_operand(bf16_t* sOp, int R, int col0, const float (&v)[8]) {
  uintx4_t o;
  o[0] = pack_bf16(v[0], v[1]); o[1] = pack_bf16(v[2], v[3]);
  o[2] = pack_bf16(v[4], v[5]); o[3] = pack_bf16(v[6], v[7]);
  const int slab = col0 >> 5, chunk = ((col0 & 31) >> 3) ^ SLK::kswz(R);
  asm volatile("ds_write_b128 %0, %1" : : "v"(lds_addr(sOp + slab * SLK::kElems + R * kBK + chunk * 8)), "v"(o) : "memory");
}

// The same values into an MN-major operand tile (contraction index = the tile row R): the
// layout SLM::fragment reads, [32 k-rows][128 columns] per slab.
__device__ __forceinline__ void rows_to_operand_mn(bf16_t* sOp, int R, int col0, const float (&v)[8]) {
  uintx4_t o;
  o[0] = pack_bf16(v[0], v[1]); o[1] = pack_bf16(v[2], v[3]);
  o[2] = pack_bf16(v[4], v[5]); o[3] = pack_bf16(v[6], v[7]);
  const int slab = R >> 5, k = R & 31;
  const int chunk = (col0 >> 3) ^ ((k & 3) << 2);
  asm volatile("ds_write_b128 %0, %1" : : "v"(lds_addr(sOp + slab * SLM::kElems + k * kTile + chunk * 8)), "v"(o) : "memory");
}

__device__ __forceinline__ void unpack8(const uintx4_t& r, float (&v)[8]) {
  v[0] = bf16_lo(r[0]); v[1] = bf16_hi(r[0]); v[2] = bf16_lo(r[1]); v[3] = bf16_hi(r[1]);
  v[4] = bf16_lo(r[2]); v[5] = bf16_hi(r[2]); v[6] = bf16_lo(r[3]); v[7] = bf16_hi(r[3]);
}

// P (rounded to storage) for 8 consecutive columns of one row from the stored scores.
// `limit`: columns >= limit are beyond the causal boundary (probability exactly 0).
__device__ __forceinline__ void probabilities8(const uintx4_t& sraw, float scale, float m, float inv, int col0,
                                               int limit, float (&p)[8]) {
  float sv[8];
  unpack8(sraw, sv);
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const float e = col0 + k < limit ? softmax_exp(softmax_logit(sv[k], scale), m) : 0.0f;
    p[k] = softmax_prob<bf16_t>(e, inv);
  }
}

// ---------------------------------------------------------------------------
// Forward: C and the row statistics of one block of 128 query rows.
// LDS: Q | K (two buffers in passes 1 and 2; in pass 3 the first is K and the staging area,
// the second is V) | Pd as an operand tile | row statistics.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) attn_fwd_fused_kernel(AttnFusedArgs g) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  bf16_t* sQ = reinterpret_cast<bf16_t*>(smem_raw);
  bf16_t* sK = sQ + kOpElems;          // two buffers
  bf16_t* sPd = sK + 2 * kOpElems;
  float* sRow = reinterpret_cast<float*>(sPd + kOpElems);  // [2][2][128]: (max | sum) x (column half) x row

  const int tiles = g.s / kTile;
  const int t = blockIdx.x / g.nz;
  const int bz = blockIdx.x - t * g.nz;
  const int tm = tiles - 1 - t;  // longest row blocks first
  const int bi = bz / g.a, hd = bz - bi * g.a;
  const bf16_t* Qb = g.qkv + (static_cast<long long>(bi) * g.s + tm * kTile) * g.ld + hd * kD;
  const bf16_t* Kb = g.qkv + static_cast<long long>(bi) * g.s * g.ld + g.p + hd * kD;
  const bf16_t* Vb = Kb + g.p;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
  const int hb = lane >> 5;

  load_tile<SLK>(Qb, g.ld, sQ, wave, lane);
  load_tile<SLK>(Kb, g.ld, sK, wave, lane);

  // ---- pass 1: row maxima of the logits ------------------------------------
  float mx[2] = {-INFINITY, -INFINITY};
  for (int tn = 0; tn <= tm; ++tn) {
    wait_vmcnt<0>();
    block_barrier();
    if (tn < tm) load_tile<SLK>(Kb + static_cast<long long>(tn + 1) * kTile * g.ld, g.ld, sK + ((tn + 1) & 1) * kOpElems, wave, lane);
    floatx16_t acc[2][2];
    clear(acc);
    product_kmajor(sQ, sK + (tn & 1) * kOpElems, wm0, wn0, lane, acc);
    const bool diag = tn == tm;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int col = wn0 + 32 * i + 8 * (r >> 2) + 4 * hb + (r & 3), row = wm0 + 32 * j + (lane & 31);
          const float z = softmax_logit(stored(acc[i][j][r]), g.scale);
          if (!diag || col <= row) mx[j] = fmaxf(mx[j], z);
        }
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    mx[j] = fmaxf(mx[j], __shfl_xor(mx[j], 32, kWave));
    if (hb == 0) sRow[(wave & 1) * kTile + wm0 + 32 * j + lane] = mx[j];
  }
  // (every wavefront is past its last read of the K buffers: the first tile of the next pass
  // can be requested; the barrier below also publishes the maxima)
  block_barrier();
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = wm0 + 32 * j + (lane & 31);
    mx[j] = fmaxf(sRow[row], sRow[kTile + row]);
  }
  asm volatile("" : "+v"(mx[0]), "+v"(mx[1]));
  load_tile<SLK>(Kb, g.ld, sK, wave, lane);

  // ---- pass 2: row sums of the exponentials, canonical order ------------------
  float sum[2] = {0.f, 0.f};
  for (int tn = 0; tn <= tm; ++tn) {
    wait_vmcnt<0>();
    block_barrier();
    if (tn < tm) load_tile<SLK>(Kb + static_cast<long long>(tn + 1) * kTile * g.ld, g.ld, sK + ((tn + 1) & 1) * kOpElems, wave, lane);
    floatx16_t acc[2][2];
    clear(acc);
    product_kmajor(sQ, sK + (tn & 1) * kOpElems, wm0, wn0, lane, acc);
    const bool diag = tn == tm;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row = wm0 + 32 * j + (lane & 31);
      float x[8];  // group sums of this lane's half (hb) of vectors 4 i + q of the 64-column block
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float e[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int col = wn0 + 32 * i + 8 * q + 4 * hb + c;
            const float z = softmax_logit(stored(acc[i][j][4 * q + c]), g.scale);
            e[c] = (!diag || col <= row) ? softmax_exp(z, mx[j]) : 0.0f;
          }
          x[4 * i + q] = softmax_group4(e[0], e[1], e[2], e[3]);
        }
      const float th = softmax_tree8(x[0], x[1], x[2], x[3], x[4], x[5], x[6], x[7]);
      sum[j] += th + __shfl_xor(th, 32, kWave);
    }
  }
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if (hb == 0) sRow[2 * kTile + (wave & 1) * kTile + wm0 + 32 * j + lane] = sum[j];
  block_barrier();
  // this lane's eight rows of the store layout: statistics and dropout indices
  const int lr = lane >> 3, lc = lane & 7;
  float rm[8], rinv[8];
  uint64_t gidx[8];
  const uint64_t rows_before = (static_cast<uint64_t>(bi) * g.global_heads + g.head0 + hd) * g.s;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int row = wm0 + 8 * u + lr;
    rm[u] = fmaxf(sRow[row], sRow[kTile + row]);
    rinv[u] = softmax_inverse(sRow[2 * kTile + row] + sRow[3 * kTile + row]);
    gidx[u] = (rows_before + tm * kTile + row) * static_cast<uint64_t>(g.s) + wn0 + lc * 8;
  }
#pragma unroll
  for (int u = 0; u < 8; ++u) asm volatile("" : "+v"(rm[u]), "+v"(rinv[u]));
  // pass 3 layout: first K buffer = K tile and staging, second = V tile
  bf16_t* sV = sK + kOpElems;
  load_tile<SLK>(Kb, g.ld, sK, wave, lane);
  load_tile<SLM>(Vb, g.ld, sV, wave, lane);
  if (wave == 0 || wave == 2) {  // one wavefront per row half writes the statistics
    if (lc == 0) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        float* st = g.stats + (static_cast<long long>(bz) * g.s + tm * kTile + wm0 + 8 * u + lr) * 2;
        st[0] = rm[u];
        st[1] = rinv[u];
      }
    }
  }

  // ---- pass 3: P, Pd and C -------------------------------------------------------
  floatx16_t accC[2][2];
  clear(accC);
  bf16_t* stage = sK + wave * (64 * 64);
  for (int tn = 0; tn <= tm; ++tn) {
    wait_vmcnt<0>();   // K(tn) (and, the first time, V(0) and the statistics' stores)
    block_barrier();   // also: every wavefront is done with V(tn - 1) and the previous Pd tile
    if (tn > 0) load_tile<SLM>(Vb + static_cast<long long>(tn) * kTile * g.ld, g.ld, sV, wave, lane);
    floatx16_t acc[2][2];
    clear(acc);
    product_kmajor(sQ, sK, wm0, wn0, lane, acc);
    block_barrier();   // every wavefront has read K(tn): its buffer becomes the staging area
    uintx4_t rows[8];
    quadrant_to_rows(acc, stage, lane, rows);
    block_barrier();   // every wavefront has its rows: the buffer can take the next K tile
    if (tn < tm) load_tile<SLK>(Kb + static_cast<long long>(tn + 1) * kTile * g.ld, g.ld, sK, wave, lane);
    const bool diag = tn == tm;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int row = wm0 + 8 * u + lr, col0 = wn0 + lc * 8;
      float p[8];
      probabilities8(rows[u], g.scale, rm[u], rinv[u], col0, diag ? row + 1 : kTile, p);
      dropout_apply8(g.key, (gidx[u] + static_cast<uint64_t>(tn) * kTile) >> 3, p);
      rows_to_operand(sPd, row, col0, p);
    }
    // V(tn) has landed (issued after it: the next K tile, if any); Pd is written
    if (tn == 0) {
      // (V(0) was waited for at the top)
    } else if (tn < tm) {
      wait_vmcnt<kTileLoads>();
    } else {
      wait_vmcnt<0>();
    }
    wait_lgkmcnt0();
    block_barrier();
    product_mixed(sPd, sV, wm0, wn0, lane, accC);
  }
  // C: round, through the (idle) staging area, whole rows out
  block_barrier();
  uintx4_t rows[8];
  quadrant_to_rows(accC, stage, lane, rows);
  bf16_t* cw = g.c + (static_cast<long long>(bi) * g.s + tm * kTile + wm0) * g.ldc + hd * kD + wn0;
#pragma unroll
  for (int u = 0; u < 8; ++u)
    *reinterpret_cast<uintx4_t*>(cw + static_cast<long long>(8 * u + lr) * g.ldc + lc * 8) = rows[u];
}

// ---------------------------------------------------------------------------
// Backward, first kernel: dS of one block of 128 query rows (B6 + B5 + B4).  Per tile the
// scores are formed again and turned into P with the stored row statistics, dPd = dC V^T is
// formed next to them, and dS = scale P (keep c dPd - dot) leaves for HBM: the one seq x seq
// tensor of the fused path, a transient that the dQ and dK products consume.
// LDS: Q | dC (resident) | K | V (streamed; after the two products they are the staging areas
// of S and dPd, and the next tiles arrive during the elementwise phase).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) attn_bwd_ds_kernel(AttnFusedArgs g, bf16_t* __restrict__ dS) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  bf16_t* sQ = reinterpret_cast<bf16_t*>(smem_raw);
  bf16_t* sdC = sQ + kOpElems;
  bf16_t* sK = sdC + kOpElems;
  bf16_t* sV = sK + kOpElems;

  const int tiles = g.s / kTile;
  const int t = blockIdx.x / g.nz;
  const int bz = blockIdx.x - t * g.nz;
  const int tm = tiles - 1 - t;
  const int bi = bz / g.a, hd = bz - bi * g.a;
  const long long tok0 = static_cast<long long>(bi) * g.s;
  const bf16_t* Qb = g.qkv + (tok0 + tm * kTile) * g.ld + hd * kD;
  const bf16_t* Kb = g.qkv + tok0 * g.ld + g.p + hd * kD;
  const bf16_t* Vb = Kb + g.p;
  const bf16_t* dCb = g.dc + (tok0 + tm * kTile) * g.lddc + hd * kD;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
  const int lr = lane >> 3, lc = lane & 7;

  // this lane's eight rows: statistics, dot products, dropout indices
  float rm[8], rinv[8], dot[8];
  uint64_t gidx[8];
  const uint64_t rows_before = (static_cast<uint64_t>(bi) * g.global_heads + g.head0 + hd) * g.s;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const long long i = tm * kTile + wm0 + 8 * u + lr;
    const float2 st = *reinterpret_cast<const float2*>(g.stats + (static_cast<long long>(bz) * g.s + i) * 2);
    rm[u] = st.x;
    rinv[u] = st.y;
    dot[u] = g.rowdot[static_cast<long long>(bz) * g.s + i];
    gidx[u] = (rows_before + i) * static_cast<uint64_t>(g.s) + wn0 + lc * 8;
  }
#pragma unroll
  for (int u = 0; u < 8; ++u) asm volatile("" : "+v"(rm[u]), "+v"(rinv[u]), "+v"(dot[u]));

  load_tile<SLK>(Qb, g.ld, sQ, wave, lane);
  load_tile<SLK>(dCb, g.lddc, sdC, wave, lane);
  load_tile<SLK>(Kb, g.ld, sK, wave, lane);
  load_tile<SLK>(Vb, g.ld, sV, wave, lane);

  bf16_t* stageS = sK + wave * (64 * 64);
  bf16_t* stageD = sV + wave * (64 * 64);
  bf16_t* out = dS + (static_cast<long long>(bz) * g.s + tm * kTile + wm0) * g.s + wn0;
  for (int tn = 0; tn <= tm; ++tn) {
    // K(tn), V(tn) have landed; issued after them: the previous tile's eight stores
    if (tn == 0) wait_vmcnt<0>();
    else wait_vmcnt<8>();
    block_barrier();
    floatx16_t accS[2][2], accD[2][2];
    clear(accS);
    clear(accD);
    product_kmajor(sQ, sK, wm0, wn0, lane, accS);
    product_kmajor(sdC, sV, wm0, wn0, lane, accD);
    block_barrier();  // every wavefront has read K(tn) and V(tn): their buffers become staging areas
    uintx4_t rowsS[8], rowsD[8];
    quadrant_to_rows(accS, stageS, lane, rowsS);
    quadrant_to_rows(accD, stageD, lane, rowsD);
    block_barrier();  // every wavefront has its rows: the buffers can take the next tiles
    if (tn < tm) {
      load_tile<SLK>(Kb + static_cast<long long>(tn + 1) * kTile * g.ld, g.ld, sK, wave, lane);
      load_tile<SLK>(Vb + static_cast<long long>(tn + 1) * kTile * g.ld, g.ld, sV, wave, lane);
    }
    const bool diag = tn == tm;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int row = wm0 + 8 * u + lr, col0 = wn0 + lc * 8;
      float p[8], dp[8], ds[8];
      probabilities8(rowsS[u], g.scale, rm[u], rinv[u], col0, diag ? row + 1 : kTile, p);
      unpack8(rowsD[u], dp);
      dropout_apply8(g.key, (gidx[u] + static_cast<uint64_t>(tn) * kTile) >> 3, dp);
#pragma unroll
      for (int k = 0; k < 8; ++k) ds[k] = softmax_bwd(p[k], dp[k], dot[u], g.scale);
      store8(out + static_cast<long long>(8 * u + lr) * g.s + tn * kTile + lc * 8, ds);
    }
  }
}

// ---------------------------------------------------------------------------
// Backward, second kernel: dV of one block of 128 key rows (the other half of B6).  Walks the
// query blocks i >= j: the scores of the tile are formed again, turned into P and Pd, and
// Pd^T dC is accumulated in ascending i.
// LDS: K (resident) | Q (two buffers: the next block is requested a tile ahead; after the
// score product the current one is the staging area and then holds Pd as an operand tile) |
// dC with the token index as the contraction row.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) attn_bwd_dv_kernel(AttnFusedArgs g) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  bf16_t* sK = reinterpret_cast<bf16_t*>(smem_raw);
  bf16_t* sQ = sK + kOpElems;  // two buffers
  bf16_t* sdC = sQ + 2 * kOpElems;

  const int tiles = g.s / kTile;
  const int t = blockIdx.x / g.nz;
  const int bz = blockIdx.x - t * g.nz;
  const int tj = t;  // key block; the longest walks (small j) first
  const int bi = bz / g.a, hd = bz - bi * g.a;
  const long long tok0 = static_cast<long long>(bi) * g.s;
  const bf16_t* Qb = g.qkv + tok0 * g.ld + hd * kD;
  const bf16_t* Kb = g.qkv + (tok0 + tj * kTile) * g.ld + g.p + hd * kD;
  const bf16_t* dCb = g.dc + tok0 * g.lddc + hd * kD;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
  const int lr = lane >> 3, lc = lane & 7;
  const uint64_t rows_before = (static_cast<uint64_t>(bi) * g.global_heads + g.head0 + hd) * g.s;

  load_tile<SLK>(Kb, g.ld, sK, wave, lane);
  load_tile<SLK>(Qb + static_cast<long long>(tj) * kTile * g.ld, g.ld, sQ, wave, lane);
  load_tile<SLM>(dCb + static_cast<long long>(tj) * kTile * g.lddc, g.lddc, sdC, wave, lane);

  floatx16_t accV[2][2];
  clear(accV);
  for (int ti = tj; ti < tiles; ++ti) {
    bf16_t* sQc = sQ + ((ti - tj) & 1) * kOpElems;
    // the statistics of this query block's rows (this lane's eight rows of the store layout)
    float rm[8], rinv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const long long i = ti * kTile + wm0 + 8 * u + lr;
      const float2 st = *reinterpret_cast<const float2*>(g.stats + (static_cast<long long>(bz) * g.s + i) * 2);
      rm[u] = st.x;
      rinv[u] = st.y;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) asm volatile("" : "+v"(rm[u]), "+v"(rinv[u]));
    wait_vmcnt<0>();   // Q(ti), dC(ti) (and, the first time, K) have landed
    block_barrier();   // also: every wavefront is done with the previous Pd operand tile
    if (ti + 1 < tiles)
      load_tile<SLK>(Qb + static_cast<long long>(ti + 1) * kTile * g.ld, g.ld, sQ + ((ti + 1 - tj) & 1) * kOpElems, wave, lane);
    floatx16_t acc[2][2];
    clear(acc);
    product_kmajor(sQc, sK, wm0, wn0, lane, acc);
    block_barrier();   // every wavefront has read Q(ti): its buffer becomes the staging area
    uintx4_t rows[8];
    quadrant_to_rows(acc, sQc + wave * (64 * 64), lane, rows);
    block_barrier();   // every wavefront has its rows: the buffer can take the Pd operand tile
    const bool diag = ti == tj;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int row = wm0 + 8 * u + lr, col0 = wn0 + lc * 8;
      float p[8];
      probabilities8(rows[u], g.scale, rm[u], rinv[u], col0, diag ? row + 1 : kTile, p);
      const uint64_t gi = (rows_before + ti * kTile + row) * static_cast<uint64_t>(g.s) + tj * kTile + col0;
      dropout_apply8(g.key, gi >> 3, p);
      rows_to_operand_mn(sQc, row, col0, p);
    }
    wait_lgkmcnt0();
    block_barrier();
    product_tn(sQc, sdC, wm0, wn0, lane, accV);
    if (ti + 1 < tiles) {
      block_barrier();  // every wavefront is done with dC(ti)
      load_tile<SLM>(dCb + static_cast<long long>(ti + 1) * kTile * g.lddc, g.lddc, sdC, wave, lane);
    }
  }
  // dV: round, through the staging area, whole rows out
  block_barrier();
  uintx4_t rows[8];
  quadrant_to_rows(accV, sK + wave * (64 * 64), lane, rows);
  bf16_t* vw = g.dqkv + (tok0 + tj * kTile + wm0) * g.lddq + 2 * g.p + hd * kD + wn0;
#pragma unroll
  for (int u = 0; u < 8; ++u)
    *reinterpret_cast<uintx4_t*>(vw + static_cast<long long>(8 * u + lr) * g.lddq + lc * 8) = rows[u];
}

constexpr size_t kFwdLds = 4 * static_cast<size_t>(kOpElems) * sizeof(bf16_t) + 4 * kTile * sizeof(float);
constexpr size_t kBwdLds = 4 * static_cast<size_t>(kOpElems) * sizeof(bf16_t);

#define LYNX_RAISE_LDS(kern, bytes)                                                              \
  do {                                                                                           \
    static std::once_flag once_;                                                                 \
    static hipError_t err_ = hipSuccess;                                                         \
    std::call_once(once_, [&] {                                                                  \
      err_ = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                            \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes)); \
    });                                                                                          \
    if (err_ != hipSuccess) return err_;                                                         \
  } while (0)

}  // namespace

bool attn_fused_supported(int dtype, int s, int d) { return dtype == 1 && d == kD && s % kTile == 0 && s >= kTile; }

size_t attn_fused_stats_bytes(int b, int a, int s) { return static_cast<size_t>(b) * a * s * 2 * sizeof(float); }

hipError_t attn_fused_fwd(const void* qkv, long long ld, void* c, long long ldc, float* stats, AttnShape sh, int d,
                          float scale, DropoutParams dp, hipStream_t st) {
  if (!attn_fused_supported(1, sh.s, d) || ld % 8 || ldc % 8) return hipErrorInvalidValue;
  AttnFusedArgs g{};
  g.qkv = static_cast<const bf16_t*>(qkv); g.ld = ld; g.p = sh.a * d;
  g.c = static_cast<bf16_t*>(c); g.ldc = ldc; g.stats = stats;
  g.s = sh.s; g.a = sh.a; g.nz = sh.b * sh.a; g.scale = scale;
  g.key = make_dropout_key(dp, 0); g.global_heads = sh.global_heads; g.head0 = sh.head0;
  LYNX_RAISE_LDS(attn_fwd_fused_kernel, kFwdLds);
  hipLaunchKernelGGL(attn_fwd_fused_kernel, dim3((sh.s / kTile) * g.nz), dim3(kThreads), kFwdLds, st, g);
  return hipGetLastError();
}


namespace {
AttnFusedArgs bwd_args(const void* qkv, long long ld, const void* dc, long long lddc, const float* stats, AttnShape sh,
                       int d, float scale, DropoutParams dp) {
  AttnFusedArgs g{};
  g.qkv = static_cast<const bf16_t*>(qkv); g.ld = ld; g.p = sh.a * d;
  g.stats = const_cast<float*>(stats); g.dc = static_cast<const bf16_t*>(dc); g.lddc = lddc;
  g.s = sh.s; g.a = sh.a; g.nz = sh.b * sh.a; g.scale = scale;
  g.key = make_dropout_key(dp, 0); g.global_heads = sh.global_heads; g.head0 = sh.head0;
  return g;
}
}  // namespace

hipError_t attn_fused_bwd_ds(const void* qkv, long long ld, const void* dc, long long lddc, const float* stats,
                             const float* rowdot, void* ds, AttnShape sh, int d, float scale, DropoutParams dp,
                             hipStream_t st) {
  if (!attn_fused_supported(1, sh.s, d) || ld % 8 || lddc % 8) return hipErrorInvalidValue;
  AttnFusedArgs g = bwd_args(qkv, ld, dc, lddc, stats, sh, d, scale, dp);
  g.rowdot = rowdot;
  LYNX_RAISE_LDS(attn_bwd_ds_kernel, kBwdLds);
  hipLaunchKernelGGL(attn_bwd_ds_kernel, dim3((sh.s / kTile) * g.nz), dim3(kThreads), kBwdLds, st, g,
                     static_cast<bf16_t*>(ds));
  return hipGetLastError();
}

hipError_t attn_fused_bwd_dv(const void* qkv, long long ld, const void* dc, long long lddc, const float* stats,
                             void* dqkv, long long lddq, AttnShape sh, int d, float scale, DropoutParams dp,
                             hipStream_t st) {
  if (!attn_fused_supported(1, sh.s, d) || ld % 8 || lddc % 8 || lddq % 8) return hipErrorInvalidValue;
  AttnFusedArgs g = bwd_args(qkv, ld, dc, lddc, stats, sh, d, scale, dp);
  g.dqkv = static_cast<bf16_t*>(dqkv); g.lddq = lddq;
  LYNX_RAISE_LDS(attn_bwd_dv_kernel, kBwdLds);
  hipLaunchKernelGGL(attn_bwd_dv_kernel, dim3((sh.s / kTile) * g.nz), dim3(kThreads), kBwdLds, st, g);
  return hipGetLastError();
}

}  // namespace lynx
