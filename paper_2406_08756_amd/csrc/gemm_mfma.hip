// bf16 matrix products on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16).
//
//   C[M, N] = sum_k A(m, k) * B(k, n) (+ bias[n]),   fp32 accumulation
//
// Either operand may be stored "K-major" (the contraction index is the
// contiguous one: activations and weights of a forward linear layer) or
// "MN-major" (the contraction index is the row index: the weight in an input
// gradient, both operands in a weight gradient).
//
// Design.  One workgroup of 4 wavefronts (one per SIMD, up to 512 registers
// each) owns a BM x BN output tile (256 x 256 when it divides); each
// wavefront owns a quarter of it, so every fragment read from LDS feeds four
// MFMAs.  K is walked in slabs of 32.  Slabs travel global memory -> LDS
// directly (global_load_lds_dwordx4, no staging registers) through a ring of
// four LDS stages: while one slab is multiplied, three more are in flight,
// which is what it takes to cover L2 latency at this MFMA rate.  Bank
// conflicts are avoided by permuting 16-byte chunks, applied on the global
// address side since a direct load writes lane i to LDS offset 16 i:
//   K-major slab  [mn][32]: chunk ^= (row >> 2) & 3
//   MN-major slab [32][mn]: chunk ^= (k & 3) << 2, read with the transposing
//     LDS read (ds_read_b64_tr_b16) that hands each lane four consecutive k.
// The product is formed transposed (B fragment as the first MFMA operand) so
// each lane ends with four consecutive n of one row m; the epilogue passes the
// tile through LDS and stores whole rows, 16 bytes per lane.
#include <mutex>
#include <type_traits>

#include "dropout_host.h"
#include "mfma_common.h"
#include "pointwise_math.h"
#include "reduce_partials.h"

namespace lynx {
namespace {

constexpr int kStages = 4;     // LDS ring depth
constexpr double kPairCutFraction = 0.9;  // see plan_pair

struct MfmaGemmArgs {
  const bf16_t* A; long long lda;
  const bf16_t* B; long long ldb;
  bf16_t* C; long long ldc;
  const bf16_t* bias;
  int M, N, K;
  int tiles_m, tiles_n;
  // batched use (attention): matrix z = z1 * nz2 + z2 starts at these element offsets
  long long a_z1, a_z2, b_z1, b_z2, c_z1, c_z2;
  int nz, nz2;
  int causal;  // CausalMode
  // split contraction: workgroup x computes K range x / (tiles_m tiles_n) of k_splits equal
  // ranges and leaves its fp32 sums in partial[split][M][N] instead of rounding into C
  int k_splits;
  float* partial;
  // fused epilogue (GemmEpilogueKind).  aux / vec / plain are indexed with the absolute
  // column col0 + n, so a launch that covers a column range of the output (edge strips)
  // passes them unchanged; row_len is the full row length (the dropout element index).
  int epi;
  int col0, row_len;
  const bf16_t* aux; long long aux_ld;
  const bf16_t* vec;
  bf16_t* plain;
  float* colsum_partial;
  DropoutKey key;
  // kEpiSoftmaxBwd (attention): per-row dot products, 1 / sqrt(d), dropout index map
  const float* rowdot;
  float scale;
  int global_heads, head0;
};

// One output tile: `block_x` selects the tile, `block_z` the matrix of a batch.
template <bool A_KMAJOR, bool B_KMAJOR, int BM, int BN, bool SPLITK = false, int STAGES = kStages>
__device__ __forceinline__ void gemm_tile(const MfmaGemmArgs& g, const int block_x, const int block_z) {
  constexpr int WM = BM / 2, WN = BN / 2;  // wavefronts in a 2 x 2 grid
  constexpr int TM = WM / 32, TN = WN / 32;
  using SA = Slab<BM, A_KMAJOR>;
  using SB = Slab<BN, B_KMAJOR>;
  constexpr int kStageElems = SA::kElems + SB::kElems;
  constexpr int kLoads = SA::kLoadsPerWave + SB::kLoadsPerWave;  // per wavefront per slab
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

  // workgroup -> output tile
  int tm, tn, bz = block_z;
  if (g.causal == kCausalKLeM || g.causal == kCausalKGeM) {
    // One-dimensional grid over (tile, matrix), longest contraction first: tile row tm
    // contracts over tm + 1 (k <= m) or tiles_m - tm (k >= m) row blocks, and a launch
    // that ends on the long tiles leaves most compute units idle meanwhile.  Matrix z
    // stays on XCD z % 8, whose L2 then keeps its small operand.
    const int t = block_x / g.nz;
    bz = block_x - t * g.nz;
    const int row = t / g.tiles_n;
    tn = t - row * g.tiles_n;
    tm = g.causal == kCausalKLeM ? g.tiles_m - 1 - row : row;
  } else if (g.causal == kCausalOutLower) {
    // square output, only tiles on or below the diagonal: t = tm (tm + 1) / 2 + tn
    const int t = block_x;
    tm = static_cast<int>((sqrtf(8.0f * static_cast<float>(t) + 1.0f) - 1.0f) * 0.5f);
    while (tm * (tm + 1) / 2 > t) --tm;
    while ((tm + 1) * (tm + 2) / 2 <= t) ++tm;
    tn = t - tm * (tm + 1) / 2;
  } else {
    // Consecutive workgroup ids land on different XCDs (round robin over 8), so give
    // each XCD a contiguous run of tiles, ordered in bands of 8 tile-rows so a band's
    // panels stay in that XCD's L2.
    const int ntiles = g.tiles_m * g.tiles_n;
    int tile = block_x;
    if (SPLITK) tile = block_x % ntiles;
    const int per_xcd = ntiles / 8;
    if (tile < per_xcd * 8) tile = (tile & 7) * per_xcd + (tile >> 3);
    constexpr int kBand = 8;
    const int band = tile / (kBand * g.tiles_n);
    const int band_rows = min(kBand, g.tiles_m - band * kBand);
    const int in_band = tile - band * kBand * g.tiles_n;
    tm = band * kBand + in_band % band_rows;
    tn = in_band / band_rows;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  // contraction range: causal products skip the slabs that are identically zero
  int k_begin = 0, k_end = g.K;
  if (g.causal == kCausalKLeM) k_end = min(g.K, m0 + BM);
  if (g.causal == kCausalKGeM) k_begin = m0;
  const int split = SPLITK ? block_x / (g.tiles_m * g.tiles_n) : 0;
  if (SPLITK) {
    k_begin = split * (g.K / g.k_splits);
    k_end = k_begin + g.K / g.k_splits;
  }
  const int z1 = bz / g.nz2, z2 = bz - z1 * g.nz2;
  const bf16_t* Abase = g.A + z1 * g.a_z1 + z2 * g.a_z2;
  const bf16_t* Bbase = g.B + z1 * g.b_z1 + z2 * g.b_z2;
  bf16_t* Cbase = g.C + z1 * g.c_z1 + z2 * g.c_z2;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

  // this lane's global source of each direct load, at slab 0
  const bf16_t* ga[SA::kLoadsPerWave];
  const bf16_t* gb[SB::kLoadsPerWave];
#pragma unroll
  for (int j = 0; j < SA::kLoadsPerWave; ++j)
    ga[j] = Abase + (A_KMAJOR ? static_cast<long long>(m0) * g.lda + k_begin
                              : static_cast<long long>(k_begin) * g.lda + m0) +
            SA::global_offset(wave, j, lane, g.lda);
#pragma unroll
  for (int j = 0; j < SB::kLoadsPerWave; ++j)
    gb[j] = Bbase + (B_KMAJOR ? static_cast<long long>(n0) * g.ldb + k_begin
                              : static_cast<long long>(k_begin) * g.ldb + n0) +
            SB::global_offset(wave, j, lane, g.ldb);
  const long long a_step = A_KMAJOR ? kBK : kBK * g.lda;  // elements per slab
  const long long b_step = B_KMAJOR ? kBK : kBK * g.ldb;

  // j-th direct load of slab kt (A pieces first, then B) -> ring stage kt % kStages
  auto issue_load = [&](int kt, int j) {
    bf16_t* sa = smem + (kt % STAGES) * kStageElems;
    if (j < SA::kLoadsPerWave) {
      __builtin_amdgcn_global_load_lds((global_void_ptr)(ga[j] + kt * a_step),
                                       (lds_void_ptr)(sa + SA::lds_offset(wave, j)), 16, 0, 0);
    } else {
      const int jb = j - SA::kLoadsPerWave;
      __builtin_amdgcn_global_load_lds((global_void_ptr)(gb[jb] + kt * b_step),
                                       (lds_void_ptr)(sa + SA::kElems + SB::lds_offset(wave, jb)), 16,
                                       0, 0);
    }
  };
  auto issue_slab = [&](int kt) {
#pragma unroll
    for (int j = 0; j < kLoads; ++j) issue_load(kt, j);
  };

  floatx16_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (k_end - k_begin) / kBK;
  // prologue: STAGES - 1 slabs in flight, the first one landed
  constexpr int kAhead = STAGES - 1;
  static_assert(kAhead == 2 || kAhead == 3, "ring depth");
  issue_slab(0);
  if (nk > 1) issue_slab(1);
  if (kAhead > 2 && nk > 2) issue_slab(2);
  if (kAhead > 2 && nk > 2) wait_vmcnt<2 * kLoads>();
  else if (nk > 1) wait_vmcnt<kLoads>();
  else wait_vmcnt<0>();
  block_barrier();

  Frag<A_KMAJOR> fa0[TM], fa1[TM];
  Frag<B_KMAJOR> fb0[TN], fb1[TN];
  {
    const bf16_t* sa = smem;
    const bf16_t* sb = sa + SA::kElems;
#pragma unroll
    for (int j = 0; j < TM; ++j) fa0[j] = SA::fragment(sa, wm0 + 32 * j, 0, lane);
#pragma unroll
    for (int i = 0; i < TN; ++i) fb0[i] = SB::fragment(sb, wn0 + 32 * i, 0, lane);
  }

  // One slab = two halves of TM x TN MFMAs.  The side work is spread between the MFMAs
  // so the matrix pipe never waits for an issue burst: during the first half the
  // second-half fragments are read and the ring stage that every wavefront finished
  // before the last barrier is refilled; then [next slab landed?] [barrier]; during the
  // second half the next slab's first-half fragments are read.  `steady` = STAGES - 1 more
  // slabs exist, so the refill and the waits need no conditions.
  constexpr int kMfmas = TM * TN;
  constexpr int kSide1 = TM + TN + kLoads;               // side operations of the first half
  constexpr int kPer1 = (kSide1 + kMfmas - 1) / kMfmas;  // per MFMA
  constexpr int kPer2 = (TM + TN + kMfmas - 1) / kMfmas;
  auto slab_step = [&](int kt, auto steady_tag) {
    constexpr bool steady = decltype(steady_tag)::value;
    const bf16_t* sa = smem + (kt % STAGES) * kStageElems;
    const bf16_t* sb = sa + SA::kElems;
    const bool refill = steady || kt + kAhead < nk;
#pragma unroll
    for (int m = 0; m < kMfmas; ++m) {
      const int i = m / TM, j = m % TM;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb0[i].operand(), fa0[j].operand(), acc[i][j], 0, 0, 0);
#pragma unroll
      for (int u = 0; u < kPer1; ++u) {
        const int op = m * kPer1 + u;
        if (op < TM) fa1[op] = SA::fragment(sa, wm0 + 32 * op, 1, lane);
        else if (op < TM + TN) fb1[op - TM] = SB::fragment(sb, wn0 + 32 * (op - TM), 1, lane);
        else if (op < kSide1) { if (refill) issue_load(kt + kAhead, op - TM - TN); }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // the next slab must have landed (two newer ones may still be in flight), and all
    // of this wavefront's reads of the current slab must be complete
    if (steady || kt + kAhead < nk) wait_vmcnt<(kAhead - 1) * kLoads>();
    else if (kAhead > 2 && kt + 2 < nk) wait_vmcnt<kLoads>();
    else wait_vmcnt<0>();
    wait_lgkmcnt0();
    block_barrier();
#pragma unroll
    for (int j = 0; j < TM; ++j) fa1[j].settle();
#pragma unroll
    for (int i = 0; i < TN; ++i) fb1[i].settle();
    const bool more = steady || kt + 1 < nk;
    const bf16_t* na = smem + ((kt + 1) % STAGES) * kStageElems;
    const bf16_t* nb = na + SA::kElems;
#pragma unroll
    for (int m = 0; m < kMfmas; ++m) {
      const int i = m / TM, j = m % TM;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb1[i].operand(), fa1[j].operand(), acc[i][j], 0, 0, 0);
#pragma unroll
      for (int u = 0; u < kPer2; ++u) {
        const int op = m * kPer2 + u;
        if (more) {
          if (op < TM) fa0[op] = SA::fragment(na, wm0 + 32 * op, 0, lane);
          else if (op < TM + TN) fb0[op - TM] = SB::fragment(nb, wn0 + 32 * (op - TM), 0, lane);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    wait_lgkmcnt0();  // the next slab's first fragments have arrived
    if (more) {
#pragma unroll
      for (int j = 0; j < TM; ++j) fa0[j].settle();
#pragma unroll
      for (int i = 0; i < TN; ++i) fb0[i].settle();
    }
  };
  wait_lgkmcnt0();
#pragma unroll
  for (int j = 0; j < TM; ++j) fa0[j].settle();
#pragma unroll
  for (int i = 0; i < TN; ++i) fb0[i].settle();
  int kt = 0;
  for (; kt + kAhead < nk; ++kt) slab_step(kt, std::true_type{});
  for (; kt < nk; ++kt) slab_step(kt, std::false_type{});

  // Epilogue.  acc[i][j][r] is the element n = wn0 + 32 i + 8 (r/4) + 4 (lane/32) + r%4,
  // m = wm0 + 32 j + lane%32.  Each wavefront rounds its quarter tile (+ bias) to bf16 into
  // its own region of the now idle LDS ring and writes it out as whole rows, 16 bytes per
  // lane.  16-byte chunks of LDS row r are XORed with r so both the 8-byte writes and the
  // 16-byte row reads spread over all banks.
  if (SPLITK) {
    // partial sums of one K range: fp32, four consecutive n per lane
    float* pw = g.partial + (static_cast<long long>(split) * g.M + m0 + wm0 + (lane & 31)) * g.N + n0 + wn0 +
                4 * (lane >> 5);
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 v = {acc[i][j][4 * q + 0], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                            acc[i][j][4 * q + 3]};
          *reinterpret_cast<float4*>(pw + static_cast<long long>(32 * j) * g.N + 32 * i + 8 * q) = v;
        }
    return;
  }
  // The bias values of this wavefront's columns, requested in one batch (one exposed L2
  // round trip instead of one per group of columns).
  uint2 braw[TN][4];
  if (g.bias != nullptr) {
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        braw[i][q] = *reinterpret_cast<const uint2*>(g.bias + n0 + wn0 + 32 * i + 8 * q + 4 * (lane >> 5));
  }
  constexpr int kRowChunks = WN / 8;
  constexpr int kRowsPerStore = kWave / kRowChunks;
  constexpr int kIters = WM / kRowsPerStore;
  // (an opaque copy of the lane index: nothing derived from it can be computed, and kept
  // in registers, ahead of the contraction loop)
  int elane = lane;
  asm volatile("" : "+v"(elane));
  const int lr = elane / kRowChunks, lc = elane % kRowChunks;
  const long long row0 = m0 + wm0;
  const int col = g.col0 + n0 + wn0 + lc * 8;  // absolute column of this lane's 8 outputs
  // Fused epilogues combine every 8 outputs with the same 8 elements of `aux`, fetched in
  // batches of 8 per lane, two batches in flight; the first is requested here, so it
  // arrives while the tile is rounded into LDS.
  constexpr int kBatch = 8;
  constexpr int kBatches = kIters / kBatch;
  static_assert(kIters % kBatch == 0, "epilogue batches");
  uintx4_t ra0[kBatch], ra1[kBatch];
  const bf16_t* auxp = g.epi != kEpiNone ? g.aux + row0 * g.aux_ld + col : nullptr;
  auto aux_load = [&](uintx4_t (&ra)[kBatch], int batch) {
#pragma unroll
    for (int k = 0; k < kBatch; ++k)
      ra[k] = *reinterpret_cast<const uintx4_t*>(
          auxp + static_cast<long long>((batch * kBatch + k) * kRowsPerStore + lr) * g.aux_ld);
  };
  if (g.epi != kEpiNone) aux_load(ra0, 0);
  block_barrier();  // every wavefront is done with the ring (no load is in flight any more)
  bf16_t* stage = smem + wave * (WM * WN);
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int nl = 32 * i + 8 * q + 4 * (lane >> 5);
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (g.bias != nullptr) {
        const uint2 b = braw[i][q];
        bv[0] = bf16_lo(b.x); bv[1] = bf16_hi(b.x); bv[2] = bf16_lo(b.y); bv[3] = bf16_hi(b.y);
      }
#pragma unroll
      for (int j = 0; j < TM; ++j) {
        const int ml = 32 * j + (lane & 31);
        uint2 o;
        o.x = pack_bf16(acc[i][j][4 * q + 0] + bv[0], acc[i][j][4 * q + 1] + bv[1]);
        o.y = pack_bf16(acc[i][j][4 * q + 2] + bv[2], acc[i][j][4 * q + 3] + bv[3]);
        const int chunk = (nl >> 3) ^ (ml & (kRowChunks - 1));
        *reinterpret_cast<uint2*>(stage + ml * WN + chunk * 8 + (nl & 7)) = o;
      }
    }
  bf16_t* cw = Cbase + static_cast<long long>(m0 + wm0) * g.ldc + n0 + wn0;
  if (g.epi == kEpiNone) {
#pragma unroll
    for (int t = 0; t < kIters; ++t) {
      const int r = t * kRowsPerStore + lr;
      const uint4 v = *reinterpret_cast<const uint4*>(stage + r * WN + ((lc ^ (r & (kRowChunks - 1))) << 3));
      *reinterpret_cast<uint4*>(cw + static_cast<long long>(r) * g.ldc + lc * 8) = v;
    }
    return;
  }
  float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (g.epi == kEpiBiasDropoutAdd) load8(g.vec + col, bv);
  float colacc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  auto finish = [&](const uintx4_t (&ra)[kBatch], int batch) {
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const int r = (batch * kBatch + k) * kRowsPerStore + lr;
      Raw8<bf16_t> pv, xv;
      pv.v = *reinterpret_cast<const uint4*>(stage + r * WN + ((lc ^ (r & (kRowChunks - 1))) << 3));
      xv.v = make_uint4(ra[k][0], ra[k][1], ra[k][2], ra[k][3]);
      float prod[8], x[8], o[8];
      unpack(pv, prod);
      unpack(xv, x);
      if (g.epi == kEpiBiasDropoutAdd) {
        if (g.plain != nullptr)
          *reinterpret_cast<uint4*>(g.plain + (row0 + r) * g.ldc + col) = pv.v;
        const uint64_t elem = static_cast<uint64_t>(row0 + r) * static_cast<uint64_t>(g.row_len) + col;
        bias_dropout_add8(prod, bv, x, g.key, elem >> 3, o);
      } else {
        gelu_bwd8<bf16_t>(prod, x, o);
#pragma unroll
        for (int i = 0; i < 8; ++i) colacc[i] += o[i];
      }
      store8(cw + static_cast<long long>(r) * g.ldc + lc * 8, o);
    }
  };
  if (kBatches > 1) aux_load(ra1, 1);
  for (int bt = 0; bt < kBatches; bt += 2) {
    finish(ra0, bt);
    if (bt + 2 < kBatches) aux_load(ra0, bt + 2);
    if (bt + 1 < kBatches) {
      finish(ra1, bt + 1);
      if (bt + 3 < kBatches) aux_load(ra1, bt + 3);
    }
  }
  if (g.epi == kEpiGeluBwd) {
    // column sums of this wavefront's WM rows: lanes with the same lc hold different rows
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int o = kRowChunks; o < kWave; o <<= 1) colacc[i] += __shfl_xor(colacc[i], o, kWave);
    if (lane < kRowChunks)
      store8(g.colsum_partial + (row0 / WM) * g.row_len + col, colacc);
  }
}

template <bool A_KMAJOR, bool B_KMAJOR, int BM, int BN>
__global__ void __launch_bounds__(kThreads) gemm_mfma_kernel(MfmaGemmArgs g) {
  gemm_tile<A_KMAJOR, B_KMAJOR, BM, BN>(g, blockIdx.x, blockIdx.y);
}

// 256 x 128 tiles with a three-stage ring (72 KB) and at most 256 registers, so that two
// workgroups share a compute unit: for launches whose store pass is long (bias + dropout +
// residual: one Philox call per 8 outputs, about as long as a 20-slab contraction), one
// workgroup's store pass then runs on the vector ALUs while the other's contraction keeps
// the matrix cores busy.
constexpr int kDuoStages = 3;
// contractions up to this length take the two-workgroup form (measured at the 13B shard: the
// attention projection, K = 640, 0.198 -> 0.178 ms; FC2, K = 2560, 0.442 -> 0.461 ms: there the
// larger tile's lower LDS and L2 traffic wins over the overlapped store pass)
constexpr int kDuoMaxK = 1024;
template <bool A_KMAJOR, bool B_KMAJOR>
__global__ void __launch_bounds__(kThreads, 2) gemm_mfma_duo_kernel(MfmaGemmArgs g) {
  gemm_tile<A_KMAJOR, B_KMAJOR, 256, 128, false, kDuoStages>(g, blockIdx.x, blockIdx.y);
}

// Work items of the score-shaped row-block kernels: row block tm (128 rows) owns tiles
// tn = 0..tm; it is cut into runs of at most kAttnRun tiles, one workgroup each, so that no
// workgroup walks more than kAttnRun tiles (a workgroup per whole row block leaves the launch
// waiting for the 16-tile blocks while most compute units have run out of work).  Items are
// numbered longest row block first; item * nz + z is the workgroup of matrix z.
constexpr int kAttnRun = 4;
__host__ __device__ inline int attn_runs_of(int tm) { return (tm + kAttnRun) / kAttnRun; }
inline int attn_items(int tiles_m) {
  int n = 0;
  for (int tm = 0; tm < tiles_m; ++tm) n += attn_runs_of(tm);
  return n;
}
// item -> (tm, first tile, one past the last tile)
__device__ __forceinline__ void attn_item(int item, int tiles_m, int& tm, int& tn0, int& tn1) {
  tm = tiles_m - 1;
  while (tm > 0 && item >= attn_runs_of(tm)) {
    item -= attn_runs_of(tm);
    --tm;
  }
  tn0 = item * kAttnRun;
  tn1 = min(tn0 + kAttnRun, tm + 1);
}

// Score-shaped batched products with a short contraction (S = Q K^T, dPd = dC V^T: K = head
// dimension), lower triangle only.  A tile of such a product is all latency: load two small
// operand tiles, 32 MFMAs per wavefront, store 32 KB.  Here a workgroup owns a run of tiles of
// one block of 128 rows of one matrix: the A tile stays in LDS; the one B buffer doubles as
// the staging area of the store pass, the next B tile is requested as soon as every wavefront
// has its rows back in registers, and the stores are never waited for.  At 64 KB of LDS (head
// dimension 128) two workgroups share a compute unit: one loads and stores while the other
// multiplies.
template <int KD>
__global__ void __launch_bounds__(kThreads, 2) attn_outer_kernel(MfmaGemmArgs g) {
  constexpr int WM = 64, WN = 64, TM = 2, TN = 2;
  constexpr int kSlabs = KD / kBK;
  using SL = Slab<128, true>;
  constexpr int kOpElems = kSlabs * SL::kElems;       // one 128 x KD operand tile
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);
  bf16_t* sB = sA + kOpElems;                           // B tile, then 4 x (64 x 64) of staging

  const int item = blockIdx.x / g.nz;
  const int bz = blockIdx.x - item * g.nz;
  int tm, tn0, tn1;
  attn_item(item, g.tiles_m, tm, tn0, tn1);
  const int z1 = bz / g.nz2, z2 = bz - z1 * g.nz2;
  const bf16_t* Abase = g.A + z1 * g.a_z1 + z2 * g.a_z2 + static_cast<long long>(tm) * 128 * g.lda;
  const bf16_t* Bbase = g.B + z1 * g.b_z1 + z2 * g.b_z2;
  bf16_t* Cbase = g.C + z1 * g.c_z1 + z2 * g.c_z2 + static_cast<long long>(tm) * 128 * g.ldc;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

  long long offA[SL::kLoadsPerWave], offB[SL::kLoadsPerWave];
#pragma unroll
  for (int j = 0; j < SL::kLoadsPerWave; ++j) {
    offA[j] = SL::global_offset(wave, j, lane, g.lda);
    offB[j] = SL::global_offset(wave, j, lane, g.ldb);
  }
  auto load_tile = [&](const bf16_t* src, const long long (&off)[SL::kLoadsPerWave], bf16_t* dst) {
#pragma unroll
    for (int sl = 0; sl < kSlabs; ++sl)
#pragma unroll
      for (int j = 0; j < SL::kLoadsPerWave; ++j)
        __builtin_amdgcn_global_load_lds((global_void_ptr)(src + off[j] + sl * kBK),
                                         (lds_void_ptr)(dst + sl * SL::kElems + SL::lds_offset(wave, j)), 16, 0, 0);
  };
  load_tile(Abase, offA, sA);
  load_tile(Bbase + static_cast<long long>(tn0) * 128 * g.ldb, offB, sB);

  constexpr int kRowChunks = WN / 8;                    // 8
  constexpr int kRowsPerStore = kWave / kRowChunks;     // 8
  constexpr int kStores = WM / kRowsPerStore;           // 8 stores per wavefront per tile
  bf16_t* stage = sB + wave * (WM * WN);
  const int lr = lane / kRowChunks, lc = lane % kRowChunks;

  for (int tn = tn0; tn < tn1; ++tn) {
    // B(tn) (and, the first time, A) has landed: everything older than the previous tile's stores
    if (tn == tn0) wait_vmcnt<0>();
    else wait_vmcnt<kStores>();
    block_barrier();

    floatx16_t acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KD / 16; ++kk) {
      Frag<true> fa[TM], fb[TN];
#pragma unroll
      for (int j = 0; j < TM; ++j) fa[j] = SL::fragment(sA + (kk >> 1) * SL::kElems, wm0 + 32 * j, kk & 1, lane);
#pragma unroll
      for (int i = 0; i < TN; ++i) fb[i] = SL::fragment(sB + (kk >> 1) * SL::kElems, wn0 + 32 * i, kk & 1, lane);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i].operand(), fa[j].operand(), acc[i][j], 0, 0, 0);
    }
    block_barrier();  // every wavefront has read B(tn): its buffer becomes the staging area
    // round into this wavefront's staging region, then whole rows back, 16 bytes per lane
    // (acc[i][j][r]: n = wn0 + 32 i + 8 (r / 4) + 4 (lane / 32) + r % 4, m = wm0 + 32 j + lane % 32)
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nl = 32 * i + 8 * q + 4 * (lane >> 5);
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          const int ml = 32 * j + (lane & 31);
          uintx2_t o;
          o[0] = pack_bf16(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1]);
          o[1] = pack_bf16(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
          const int chunk = (nl >> 3) ^ (ml & (kRowChunks - 1));
          // As inline assembly: a store to LDS that the compiler sees is made to wait for
          // every direct-to-LDS load in flight and, with them, for the previous tile's
          // stores.  LDS executes a wavefront's accesses in order, so the row reads below
          // see these writes.
          typedef __attribute__((address_space(3))) bf16_t* lds_ptr_t;
          const uint32_t addr = static_cast<uint32_t>(
              reinterpret_cast<uintptr_t>((lds_ptr_t)(stage + ml * WN + chunk * 8 + (nl & 7))));
          asm volatile("ds_write_b64 %0, %1" : : "v"(addr), "v"(o) : "memory");
        }
      }
    uintx4_t rows[kStores];
#pragma unroll
    for (int u = 0; u < kStores; ++u) {
      const int r = u * kRowsPerStore + lr;
      typedef const __attribute__((address_space(3))) bf16_t* lds_cptr_t;
      const uint32_t addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
          (lds_cptr_t)(stage + r * WN + ((lc ^ (r & (kRowChunks - 1))) << 3))));
      asm volatile("ds_read_b128 %0, %1" : "=v"(rows[u]) : "v"(addr) : "memory");
    }
    wait_lgkmcnt0();
#pragma unroll
    for (int u = 0; u < kStores; ++u) asm volatile("" : "+v"(rows[u]));
    block_barrier();  // every wavefront has its rows: the buffer can take the next B tile
    if (tn + 1 < tn1) load_tile(Bbase + static_cast<long long>(tn + 1) * 128 * g.ldb, offB, sB);
    bf16_t* cw = Cbase + static_cast<long long>(wm0) * g.ldc + tn * 128 + wn0;
#pragma unroll
    for (int u = 0; u < kStores; ++u) {
      const int r = u * kRowsPerStore + lr;
      __builtin_nontemporal_store(rows[u], reinterpret_cast<uintx4_t*>(cw + static_cast<long long>(r) * g.ldc + lc * 8));
    }
  }
}

// dS from dC, V and P in one launch: the score-shaped product dPd = dC V^T with the backward
// of dropout and softmax (B5 + B4) in its store pass, so dPd is never written:
//   dS = scale P (keep c round(dPd) - dot),  dot_i = sum_j dP_ij P_ij.
// The row dot product comes in from a small kernel that forms it as sum_dd dC[i, dd] C[i, dd]
// (= sum_j dPd_ij Pd_ij since Pd V = C: the same number up to the rounding of Pd and dPd), so
// one pass over the tiles suffices.  Same walk as attn_outer_kernel (a workgroup owns a block
// of 128 rows, the A tile stays in LDS), but the store pass is long here (a Philox call per
// 8 elements), so: one B buffer, which doubles as the staging area; the next B tile and the
// next tile's vectors of P are requested just before the store pass and arrive during it;
// and the 64 KB of LDS let two workgroups share a compute unit.  The loads of P are inline
// assembly with waits counted by hand: loads the compiler tracks would be waited for at
// the loop's back edge together with everything issued after them.
template <int KD>
__global__ void __launch_bounds__(kThreads, 2) attn_dscores_kernel(MfmaGemmArgs g) {
  constexpr int WM = 64, WN = 64, TM = 2, TN = 2;
  constexpr int kSlabs = KD / kBK;
  using SL = Slab<128, true>;
  constexpr int kOpElems = kSlabs * SL::kElems;  // one 128 x KD operand tile
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);
  bf16_t* sB = sA + kOpElems;
  static_assert(kOpElems >= 4 * WM * WN || KD < 128, "staging fits the B buffer");

  const int item = blockIdx.x / g.nz;
  const int bz = blockIdx.x - item * g.nz;
  int tm, tn0, tn1;
  attn_item(item, g.tiles_m, tm, tn0, tn1);
  const int z1 = bz / g.nz2, z2 = bz - z1 * g.nz2;
  const bf16_t* Abase = g.A + z1 * g.a_z1 + z2 * g.a_z2 + static_cast<long long>(tm) * 128 * g.lda;
  const bf16_t* Bbase = g.B + z1 * g.b_z1 + z2 * g.b_z2;
  bf16_t* Cbase = g.C + z1 * g.c_z1 + z2 * g.c_z2 + static_cast<long long>(tm) * 128 * g.ldc;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

  long long offA[SL::kLoadsPerWave], offB[SL::kLoadsPerWave];
#pragma unroll
  for (int j = 0; j < SL::kLoadsPerWave; ++j) {
    offA[j] = SL::global_offset(wave, j, lane, g.lda);
    offB[j] = SL::global_offset(wave, j, lane, g.ldb);
  }
  auto load_tile = [&](const bf16_t* src, const long long (&off)[SL::kLoadsPerWave], bf16_t* dst) {
#pragma unroll
    for (int sl = 0; sl < kSlabs; ++sl)
#pragma unroll
      for (int j = 0; j < SL::kLoadsPerWave; ++j)
        __builtin_amdgcn_global_load_lds((global_void_ptr)(src + off[j] + sl * kBK),
                                         (lds_void_ptr)(dst + sl * SL::kElems + SL::lds_offset(wave, j)), 16, 0, 0);
  };
  constexpr int kTileLoads = kSlabs * SL::kLoadsPerWave;  // direct loads per wavefront per tile
  load_tile(Abase, offA, sA);
  load_tile(Bbase + static_cast<long long>(tn0) * 128 * g.ldb, offB, sB);

  constexpr int kRowChunks = WN / 8;                 // 8
  constexpr int kRowsPerStore = kWave / kRowChunks;  // 8
  constexpr int kStores = WM / kRowsPerStore;        // 8 rows of P / stores per lane per tile
  bf16_t* stage = sB + wave * (WM * WN);
  const int lr = lane / kRowChunks, lc = lane % kRowChunks;

  // this lane's eight rows: dot products, dropout indices, vectors of P (two sets)
  const bf16_t* Pw = g.aux + z1 * g.c_z1 + z2 * g.c_z2 + static_cast<long long>(tm * 128 + wm0) * g.ldc + wn0 + lc * 8;
  const uint64_t rows_before = (static_cast<uint64_t>(z1) * g.global_heads + g.head0 + z2) * g.M;
  float dot[kStores];
  uint64_t gidx[kStores];
  uintx4_t p0[kStores], p1[kStores];
  auto request_p = [&](int tn, uintx4_t (&pv)[kStores]) {
#pragma unroll
    for (int u = 0; u < kStores; ++u) {
      const bf16_t* src = Pw + static_cast<long long>(u * kRowsPerStore + lr) * g.ldc + tn * 128;
      asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(pv[u]) : "v"(src) : "memory");
    }
  };
  request_p(tn0, p0);
#pragma unroll
  for (int u = 0; u < kStores; ++u) {
    const int i = tm * 128 + wm0 + u * kRowsPerStore + lr;
    dot[u] = g.rowdot[static_cast<long long>(bz) * g.M + i];
    gidx[u] = (rows_before + i) * static_cast<uint64_t>(g.N) + wn0 + lc * 8;
  }
  // (a use: the compiler waits for these loads here, once, and tracks nothing into the loop)
#pragma unroll
  for (int u = 0; u < kStores; ++u) asm volatile("" : "+v"(dot[u]));

  // One tile; `pc` holds this tile's vectors of P, `pn` receives the next tile's.
  auto tile_step = [&](const int tn, uintx4_t (&pc)[kStores], uintx4_t (&pn)[kStores]) {
    // B(tn) has landed.  Issued after it: the previous step's requests for P and its stores
    // (nothing the first time, when everything issued so far is waited for).
    if (tn == tn0) wait_vmcnt<0>();
    else wait_vmcnt<2 * kStores>();
    block_barrier();
    floatx16_t acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KD / 16; ++kk) {
      Frag<true> fa[TM], fb[TN];
#pragma unroll
      for (int j = 0; j < TM; ++j) fa[j] = SL::fragment(sA + (kk >> 1) * SL::kElems, wm0 + 32 * j, kk & 1, lane);
#pragma unroll
      for (int i = 0; i < TN; ++i) fb[i] = SL::fragment(sB + (kk >> 1) * SL::kElems, wn0 + 32 * i, kk & 1, lane);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i].operand(), fa[j].operand(), acc[i][j], 0, 0, 0);
    }
    block_barrier();  // every wavefront has read B(tn): its buffer becomes the staging area
    // round into this wavefront's quarter, read whole rows back, 16 bytes per lane
    // (acc[i][j][r]: n = wn0 + 32 i + 8 (r / 4) + 4 (lane / 32) + r % 4, m = wm0 + 32 j + lane % 32)
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nl = 32 * i + 8 * q + 4 * (lane >> 5);
#pragma unroll
        for (int j = 0; j < TM; ++j) {
          const int ml = 32 * j + (lane & 31);
          uintx2_t o;
          o[0] = pack_bf16(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1]);
          o[1] = pack_bf16(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
          const int chunk = (nl >> 3) ^ (ml & (kRowChunks - 1));
          typedef __attribute__((address_space(3))) bf16_t* lds_ptr_t;
          const uint32_t addr = static_cast<uint32_t>(
              reinterpret_cast<uintptr_t>((lds_ptr_t)(stage + ml * WN + chunk * 8 + (nl & 7))));
          asm volatile("ds_write_b64 %0, %1" : : "v"(addr), "v"(o) : "memory");
        }
      }
    uintx4_t rows[kStores];
#pragma unroll
    for (int u = 0; u < kStores; ++u) {
      const int r = u * kRowsPerStore + lr;
      typedef const __attribute__((address_space(3))) bf16_t* lds_cptr_t;
      const uint32_t addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
          (lds_cptr_t)(stage + r * WN + ((lc ^ (r & (kRowChunks - 1))) << 3))));
      asm volatile("ds_read_b128 %0, %1" : "=v"(rows[u]) : "v"(addr) : "memory");
    }
    wait_lgkmcnt0();
#pragma unroll
    for (int u = 0; u < kStores; ++u) asm volatile("" : "+v"(rows[u]));
    block_barrier();  // every wavefront has its rows: the buffer can take the next B tile
    if (tn + 1 < tn1) {
      load_tile(Bbase + static_cast<long long>(tn + 1) * 128 * g.ldb, offB, sB);
      request_p(tn + 1, pn);
    }
    // this tile's P: requested a step ago; issued since: the previous step's stores and, if
    // there is a next tile, its B tile and its P
    if (tn == tn0) {
      // (waited for at the top)
    } else if (tn + 1 < tn1) {
      wait_vmcnt<2 * kStores + kTileLoads>();
    } else {
      wait_vmcnt<kStores>();
    }
    bf16_t* cw = Cbase + static_cast<long long>(wm0) * g.ldc + tn * 128 + wn0;
#pragma unroll
    for (int u = 0; u < kStores; ++u) {
      asm volatile("" : "+v"(pc[u]));
      const int r = u * kRowsPerStore + lr;
      Raw8<bf16_t> dv, pv;
      dv.v = make_uint4(rows[u][0], rows[u][1], rows[u][2], rows[u][3]);
      pv.v = make_uint4(pc[u][0], pc[u][1], pc[u][2], pc[u][3]);
      float dp[8], pr[8], ds[8];
      unpack(dv, dp);
      unpack(pv, pr);
      dropout_apply8(g.key, (gidx[u] + tn * 128) >> 3, dp);
#pragma unroll
      for (int k = 0; k < 8; ++k) ds[k] = g.scale * (pr[k] * (dp[k] - dot[u]));
      store8(cw + static_cast<long long>(r) * g.ldc + lc * 8, ds);
    }
  };
  // two tiles per trip, so the two sets of P registers swap roles without being copied
  for (int tn = tn0; tn < tn1; tn += 2) {
    tile_step(tn, p0, p1);
    if (tn + 1 < tn1) tile_step(tn + 1, p1, p0);
  }
}

// An output whose width is an odd multiple of 128: 256 x 256 tiles over the columns that
// whole tiles cover, and one column of 256 x 128 tiles (`edge`: the same product on the last
// 128 columns) behind them in the same launch, where they fill the last round of workgroups.
template <bool A_KMAJOR, bool B_KMAJOR>
__global__ void __launch_bounds__(kThreads)
gemm_mfma_edge_kernel(MfmaGemmArgs body, MfmaGemmArgs edge, int n_body) {
  if (static_cast<int>(blockIdx.x) < n_body) gemm_tile<A_KMAJOR, B_KMAJOR, 256, 256>(body, blockIdx.x, 0);
  else gemm_tile<A_KMAJOR, B_KMAJOR, 256, 128>(edge, blockIdx.x - n_body, 0);
}

// The two products of a linear layer's backward in one launch: the weight gradient
// (both operands MN-major, long contraction over the tokens) takes the first n_w
// workgroups, the input gradient (weight MN-major) the rest.  Sharing a launch lets
// the second product's tiles fill the compute units the first leaves idle in its
// last, partial round.  When one side of the weight gradient is an odd multiple of 128,
// its 256 x 256 tiles cover all but the last 128 rows (or columns) and `wedge`, the same
// product on that strip with EBM x EBN tiles, takes the n_e workgroups after them.
template <int DBM, int DBN, int WBM, int WBN, int EBM, int EBN>
__global__ void __launch_bounds__(kThreads)
gemm_mfma_pair_kernel(MfmaGemmArgs wgrad, MfmaGemmArgs wedge, MfmaGemmArgs dgrad, int n_w, int n_e) {
  const int x = static_cast<int>(blockIdx.x);
  // the input gradient starts at a multiple of 8 workgroups, so that its tile order, which
  // takes workgroup id mod 8 for the XCD, still holds; the few workgroups in between idle
  const int n_pad = (n_w + n_e + 7) & ~7;
  if (x < n_w) {
    if (wgrad.k_splits > 1) gemm_tile<false, false, WBM, WBN, true>(wgrad, x, 0);
    else gemm_tile<false, false, WBM, WBN>(wgrad, x, 0);
  } else if (EBM != 0 && x < n_w + n_e) {
    if constexpr (EBM != 0) gemm_tile<false, false, EBM, EBN>(wedge, x - n_w, 0);
  } else if (x >= n_pad) {
    gemm_tile<true, false, DBM, DBN>(dgrad, x - n_pad, 0);
  }
}

// C[m][n] = round(sum over the K ranges, in range order, of partial[split][m][n]).
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float* __restrict__ partial, bf16_t* __restrict__ C, int M, int N, long long ldc,
                     int k_splits) {
  const long long v = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;  // 8 consecutive n
  const int per_row = N / 8;
  if (v >= static_cast<long long>(M) * per_row) return;
  const int m = static_cast<int>(v / per_row), n = static_cast<int>(v - static_cast<long long>(m) * per_row) * 8;
  const float* p = partial + static_cast<long long>(m) * N + n;
  float4 lo = *reinterpret_cast<const float4*>(p), hi = *reinterpret_cast<const float4*>(p + 4);
  for (int sp = 1; sp < k_splits; ++sp) {
    p += static_cast<long long>(M) * N;
    const float4 l2 = *reinterpret_cast<const float4*>(p), h2 = *reinterpret_cast<const float4*>(p + 4);
    lo.x += l2.x; lo.y += l2.y; lo.z += l2.z; lo.w += l2.w;
    hi.x += h2.x; hi.y += h2.y; hi.z += h2.z; hi.w += h2.w;
  }
  uint4 o;
  o.x = pack_bf16(lo.x, lo.y); o.y = pack_bf16(lo.z, lo.w);
  o.z = pack_bf16(hi.x, hi.y); o.w = pack_bf16(hi.z, hi.w);
  *reinterpret_cast<uint4*>(C + static_cast<long long>(m) * ldc + n) = o;
}

// Raises a kernel's dynamic LDS limit, once per call site (i.e. per kernel instantiation) and
// safely when several host threads drive different layers at the same time.
#define LYNX_RAISE_LDS_LIMIT(kern, smem)                                                        \
  do {                                                                                          \
    static std::once_flag once_;                                                                \
    static hipError_t err_ = hipSuccess;                                                        \
    std::call_once(once_, [&] {                                                                 \
      err_ = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                           \
                                 hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem)); \
    });                                                                                         \
    if (err_ != hipSuccess) return err_;                                                        \
  } while (0)

template <bool AK, bool BK_, int BM, int BN>
hipError_t launch(const MfmaGemmArgs& a, hipStream_t st) {
  constexpr size_t smem = static_cast<size_t>(kStages) * (BM + BN) * kBK * sizeof(bf16_t);
  auto kern = gemm_mfma_kernel<AK, BK_, BM, BN>;
  LYNX_RAISE_LDS_LIMIT(kern, smem);
  const int ntiles = a.causal == kCausalOutLower ? a.tiles_m * (a.tiles_m + 1) / 2 : a.tiles_m * a.tiles_n;
  const bool flat = a.causal == kCausalKLeM || a.causal == kCausalKGeM;  // (tile, matrix) in x
  hipLaunchKernelGGL(kern, flat ? dim3(ntiles * a.nz) : dim3(ntiles, a.nz), dim3(kThreads), smem, st, a);
  return hipGetLastError();
}

template <bool AK, bool BK_>
hipError_t launch_duo(MfmaGemmArgs a, hipStream_t st) {
  constexpr size_t smem = static_cast<size_t>(kDuoStages) * (256 + 128) * kBK * sizeof(bf16_t);
  auto kern = gemm_mfma_duo_kernel<AK, BK_>;
  LYNX_RAISE_LDS_LIMIT(kern, smem);
  a.tiles_m = a.M / 256;
  a.tiles_n = a.N / 128;
  hipLaunchKernelGGL(kern, dim3(a.tiles_m * a.tiles_n, a.nz), dim3(kThreads), smem, st, a);
  return hipGetLastError();
}

template <bool AK, bool BK_>
hipError_t launch_edge(const MfmaGemmArgs& a, hipStream_t st) {
  constexpr size_t smem = static_cast<size_t>(kStages) * (256 + 256) * kBK * sizeof(bf16_t);
  auto kern = gemm_mfma_edge_kernel<AK, BK_>;
  LYNX_RAISE_LDS_LIMIT(kern, smem);
  MfmaGemmArgs body = a, edge = a;
  const int n_body_cols = a.N - 128;
  body.N = n_body_cols;
  body.tiles_m = a.M / 256; body.tiles_n = n_body_cols / 256;
  edge.N = 128;
  edge.tiles_m = a.M / 256; edge.tiles_n = 1;
  edge.B = a.B + (BK_ ? static_cast<long long>(n_body_cols) * a.ldb : static_cast<long long>(n_body_cols));
  edge.C = a.C + n_body_cols;
  if (a.bias != nullptr) edge.bias = a.bias + n_body_cols;
  edge.col0 = a.col0 + n_body_cols;
  const int n_body = body.tiles_m * body.tiles_n;
  hipLaunchKernelGGL(kern, dim3(n_body + edge.tiles_m), dim3(kThreads), smem, st, body, edge, n_body);
  return hipGetLastError();
}

template <int KD>
hipError_t launch_attn_outer(MfmaGemmArgs a, hipStream_t st) {
  // A tile + the B tile / staging area (4 x 64 x 64, the larger of the two for short head dimensions)
  constexpr size_t op = static_cast<size_t>(KD / kBK) * 128 * kBK;
  constexpr size_t smem = (op + (op > 4 * 64 * 64 ? op : 4 * 64 * 64)) * sizeof(bf16_t);
  auto kern = attn_outer_kernel<KD>;
  LYNX_RAISE_LDS_LIMIT(kern, smem);
  a.tiles_m = a.M / 128;
  a.tiles_n = a.N / 128;
  hipLaunchKernelGGL(kern, dim3(attn_items(a.tiles_m) * a.nz), dim3(kThreads), smem, st, a);
  return hipGetLastError();
}

template <int KD>
hipError_t launch_attn_dscores(MfmaGemmArgs a, hipStream_t st) {
  constexpr size_t smem = 2 * static_cast<size_t>(KD / kBK) * 128 * kBK * sizeof(bf16_t);
  auto kern = attn_dscores_kernel<KD>;
  LYNX_RAISE_LDS_LIMIT(kern, smem);
  a.tiles_m = a.M / 128;
  a.tiles_n = a.N / 128;
  hipLaunchKernelGGL(kern, dim3(attn_items(a.tiles_m) * a.nz), dim3(kThreads), smem, st, a);
  return hipGetLastError();
}

// Tile shape: the largest tile that divides the output, unless a smaller one
// fills the 256 compute units markedly better (fewer idle units in the last
// round of workgroups).
template <bool AK, bool BK_>
hipError_t launch_tiles(MfmaGemmArgs a, hipStream_t st) {
  if (a.causal == kCausalOutLower && AK && BK_ && a.bias == nullptr && a.epi == kEpiNone) {
    if (a.K == 128) return launch_attn_outer<128>(a, st);
    if (a.K == 64) return launch_attn_outer<64>(a, st);
  }
  if (a.epi == kEpiSoftmaxBwd) return launch_attn_dscores<128>(a, st);  // gemm_mfma_supported: K = 128
  if (a.causal != kCausalNone) {
    // attention products: memory-bound.  128 x 128 tiles: the zero padding of the
    // seq x seq operands reaches the next multiple of 128 only, two workgroups fit a
    // compute unit (one loads while the other stores), and the score-shaped products
    // write less beyond the diagonal
    a.tiles_m = a.M / 128;
    a.tiles_n = a.N / 128;
    return launch<AK, BK_, 128, 128>(a, st);
  }
  if (a.epi == kEpiBiasDropoutAdd && a.nz == 1 && a.M % 256 == 0 && a.N % 128 == 0 && a.K <= kDuoMaxK)
    return launch_duo<AK, BK_>(a, st);
  if (a.nz == 1 && a.M % 256 == 0 && a.N % 256 == 128 && (a.M / 256) * (a.N / 256 + 1) >= 128)
    return launch_edge<AK, BK_>(a, st);
  struct Cand { int bm, bn; float weight; };
  static const Cand cands[4] = {{256, 256, 1.0f}, {256, 128, 0.8f}, {128, 256, 0.8f}, {128, 128, 0.6f}};
  int best = -1;
  float best_score = 0.f;
  for (int c = 0; c < 4; ++c) {
    if (a.M % cands[c].bm || a.N % cands[c].bn) continue;
    const long long nt = static_cast<long long>(a.M / cands[c].bm) * (a.N / cands[c].bn);
    const long long rounds = (nt + 255) / 256;
    const float score = cands[c].weight * static_cast<float>(nt) / static_cast<float>(rounds * 256);
    if (score > best_score) { best_score = score; best = c; }
  }
  if (best < 0) return hipErrorInvalidValue;
  a.tiles_m = a.M / cands[best].bm;
  a.tiles_n = a.N / cands[best].bn;
  switch (best) {
    case 0: return launch<AK, BK_, 256, 256>(a, st);
    case 1: return launch<AK, BK_, 256, 128>(a, st);
    case 2: return launch<AK, BK_, 128, 256>(a, st);
    default: return launch<AK, BK_, 128, 128>(a, st);
  }
}

// How a pair is launched.  Tiles: the largest that divides the output (pair launches
// share their tail, so there is no reason to shrink tiles for occupancy); a weight gradient
// with one side an odd multiple of 128 and at least half a round of whole tiles gets
// 256 x 256 tiles plus an edge strip.  K ranges (1 or 2) of the weight gradient: its tiles
// contract over all tokens and are few; when one of them lasts longer than nine tenths
// of the launch's ideal duration, the compute units that have finished the input gradient
// wait for it, and halving it pays for the extra pass over the fp32 partial sums (measured:
// 10-30 % on the attention-projection shapes; finer cuts and cuts of the wide layers lose
// to that pass).  Durations in slab units: 1 per slab for a 256 x 256 tile, about 0.55 for
// the narrower ones.
struct PairPlan {
  int dbm, dbn;      // input-gradient tile
  int wbm, wbn;      // weight-gradient tile
  int edge;          // 0 none, 1 last 128 rows (128 x 256 tiles), 2 last 128 columns (256 x 128)
  int k_splits;
};

PairPlan plan_pair(int wM, int wN, int wK, int dM, int dN, int dK) {
  PairPlan p{};
  p.dbm = dM % 256 == 0 ? 256 : 128;
  p.dbn = dN % 256 == 0 ? 256 : 128;
  p.wbm = wM % 256 == 0 ? 256 : 128;
  p.wbn = wN % 256 == 0 ? 256 : 128;
  if (wM % 256 == 128 && wN % 256 == 0 && (wM / 256) * (wN / 256) >= 128) { p.edge = 1; p.wbm = 256; }
  else if (wN % 256 == 128 && wM % 256 == 0 && (wM / 256) * (wN / 256) >= 128) { p.edge = 2; p.wbn = 256; }
  auto cost = [](int bm, int bn) { return (bm == 256 && bn == 256) ? 1.0 : 0.55; };
  const double slabs_w = wK / kBK, slabs_d = dK / kBK;
  double work_w, longest;
  if (p.edge == 0) {
    work_w = static_cast<double>(wM / p.wbm) * (wN / p.wbn) * slabs_w * cost(p.wbm, p.wbn);
    longest = slabs_w * cost(p.wbm, p.wbn);
  } else {
    const double body = static_cast<double>(wM / 256) * (wN / 256);
    const double strip = p.edge == 1 ? wN / 256 : wM / 256;
    work_w = (body + strip * 0.55) * slabs_w;
    longest = slabs_w;
  }
  const double work_d = static_cast<double>(dM / p.dbm) * (dN / p.dbn) * slabs_d * cost(p.dbm, p.dbn);
  const double ideal = (work_w + work_d) / 256.0;
  // (a weight gradient with an edge strip is never cut: with half a round of whole tiles or
  // more its tiles are not the ones the launch waits for)
  const bool cut = p.edge == 0 && wK % (2 * kBK) == 0 && wK >= 2048 && longest > kPairCutFraction * ideal;
  p.k_splits = cut ? 2 : 1;
  return p;
}

template <int DBM, int DBN, int WBM, int WBN, int EBM, int EBN>
hipError_t launch_pair(MfmaGemmArgs w, MfmaGemmArgs d, const PairPlan& plan, hipStream_t st) {
  constexpr int dsum = DBM + DBN, wsum = WBM + WBN;
  constexpr size_t smem = static_cast<size_t>(kStages) * (dsum > wsum ? dsum : wsum) * kBK * sizeof(bf16_t);
  auto kern = gemm_mfma_pair_kernel<DBM, DBN, WBM, WBN, EBM, EBN>;
  LYNX_RAISE_LDS_LIMIT(kern, smem);
  // the edge strip: the same product restricted to the last 128 rows or columns of dW
  MfmaGemmArgs e = w;
  int n_e = 0;
  if (EBM != 0) {
    if (plan.edge == 1) {
      const int body_rows = w.M - 128;
      e.A = w.A + body_rows;  // A is MN-major: column m of the stored [K, M] array
      e.C = w.C + static_cast<long long>(body_rows) * w.ldc;
      e.M = 128;
      w.M = body_rows;
    } else {
      const int body_cols = w.N - 128;
      e.B = w.B + body_cols;
      e.C = w.C + body_cols;
      e.N = 128;
      w.N = body_cols;
    }
    e.tiles_m = e.M / EBM; e.tiles_n = e.N / EBN;
    n_e = e.tiles_m * e.tiles_n;
  }
  w.tiles_m = w.M / WBM; w.tiles_n = w.N / WBN;
  d.tiles_m = d.M / DBM; d.tiles_n = d.N / DBN;
  const int n_w = w.tiles_m * w.tiles_n * w.k_splits;
  const int n_pad = (n_w + n_e + 7) & ~7;
  hipLaunchKernelGGL(kern, dim3(n_pad + d.tiles_m * d.tiles_n), dim3(kThreads), smem, st, w, e, d, n_w, n_e);
  if (w.k_splits > 1) {
    const long long vecs = static_cast<long long>(w.M) * (w.N / 8);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(static_cast<unsigned>((vecs + 255) / 256)), dim3(256), 0, st,
                       w.partial, w.C, w.M, w.N, w.ldc, w.k_splits);
  }
  return hipGetLastError();
}

MfmaGemmArgs make_args(const GemmDesc& d) {
  MfmaGemmArgs a{};
  const bool a_k = d.a_sk == 1, b_k = d.b_sk == 1;
  a.A = static_cast<const bf16_t*>(d.A); a.lda = a_k ? d.a_sm : d.a_sk;
  a.B = static_cast<const bf16_t*>(d.B); a.ldb = b_k ? d.b_sn : d.b_sk;
  a.C = static_cast<bf16_t*>(d.C); a.ldc = d.c_sm;
  a.bias = static_cast<const bf16_t*>(d.bias);
  a.M = d.M; a.N = d.N; a.K = d.K;
  a.a_z1 = d.a_sz1; a.a_z2 = d.a_sz2; a.b_z1 = d.b_sz1; a.b_z2 = d.b_sz2;
  a.c_z1 = d.c_sz1; a.c_z2 = d.c_sz2;
  a.nz = d.nz1 * d.nz2; a.nz2 = d.nz2; a.causal = d.causal;
  a.k_splits = 1; a.partial = nullptr;
  a.epi = d.epi.kind;
  a.col0 = 0; a.row_len = d.N;
  if (d.epi.kind != kEpiNone) {
    a.aux = static_cast<const bf16_t*>(d.epi.aux); a.aux_ld = d.epi.aux_ld;
    a.vec = static_cast<const bf16_t*>(d.epi.vec);
    a.plain = static_cast<bf16_t*>(d.epi.plain);
    a.colsum_partial = d.epi.colsum_partial;
    if (d.epi.kind == kEpiBiasDropoutAdd) a.key = make_dropout_key(d.epi.dp, d.epi.site);
    if (d.epi.kind == kEpiSoftmaxBwd) {
      a.key = make_dropout_key(d.epi.dp, 0);
      a.rowdot = d.epi.rowdot; a.scale = d.epi.scale;
      a.global_heads = d.epi.global_heads; a.head0 = d.epi.head0;
    }
  }
  return a;
}

}  // namespace

bool gemm_mfma_supported(int dtype, const GemmDesc& d) {
  if (dtype != 1) return false;
  if (d.M % 128 || d.N % 128 || d.K % kBK || d.K < kBK) return false;
  if (d.causal == kCausalOutLower && d.M != d.N) return false;
  if ((d.causal == kCausalKLeM || d.causal == kCausalKGeM) && (d.M != d.K || d.bias != nullptr)) return false;
  const bool a_k = d.a_sk == 1, a_mn = d.a_sm == 1;
  const bool b_k = d.b_sk == 1, b_mn = d.b_sn == 1;
  if (!(a_k || a_mn) || !(b_k || b_mn)) return false;
  if ((a_k ? d.a_sm : d.a_sk) % 8 || (b_k ? d.b_sn : d.b_sk) % 8 || d.c_sm % 8) return false;
  if (d.a_sz1 % 8 || d.a_sz2 % 8 || d.b_sz1 % 8 || d.b_sz2 % 8 || d.c_sz1 % 8 || d.c_sz2 % 8) return false;
  if ((reinterpret_cast<uintptr_t>(d.A) | reinterpret_cast<uintptr_t>(d.B)) & 15) return false;
  if (reinterpret_cast<uintptr_t>(d.C) & 15) return false;
  if (d.bias != nullptr && (reinterpret_cast<uintptr_t>(d.bias) & 7)) return false;
  if (d.epi.kind != kEpiNone) {
    if (d.epi.kind == kEpiSoftmaxBwd) {
      // only the row-block kernel of the score-shaped products carries it (head dimension 128:
      // the staging area is the B buffer)
      if (d.causal != kCausalOutLower || d.bias != nullptr || d.K != 128) return false;
      if (!(d.a_sk == 1 && d.b_sk == 1)) return false;
      if (d.epi.aux == nullptr || (reinterpret_cast<uintptr_t>(d.epi.aux) & 15) || d.epi.rowdot == nullptr) return false;
      return true;
    }
    if (d.epi.kind != kEpiBiasDropoutAdd && d.epi.kind != kEpiGeluBwd) return false;
    if (d.causal != kCausalNone || d.nz1 * d.nz2 != 1 || d.bias != nullptr) return false;
    if (d.epi.aux == nullptr || (reinterpret_cast<uintptr_t>(d.epi.aux) & 15) || d.epi.aux_ld % 8) return false;
    if (d.epi.kind == kEpiBiasDropoutAdd) {
      if (d.epi.vec == nullptr || (reinterpret_cast<uintptr_t>(d.epi.vec) & 15)) return false;
      if (d.epi.plain != nullptr && (reinterpret_cast<uintptr_t>(d.epi.plain) & 15)) return false;
    } else {
      // column partials are laid out per 128 rows: 256-row tiles only, which the pair launch uses
      if (d.M % 256 || d.epi.colsum_partial == nullptr || d.epi.colsum_out == nullptr) return false;
      if (reinterpret_cast<uintptr_t>(d.epi.colsum_partial) & 15) return false;
    }
  }
  return true;
}

size_t gemm_colsum_partial_bytes(int M, int N) {
  return static_cast<size_t>((M + 127) / 128) * static_cast<size_t>(N) * sizeof(float);
}

hipError_t gemm_mfma(const GemmDesc& d, hipStream_t st) {
  if (d.epi.kind == kEpiGeluBwd) return hipErrorInvalidValue;  // needs the pair launch's 256-row tiles
  const MfmaGemmArgs a = make_args(d);
  const bool a_k = d.a_sk == 1, b_k = d.b_sk == 1;
  if (a_k && b_k) return launch_tiles<true, true>(a, st);
  if (a_k && !b_k) return launch_tiles<true, false>(a, st);
  if (!a_k && b_k) return launch_tiles<false, true>(a, st);
  return launch_tiles<false, false>(a, st);
}

bool gemm_mfma_pair_supported(int dtype, const GemmDesc& dgrad, const GemmDesc& wgrad) {
  if (!gemm_mfma_supported(dtype, dgrad) || !gemm_mfma_supported(dtype, wgrad)) return false;
  if (dgrad.nz1 * dgrad.nz2 != 1 || wgrad.nz1 * wgrad.nz2 != 1) return false;
  if (dgrad.causal != kCausalNone || wgrad.causal != kCausalNone) return false;
  if (!(dgrad.a_sk == 1 && dgrad.b_sn == 1 && dgrad.b_sk != 1)) return false;  // A K-major, B MN-major
  if (!(wgrad.a_sm == 1 && wgrad.a_sk != 1 && wgrad.b_sn == 1 && wgrad.b_sk != 1)) return false;
  if (wgrad.epi.kind != kEpiNone || (dgrad.epi.kind != kEpiNone && dgrad.epi.kind != kEpiGeluBwd)) return false;
  const PairPlan p = plan_pair(wgrad.M, wgrad.N, wgrad.K, dgrad.M, dgrad.N, dgrad.K);
  if (p.dbm != 256) return false;
  if (p.wbm == 128 && p.wbn == 128) return false;
  return true;
}

size_t gemm_pair_scratch_bytes(int dtype, const GemmDesc& dgrad, const GemmDesc& wgrad) {
  if (dtype != 1) return 0;
  const PairPlan p = plan_pair(wgrad.M, wgrad.N, wgrad.K, dgrad.M, dgrad.N, dgrad.K);
  return p.k_splits > 1 ? static_cast<size_t>(p.k_splits) * wgrad.M * wgrad.N * sizeof(float) : 0;
}

hipError_t gemm_mfma_pair(const GemmDesc& dgrad, const GemmDesc& wgrad, float* scratch, size_t scratch_bytes,
                          hipStream_t st) {
  const MfmaGemmArgs d = make_args(dgrad);
  MfmaGemmArgs w = make_args(wgrad);
  const PairPlan p = plan_pair(w.M, w.N, w.K, d.M, d.N, d.K);
  if (p.k_splits > 1) {
    // The cut is part of the shape's fixed summation order: a scratch block that cannot hold
    // the partial sums is an error, never a silent change of the gradient's bits.
    if (scratch == nullptr || (reinterpret_cast<uintptr_t>(scratch) & 15) != 0 ||
        scratch_bytes < static_cast<size_t>(p.k_splits) * w.M * w.N * sizeof(float))
      return hipErrorInvalidValue;
    w.k_splits = p.k_splits;
    w.partial = scratch;
  }
  auto run = [&]() -> hipError_t {
    if (p.dbn == 256) {
      if (p.edge == 1) return launch_pair<256, 256, 256, 256, 128, 256>(w, d, p, st);
      if (p.edge == 2) return launch_pair<256, 256, 256, 256, 256, 128>(w, d, p, st);
      if (p.wbm == 256 && p.wbn == 256) return launch_pair<256, 256, 256, 256, 0, 0>(w, d, p, st);
      if (p.wbm == 256) return launch_pair<256, 256, 256, 128, 0, 0>(w, d, p, st);
      return launch_pair<256, 256, 128, 256, 0, 0>(w, d, p, st);
    }
    if (p.edge == 1) return launch_pair<256, 128, 256, 256, 128, 256>(w, d, p, st);
    if (p.edge == 2) return launch_pair<256, 128, 256, 256, 256, 128>(w, d, p, st);
    if (p.wbm == 256 && p.wbn == 256) return launch_pair<256, 128, 256, 256, 0, 0>(w, d, p, st);
    if (p.wbm == 256) return launch_pair<256, 128, 256, 128, 0, 0>(w, d, p, st);
    return launch_pair<256, 128, 128, 256, 0, 0>(w, d, p, st);
  };
  const hipError_t e = run();
  if (e != hipSuccess) return e;
  if (dgrad.epi.kind == kEpiGeluBwd) {
    // second, fixed-order stage of the bias gradient: one partial row per 128 output rows
    launch_reduce_partials<bf16_t>(dgrad.epi.colsum_partial, static_cast<bf16_t*>(dgrad.epi.colsum_out), nullptr,
                                   nullptr, dgrad.M / 128, dgrad.N, st);
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace lynx
