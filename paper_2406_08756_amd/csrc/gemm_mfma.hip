// bf16 matrix products on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16).
//
//   C[M, N] = sum_k A(m, k) * B(k, n) (+ bias[n]),   fp32 accumulation
//
// Either operand may be stored "K-major" (the contraction index is the
// contiguous one: activations and weights in a forward linear layer) or
// "MN-major" (the contraction index is the row index: the weight in an input
// gradient, both operands in a weight gradient).  One workgroup of 8
// wavefronts owns a BM x BN output tile and walks K in slabs of 64:
//   global -> registers (16-byte loads) -> LDS, double buffered;
//   K-major slabs sit in LDS as [mn][64] with the 16-byte chunk index XORed
//   with (row & 7), so the 32 rows a fragment read touches spread over all
//   banks; MN-major slabs sit as [64][mn + 16] and are read with the
//   transposing LDS read (ds_read_b64_tr_b16), which hands each lane four
//   consecutive k for its own mn - no shuffles and no transposed copies.
// The product is formed transposed (B fragment as the first MFMA operand) so
// that every lane ends up with four consecutive n of one row m and can store
// 8 bytes at a time.
#include "device_common.h"
#include "kernels.h"

namespace lynx {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;          // K slab
constexpr int kThreads = 512;    // 8 wavefronts
constexpr int kPadMN = 16;       // row padding (elements) of MN-major slabs

struct MfmaGemmArgs {
  const bf16_t* A; long long lda;
  const bf16_t* B; long long ldb;
  bf16_t* C; long long ldc;
  const bf16_t* bias;
  int M, N, K;
  int tiles_m, tiles_n;
};

template <int ROWS, bool KMAJOR>
struct Slab {  // LDS footprint of one operand slab, in bf16 elements
  static constexpr int kElems = KMAJOR ? ROWS * kBK : kBK * (ROWS + kPadMN);
  static constexpr int kChunks = ROWS * kBK / 8;            // 16-byte chunks
  static constexpr int kPerThread = kChunks / kThreads;
  static_assert(kChunks % kThreads == 0, "slab must divide over the workgroup");
};

// Global address (in elements) of 16-byte chunk c of the slab starting at
// (row0, k0), and the LDS element offset it is staged to.
template <int ROWS, bool KMAJOR>
__device__ __forceinline__ void chunk_coords(int c, long long ld, int row0, int k0, long long* goff,
                                             int* loff) {
  if (KMAJOR) {
    const int r = c >> 3, kc = c & 7;                      // 8 chunks per row of 64 k
    *goff = static_cast<long long>(row0 + r) * ld + k0 + kc * 8;
    *loff = r * kBK + ((kc ^ (r & 7)) << 3);
  } else {
    constexpr int kRowChunks = ROWS / 8;
    const int kr = c / kRowChunks, mc = c - kr * kRowChunks;
    *goff = static_cast<long long>(k0 + kr) * ld + row0 + mc * 8;
    *loff = kr * (ROWS + kPadMN) + mc * 8;
  }
}

// One MFMA operand fragment: 8 consecutive k (at 16*ks + 8*(lane/32)) of row
// `r` (= tile base + lane%32) of the slab.
template <int ROWS, bool KMAJOR>
__device__ __forceinline__ bf16x8_t read_fragment(const bf16_t* slab, int tile_row0, int ks, int lane) {
  if (KMAJOR) {
    const int r = tile_row0 + (lane & 31);
    const int chunk = (ks * 2 + (lane >> 5)) ^ (r & 7);
    return *reinterpret_cast<const bf16x8_t*>(slab + r * kBK + (chunk << 3));
  } else {
    // lanes form four blocks of 16: block b covers rows (b&1)*16.. and k-group b>>1;
    // inside a block lane i points at k-row i/4, columns 4*(i%4)..+3, and receives
    // the four k of column i.
    const int b = lane >> 4, i = lane & 15;
    const int k = ks * 16 + (b >> 1) * 8 + (i >> 2);
    const int col = tile_row0 + (b & 1) * 16 + ((i & 3) << 2);
    const bf16_t* p = slab + k * (ROWS + kPadMN) + col;
    typedef __attribute__((address_space(3))) short4_t* lds_ptr_t;
    const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * (ROWS + kPadMN)));
    typedef short short8_t __attribute__((ext_vector_type(8)));
    const short8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8_t, v);
  }
}

template <bool A_KMAJOR, bool B_KMAJOR, int BM, int BN, int WAVES_M, int WAVES_N>
__global__ void __launch_bounds__(kThreads) gemm_mfma_kernel(MfmaGemmArgs g) {
  static_assert(WAVES_M * WAVES_N == kThreads / kWave, "8 wavefronts");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  using SlabA = Slab<BM, A_KMAJOR>;
  using SlabB = Slab<BN, B_KMAJOR>;
  constexpr int kStage = SlabA::kElems + SlabB::kElems;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

  // workgroup -> output tile.  Consecutive workgroup ids land on different
  // XCDs (round robin over 8), so give each XCD a contiguous run of tiles,
  // and order tiles in bands of 8 tile-rows so a band's A and B panels stay
  // in that XCD's L2.
  const int ntiles = g.tiles_m * g.tiles_n;
  int tile = blockIdx.x;
  {
    const int per_xcd = ntiles / 8;
    if (tile < per_xcd * 8) tile = (tile & 7) * per_xcd + (tile >> 3);
  }
  constexpr int kBand = 8;
  const int band = tile / (kBand * g.tiles_n);
  const int band_rows = min(kBand, g.tiles_m - band * kBand);
  const int in_band = tile - band * kBand * g.tiles_n;
  const int tm = band * kBand + in_band % band_rows;
  const int tn = in_band / band_rows;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

  floatx16_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 stage_a[SlabA::kPerThread], stage_b[SlabB::kPerThread];
  auto load_slabs = [&](int k0) {
#pragma unroll
    for (int i = 0; i < SlabA::kPerThread; ++i) {
      long long go; int lo;
      chunk_coords<BM, A_KMAJOR>(tid + i * kThreads, g.lda, m0, k0, &go, &lo);
      stage_a[i] = *reinterpret_cast<const uint4*>(g.A + go);
    }
#pragma unroll
    for (int i = 0; i < SlabB::kPerThread; ++i) {
      long long go; int lo;
      chunk_coords<BN, B_KMAJOR>(tid + i * kThreads, g.ldb, n0, k0, &go, &lo);
      stage_b[i] = *reinterpret_cast<const uint4*>(g.B + go);
    }
  };
  auto store_slabs = [&](int buf) {
    bf16_t* sa = smem + buf * kStage;
    bf16_t* sb = sa + SlabA::kElems;
#pragma unroll
    for (int i = 0; i < SlabA::kPerThread; ++i) {
      long long go; int lo;
      chunk_coords<BM, A_KMAJOR>(tid + i * kThreads, g.lda, m0, 0, &go, &lo);
      *reinterpret_cast<uint4*>(sa + lo) = stage_a[i];
    }
#pragma unroll
    for (int i = 0; i < SlabB::kPerThread; ++i) {
      long long go; int lo;
      chunk_coords<BN, B_KMAJOR>(tid + i * kThreads, g.ldb, n0, 0, &go, &lo);
      *reinterpret_cast<uint4*>(sb + lo) = stage_b[i];
    }
  };

  const int nk = g.K / kBK;
  load_slabs(0);
  store_slabs(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_slabs((kt + 1) * kBK);
    const bf16_t* sa = smem + buf * kStage;
    const bf16_t* sb = sa + SlabA::kElems;
#pragma unroll
    for (int ks = 0; ks < kBK / 16; ++ks) {
      bf16x8_t fa[TM], fb[TN];
#pragma unroll
      for (int j = 0; j < TM; ++j) fa[j] = read_fragment<BM, A_KMAJOR>(sa, wm0 + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < TN; ++i) fb[i] = read_fragment<BN, B_KMAJOR>(sb, wn0 + i * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i], fa[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_slabs(buf ^ 1);
    __syncthreads();
  }

  // acc[i][j][r]: n = wn0 + 32 i + 8 (r/4) + 4 (lane/32) + r%4,  m = wm0 + 32 j + lane%32
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int n = n0 + wn0 + 32 * i + 8 * q + 4 * (lane >> 5);
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (g.bias != nullptr) {
        const uint2 braw = *reinterpret_cast<const uint2*>(g.bias + n);
        bv[0] = bf16_lo(braw.x); bv[1] = bf16_hi(braw.x); bv[2] = bf16_lo(braw.y); bv[3] = bf16_hi(braw.y);
      }
#pragma unroll
      for (int j = 0; j < TM; ++j) {
        const int m = m0 + wm0 + 32 * j + (lane & 31);
        uint2 o;
        o.x = pack_bf16(acc[i][j][4 * q + 0] + bv[0], acc[i][j][4 * q + 1] + bv[1]);
        o.y = pack_bf16(acc[i][j][4 * q + 2] + bv[2], acc[i][j][4 * q + 3] + bv[3]);
        *reinterpret_cast<uint2*>(g.C + static_cast<long long>(m) * g.ldc + n) = o;
      }
    }
}

template <bool AK, bool BK_, int BM, int BN, int WM_, int WN_>
hipError_t launch(const MfmaGemmArgs& a, hipStream_t st) {
  using SA = Slab<BM, AK>;
  using SB = Slab<BN, BK_>;
  constexpr size_t smem = 2 * (SA::kElems + SB::kElems) * sizeof(bf16_t);
  auto kern = gemm_mfma_kernel<AK, BK_, BM, BN, WM_, WN_>;
  static bool configured = false;  // raise the dynamic LDS limit once per instantiation
  if (!configured) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                             static_cast<int>(smem));
    if (e != hipSuccess) return e;
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3(a.tiles_m * a.tiles_n), dim3(kThreads), smem, st, a);
  return hipGetLastError();
}

// Tile shape: the largest tile that divides the output, unless a smaller one
// fills the 256 compute units markedly better (fewer idle units in the last
// round of workgroups).
template <bool AK, bool BK_>
hipError_t launch_tiles(MfmaGemmArgs a, hipStream_t st) {
  struct Cand { int bm, bn; float weight; };
  static const Cand cands[4] = {{256, 256, 1.0f}, {256, 128, 0.88f}, {128, 256, 0.88f}, {128, 128, 0.72f}};
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
    case 0: return launch<AK, BK_, 256, 256, 2, 4>(a, st);
    case 1: return launch<AK, BK_, 256, 128, 4, 2>(a, st);
    case 2: return launch<AK, BK_, 128, 256, 2, 4>(a, st);
    default: return launch<AK, BK_, 128, 128, 2, 4>(a, st);
  }
}

}  // namespace

bool gemm_mfma_supported(int dtype, const GemmDesc& d) {
  if (dtype != 1 || d.nz1 * d.nz2 != 1 || d.causal != kCausalNone) return false;
  if (d.M % 128 || d.N % 128 || d.K % kBK || d.K < kBK) return false;
  const bool a_k = d.a_sk == 1, a_mn = d.a_sm == 1;
  const bool b_k = d.b_sk == 1, b_mn = d.b_sn == 1;
  if (!(a_k || a_mn) || !(b_k || b_mn)) return false;
  if ((a_k ? d.a_sm : d.a_sk) % 8 || (b_k ? d.b_sn : d.b_sk) % 8 || d.c_sm % 4) return false;
  return true;
}

hipError_t gemm_mfma(const GemmDesc& d, hipStream_t st) {
  MfmaGemmArgs a{};
  const bool a_k = d.a_sk == 1, b_k = d.b_sk == 1;
  a.A = static_cast<const bf16_t*>(d.A); a.lda = a_k ? d.a_sm : d.a_sk;
  a.B = static_cast<const bf16_t*>(d.B); a.ldb = b_k ? d.b_sn : d.b_sk;
  a.C = static_cast<bf16_t*>(d.C); a.ldc = d.c_sm;
  a.bias = static_cast<const bf16_t*>(d.bias);
  a.M = d.M; a.N = d.N; a.K = d.K;
  if (a_k && b_k) return launch_tiles<true, true>(a, st);
  if (a_k && !b_k) return launch_tiles<true, false>(a, st);
  if (!a_k && b_k) return launch_tiles<false, true>(a, st);
  return launch_tiles<false, false>(a, st);
}

}  // namespace lynx
