// Host-callable launchers of the HIP kernels.  Every launcher enqueues on the
// given stream, never synchronises, and returns the launch status.  `dtype`
// is 0 for fp32 storage and 1 for bf16 storage; arithmetic is fp32 throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lynx {

struct DropoutParams {
  uint64_t seed;
  uint64_t step;
  uint32_t layer_id;
  float p;
};

// Index map of the attention-dropout site: element (bi, hd, i, j) of a shard
// has flat index ((bi * global_heads + head0 + hd) * s + i) * s + j.
struct AttnShape {
  int b, a, s;
  int global_heads, head0;
};

// ---- LayerNorm ------------------------------------------------------------
hipError_t layernorm_fwd(int dtype, const void* x, const void* gamma, const void* beta, void* y,
                         float* mean, float* rstd, int rows, int cols, float eps, hipStream_t st);
// dx_out = dres + dLN/dx (dres may alias nothing; dx_out may alias dres);
// dgamma/dbeta are reduced over rows in two fixed-order stages through scratch.
size_t layernorm_bwd_scratch_bytes(int rows, int cols);
hipError_t layernorm_bwd(int dtype, const void* dy, const void* x, const float* mean,
                         const float* rstd, const void* gamma, const void* dres, void* dx_out,
                         void* dgamma, void* dbeta, float* scratch, int rows, int cols,
                         hipStream_t st);
// The same, and in the same pass the backward of the bias + dropout + residual operator
// whose output the LayerNorm read: dropped = keep c round(dx_out), dbias = its column sums.
hipError_t layernorm_bwd_dropout_bwd(int dtype, const void* dy, const void* x, const float* mean,
                                     const float* rstd, const void* gamma, const void* dres, void* dx_out,
                                     void* dgamma, void* dbeta, void* dropped, void* dbias, float* scratch,
                                     int rows, int cols, int site, DropoutParams dp, hipStream_t st);

// ---- attention softmax / dropout -----------------------------------------
// P = softmax_{j<=i}(S * scale) (written if P != null), Pd = keep * P * c
// (written if Pd != null; computed from the storage-rounded P).  Columns
// (i, round_up(i+1, 128)) of every written row are zero-filled.
hipError_t softmax_dropout_fwd(int dtype, const void* S, void* P, void* Pd, AttnShape sh,
                               float scale, DropoutParams dp, hipStream_t st);
// Pd = keep * P * c from a resident P.
hipError_t attn_dropout_fwd(int dtype, const void* P, void* Pd, AttnShape sh, DropoutParams dp,
                            hipStream_t st);
// dS = scale * P * (dP - sum_j dP * P), dP = keep * dPd * c; dS may alias dPd.
hipError_t softmax_dropout_bwd(int dtype, const void* dPd, const void* P, void* dS, AttnShape sh,
                               float scale, DropoutParams dp, hipStream_t st);

// ---- elementwise over [rows, cols] -----------------------------------------
hipError_t gelu_fwd(int dtype, const void* u, void* g, size_t n, hipStream_t st);
size_t colsum_scratch_bytes(int rows, int cols);
// du = dg * gelu'(u); dbias[c] = sum_r du[r, c]
hipError_t gelu_bwd(int dtype, const void* dg, const void* u, void* du, void* dbias,
                    float* scratch, int rows, int cols, hipStream_t st);
// out = res + keep * (in + bias) * c, dropout site `site`, element index r*cols + c
hipError_t bias_dropout_add_fwd(int dtype, const void* in, const void* bias, const void* res,
                                void* out, int rows, int cols, int site, DropoutParams dp,
                                hipStream_t st);
// din = keep * dout * c; dbias[c] = sum_r din[r, c]
hipError_t dropout_bwd(int dtype, const void* dout, void* din, void* dbias, float* scratch,
                       int rows, int cols, int site, DropoutParams dp, hipStream_t st);
// dbias[c] = sum_r x[r, c]
hipError_t column_sum(int dtype, const void* x, void* dbias, float* scratch, int rows, int cols,
                      hipStream_t st);
// out[(bi * a + hd) * s + i] = sum_dd x[t, hd * d + dd] * y[t, hd * d + dd], t = bi * s + i (fp32);
// x and y are [T, a * d] with row stride ld.  With x = dC and y = C this is the row dot
// product sum_j dP_ij P_ij of the softmax backward.
hipError_t attn_rowdot(int dtype, const void* x, const void* y, float* out, int b, int a, int s, int d,
                       long long ld, hipStream_t st);
// ---- attention without the seq x seq tensors (attn_fused.hip) ----------------------------
// bf16 storage, head dimension 128, sequence a multiple of 128.
bool attn_fused_supported(int dtype, int s, int d);
size_t attn_fused_stats_bytes(int b, int a, int s);
// Operators 3-6 in one launch: C [T, a * d] (row stride ldc) from QKV [T, 3 a d] (row stride
// ld), bit-identical to S -> softmax -> dropout -> Pd V run one after the other; also leaves
// per row (b, head, i) the maximum of the logits and the reciprocal of the row sum in
// stats [b * a * s][2], from which the backward kernels rebuild P.
hipError_t attn_fused_fwd(const void* qkv, long long ld, void* c, long long ldc, float* stats, AttnShape sh, int d,
                          float scale, DropoutParams dp, hipStream_t st);

// Backward of operators 6-4 without P and Pd.  First kernel: dS [b, a, s, s] (dense layout,
// j <= i defined) = scale P (keep c round(dC V^T) - rowdot), P rebuilt from QKV and stats.
// Second kernel: the v block of dqkv [T, 3 a d] = Pd^T dC, Pd rebuilt likewise.  Both
// bit-identical to the unfused kernels run on stored P and Pd.
hipError_t attn_fused_bwd_ds(const void* qkv, long long ld, const void* dc, long long lddc, const float* stats,
                             const float* rowdot, void* ds, AttnShape sh, int d, float scale, DropoutParams dp,
                             hipStream_t st);
hipError_t attn_fused_bwd_dv(const void* qkv, long long ld, const void* dc, long long lddc, const float* stats,
                             void* dqkv, long long lddq, AttnShape sh, int d, float scale, DropoutParams dp,
                             hipStream_t st);

// keep-mask bytes for parity checks: n elements starting at flat index 0 of
// site 1/2, or the [b, a, s, s] tensor of site 0.
hipError_t dropout_mask_hidden(uint8_t* out, size_t n, int site, DropoutParams dp, hipStream_t st);
hipError_t dropout_mask_attn(uint8_t* out, AttnShape sh, DropoutParams dp, hipStream_t st);

// ---- matrix products ------------------------------------------------------
enum CausalMode : int {
  kCausalNone = 0,
  kCausalOutLower = 1,  // only outputs with n <= m are needed (others may be skipped)
  kCausalKLeM = 2,      // contraction restricted to k <= m
  kCausalKGeM = 3       // contraction restricted to k >= m
};

// Elementwise work a matrix-core product can absorb into the pass that stores its output
// tile, so the operator that would read the product back never runs as a kernel of its
// own.  P = the product rounded to storage, exactly what an unfused launch would store.
enum GemmEpilogueKind : int {
  kEpiNone = 0,
  // bias + dropout + residual (operators 8, 13): C = aux + keep (P + vec) c at dropout site
  // `site`, element index m * N + n; if `plain` is not null P is stored there as well (row
  // stride = c_sm).  Bit-identical to bias_dropout_add_fwd run on a stored P.
  kEpiBiasDropoutAdd = 1,
  // GeLU backward (input gradient of FC2 only, inside gemm_pair): C = P gelu'(aux) and
  // colsum_out[n] = sum_m C[m, n] (the FC1 bias gradient), reduced in two fixed-order stages
  // through `colsum_partial` (gemm_colsum_partial_bytes).
  kEpiGeluBwd = 2,
  // dropout + softmax backward (B5 + B4) on the score-shaped product dPd = dC V^T (causal,
  // batched): C = dS = scale aux (keep c P - rowdot), aux = the softmax output P in the layout
  // of C, rowdot[z * M + i] the row's sum_j dP_ij P_ij (attn_rowdot), dropout site 0 with the
  // attention index map (global_heads, head0).  dPd itself is never stored.
  kEpiSoftmaxBwd = 4
};
struct GemmEpilogue {
  int kind;
  const void* aux;        // [M, N], row stride aux_ld: the residual (1) or U (2)
  long long aux_ld;
  const void* vec;        // (1) bias[N]
  void* plain;            // (1) nullable
  int site;               // (1)
  DropoutParams dp;       // (1)
  float* colsum_partial;  // (2)
  void* colsum_out;       // (2) [N], storage dtype
  const float* rowdot;    // (4)
  float scale;            // (4)
  int global_heads, head0;  // (4)
};

// C[z][m, n] = sum_k A[z][m, k] * B[z][k, n] (+ bias[n]), z = (z1, z2) a
// two-level batch.  Element strides are explicit, so any operand may be a
// transposed or column-sliced view.  Accumulation is fp32 in a fixed order.
struct GemmDesc {
  int M, N, K;
  const void* A; long long a_sm, a_sk, a_sz1, a_sz2;
  const void* B; long long b_sk, b_sn, b_sz1, b_sz2;
  void* C; long long c_sm, c_sz1, c_sz2;  // C is row-major within a matrix (n stride 1)
  const void* bias;                        // nullable, length N, same dtype
  int nz1, nz2;
  int causal;                              // CausalMode
  GemmEpilogue epi;                        // kind 0 (none) unless the matrix-core path is used
};
hipError_t gemm(int dtype, const GemmDesc& d, hipStream_t st);          // picks a kernel
hipError_t gemm_generic(int dtype, const GemmDesc& d, hipStream_t st);  // any shape, vector ALUs
bool gemm_mfma_supported(int dtype, const GemmDesc& d);                  // bf16, tile-aligned, unbatched
hipError_t gemm_mfma(const GemmDesc& d, hipStream_t st);                // matrix cores
// Input gradient and weight gradient of one linear layer, in one launch when the
// matrix-core kernel can pair them, else one after the other.
// `scratch` (fp32, 16-byte aligned, gemm_pair_scratch_bytes or more; may be null) lets the
// weight gradient be cut into K ranges whose partial sums are added in a fixed order.
hipError_t gemm_pair(int dtype, const GemmDesc& dgrad, const GemmDesc& wgrad, float* scratch,
                     size_t scratch_bytes, hipStream_t st);
size_t gemm_pair_scratch_bytes(int dtype, const GemmDesc& dgrad, const GemmDesc& wgrad);  // shapes only
bool gemm_mfma_pair_supported(int dtype, const GemmDesc& dgrad, const GemmDesc& wgrad);
size_t gemm_colsum_partial_bytes(int M, int N);  // kEpiGeluBwd
hipError_t gemm_mfma_pair(const GemmDesc& dgrad, const GemmDesc& wgrad, float* scratch, size_t scratch_bytes,
                          hipStream_t st);

}  // namespace lynx
