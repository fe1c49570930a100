// Chooses the kernel for a matrix product.
#include "kernels.h"

namespace lynx {

hipError_t gemm(int dtype, const GemmDesc& d, hipStream_t st) {
  if (gemm_mfma_supported(dtype, d)) return gemm_mfma(d, st);
  if (d.epi.kind != kEpiNone) return hipErrorInvalidValue;  // only the matrix-core kernels carry epilogues
  return gemm_generic(dtype, d, st);
}

hipError_t gemm_pair(int dtype, const GemmDesc& dgrad, const GemmDesc& wgrad, float* scratch,
                     size_t scratch_bytes, hipStream_t st) {
  if (gemm_mfma_pair_supported(dtype, dgrad, wgrad))
    return gemm_mfma_pair(dgrad, wgrad, scratch, scratch_bytes, st);
  if (dgrad.epi.kind != kEpiNone || wgrad.epi.kind != kEpiNone) return hipErrorInvalidValue;
  const hipError_t e = gemm(dtype, dgrad, st);
  if (e != hipSuccess) return e;
  return gemm(dtype, wgrad, st);
}

}  // namespace lynx
