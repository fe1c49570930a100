// Chooses the kernel for a matrix product.
#include "kernels.h"

namespace lynx {

hipError_t gemm(int dtype, const GemmDesc& d, hipStream_t st) {
  if (gemm_mfma_supported(dtype, d)) return gemm_mfma(d, st);
  return gemm_generic(dtype, d, st);
}

}  // namespace lynx
