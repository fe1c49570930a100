// Chooses the kernel for a matrix product.
#include "kernels.h"

namespace lynx {

hipError_t gemm(int dtype, const GemmDesc& d, hipStream_t st) {
  return gemm_generic(dtype, d, st);
}

}  // namespace lynx
