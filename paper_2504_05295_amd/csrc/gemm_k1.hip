// Z = (M + G) Q   (PowerIter1, first product): A = fused sum read along k = n, B = Q read across k.
#include "gemm_dispatch.hpp"
namespace dion {
hipError_t gemm_k1(int variant, bool bf16, bool gbf16, GemmArgs g, int batch, hipStream_t s) {
  DION_DISPATCH_TYPES(SRC_SUM_KC, SRC_F32_KS, EPI_STORE, false)
}
}  // namespace dion
