// R = (M + G)^T P   (PowerIter1, second product): A = fused sum read across k = m (transposed on the
// way into LDS, so the big matrix is still read along its rows), B = P read across k.
#include "gemm_dispatch.hpp"
namespace dion {
hipError_t gemm_k2(int variant, bool bf16, bool gbf16, GemmArgs g, int batch, hipStream_t s) {
  DION_DISPATCH_TYPES(SRC_SUM_KS, SRC_F32_KS, EPI_STORE, false)
}
}  // namespace dion
