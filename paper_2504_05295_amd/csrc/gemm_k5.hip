// Fused rank-r updates of the unsharded update rule: one pass over M, G, X computing both
// P R^T (error feedback) and P Q_new^T (weight update) with the P tile shared.
#include "gemm_dispatch.hpp"
namespace dion {
hipError_t gemm_k5(int variant, bool bf16, bool gbf16, GemmArgs g, int batch, hipStream_t s) {
  DION_DISPATCH_TYPES(SRC_F32_KC, SRC_F32_KC, EPI_UPDATE, true)
}
}  // namespace dion
