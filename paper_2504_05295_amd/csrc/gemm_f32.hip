// fp32 products of the orthonormalisation (Gram matrix, panel solves, trailing updates, inverse merges).
#include "gemm_dispatch.hpp"
namespace dion {
hipError_t gemm_f32_nt(int variant, GemmArgs g, int batch, hipStream_t s) {
  DION_DISPATCH_VARIANT(false, SRC_F32_KC, SRC_F32_KC, false, EPI_STORE, false)
}
hipError_t gemm_f32_nn(int variant, GemmArgs g, int batch, hipStream_t s) {
  DION_DISPATCH_VARIANT(false, SRC_F32_KC, SRC_F32_KS, false, EPI_STORE, false)
}
hipError_t gemm_f32_tn(int variant, GemmArgs g, int batch, hipStream_t s) {
  DION_DISPATCH_VARIANT(false, SRC_F32_KS, SRC_F32_KS, false, EPI_STORE, false)
}
}  // namespace dion
