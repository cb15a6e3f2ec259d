// R = (M + G)^T P with bf16 operands on large tiles: A = the fused sum, or the bf16 copy of it that K1 left in
// memory, transposed on its way into LDS (the big matrices are still read along their rows), B = P^T (bf16).
#include "gemm_core2.hpp"
#include "internal.hpp"
namespace dion {
hipError_t gemm2_k2(int cfg, bool gbf16, GemmArgs g, int batch, hipStream_t s, bool from_bf16) {
  using Big = TileCfg2<256, 256, 64, 2, 4, 2, 1>;
  using Mid = TileCfg2<128, 128, 64, 2, 2, 1, 2>;
  if (from_bf16)   // A = the bf16 copy of M + G that K1 left behind, read across k
    return cfg == G2_256x256 ? launch_gemm2<Big, SRC2_BF16_KS, false, EPI_STORE, false>(g, batch, s)
                             : launch_gemm2<Mid, SRC2_BF16_KS, false, EPI_STORE, false>(g, batch, s);
  if (cfg == G2_256x256)
    return gbf16 ? launch_gemm2<Big, SRC2_SUM_KS, true, EPI_STORE, false>(g, batch, s)
                 : launch_gemm2<Big, SRC2_SUM_KS, false, EPI_STORE, false>(g, batch, s);
  return gbf16 ? launch_gemm2<Mid, SRC2_SUM_KS, true, EPI_STORE, false>(g, batch, s)
               : launch_gemm2<Mid, SRC2_SUM_KS, false, EPI_STORE, false>(g, batch, s);
}
int gemm2_k2_splitk(int cfg, const GemmArgs& g) {
  return cfg == G2_256x256 ? gemm2_effective_splitk<TileCfg2<256, 256, 64, 2, 4, 2, 1>>(g)
                           : gemm2_effective_splitk<TileCfg2<128, 128, 64, 2, 2, 1, 2>>(g);
}
}  // namespace dion
