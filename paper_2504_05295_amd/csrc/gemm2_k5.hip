// Fused rank-r updates on large tiles: A = P, B = R, B2 = Q_new (all bf16 copies), epilogue updates M and X.
#include "gemm_core2.hpp"
#include "gemm_core3.hpp"
#include "internal.hpp"
namespace dion {
hipError_t gemm2_k5(int cfg, bool gbf16, GemmArgs g, int batch, hipStream_t s) {
  using Big = TileCfg2<256, 128, 64, 2, 4, 1, 2>;
  using Mid = TileCfg2<128, 128, 64, 2, 2, 1, 2>;
  using Direct = TileCfg3<256, 128, 2, 4>;   // same tile, operands loaded straight into LDS
  if (cfg == G2_256x256 && gemm3_fits<Direct>(g) && g.B2.ld == g.B.ld) {
    if (g.E.stream_hint)
      return gbf16 ? launch_gemm3<Direct, true, EPI_UPDATE_STREAM, true>(g, batch, s)
                   : launch_gemm3<Direct, false, EPI_UPDATE_STREAM, true>(g, batch, s);
    return gbf16 ? launch_gemm3<Direct, true, EPI_UPDATE, true>(g, batch, s)
                 : launch_gemm3<Direct, false, EPI_UPDATE, true>(g, batch, s);
  }
  if (cfg == G2_256x256)
    return gbf16 ? launch_gemm2<Big, SRC2_BF16_KC, true, EPI_UPDATE, true>(g, batch, s)
                 : launch_gemm2<Big, SRC2_BF16_KC, false, EPI_UPDATE, true>(g, batch, s);
  return gbf16 ? launch_gemm2<Mid, SRC2_BF16_KC, true, EPI_UPDATE, true>(g, batch, s)
               : launch_gemm2<Mid, SRC2_BF16_KC, false, EPI_UPDATE, true>(g, batch, s);
}
hipError_t gemm2_k5_prepare() {
  using Direct = TileCfg3<256, 128, 2, 4>;
  hipError_t e = gemm3_prepare<Direct, true, EPI_UPDATE, true>();
  if (e == hipSuccess) e = gemm3_prepare<Direct, false, EPI_UPDATE, true>();
  if (e == hipSuccess) e = gemm3_prepare<Direct, true, EPI_UPDATE_STREAM, true>();
  if (e == hipSuccess) e = gemm3_prepare<Direct, false, EPI_UPDATE_STREAM, true>();
  return e;
}
}  // namespace dion
