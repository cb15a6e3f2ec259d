// Plain bf16 x bf16 products C = sum over operand pairs of A_s B_s^T on large tiles.  With the pairs
// (hi,hi), (hi,lo), (lo,hi) of split-bf16 operands this evaluates an fp32-grade product on the bf16
// matrix pipe; used for the Gram matrix and the triangular multiply of Cholesky-QR (Appendix A).  With one
// pair it is also K1 and K2 of the step on the direct-load path (A = bf16(M+G) or its transpose).
#include "gemm_core2.hpp"
#include "gemm_core3.hpp"
#include "internal.hpp"
namespace dion {
using NtBig = TileCfg2<256, 256, 64, 2, 4, 2, 1>;
using NtMid = TileCfg2<128, 128, 64, 2, 2, 1, 2>;
hipError_t gemm2_nt(int cfg, GemmArgs g, int batch, hipStream_t s, int ks) {
  if (ks != 0) {
    // operands stored with k as the slow index (direct-load core, 256 x 256 tiles only)
    using Direct = TileCfg3<256, 256, 2, 4>;
    if (cfg != G2_256x256) return hipErrorInvalidValue;
    if (ks == (KS_A | KS_B)) return launch_gemm3<Direct, false, EPI_STORE, false, true, true>(g, batch, s);
    if (ks == KS_B) return launch_gemm3<Direct, false, EPI_STORE, false, false, true>(g, batch, s);
    return hipErrorInvalidValue;
  }
  if (cfg == G2_256x128) {
    // narrower column tiles for the triangular multiply of a single matrix: twice as many workgroups as compute
    // units, costliest first (GemmArgs::heavy_first), instead of one round in which the last column tile sets the time
    using Narrow = TileCfg3<256, 128, 4, 2>;   // wave tiles of 64 x 64
    if (gemm3_fits<Narrow>(g)) return launch_gemm3<Narrow, false, EPI_STORE, false>(g, batch, s);
    cfg = G2_256x256;
  }
  if (cfg == G2_256x256) {
    using Direct = TileCfg3<256, 256, 2, 4>;   // same tile, operands loaded straight into LDS
    if (gemm3_fits<Direct>(g)) return launch_gemm3<Direct, false, EPI_STORE, false>(g, batch, s);
    return launch_gemm2<NtBig, SRC2_BF16_KC, false, EPI_STORE, false>(g, batch, s);
  }
  return launch_gemm2<NtMid, SRC2_BF16_KC, false, EPI_STORE, false>(g, batch, s);
}
hipError_t gemm2_nt_prepare() {
  hipError_t e = gemm3_prepare<TileCfg3<256, 256, 2, 4>, false, EPI_STORE, false>();
  if (e == hipSuccess) e = gemm3_prepare<TileCfg3<256, 128, 4, 2>, false, EPI_STORE, false>();
  if (e == hipSuccess) e = gemm3_prepare<TileCfg3<256, 256, 2, 4>, false, EPI_STORE, false, true, true>();
  if (e == hipSuccess) e = gemm3_prepare<TileCfg3<256, 256, 2, 4>, false, EPI_STORE, false, false, true>();
  return e;
}
bool gemm2_nt_is_direct(int cfg, const GemmArgs& g) {
  if (cfg == G2_256x128 && gemm3_fits<TileCfg3<256, 128, 4, 2>>(g)) return true;
  return (cfg == G2_256x128 || cfg == G2_256x256) && gemm3_fits<TileCfg3<256, 256, 2, 4>>(g);
}
int gemm2_nt_colsq_chunks(int cfg, const GemmArgs& g, int ks) {
  using Direct = TileCfg3<256, 256, 2, 4>;
  if (cfg != G2_256x256 || g.splitk > 1) return 0;
  const bool fits = ks == (KS_A | KS_B) ? gemm3_fits<Direct, true, true>(g) : ks == KS_B ? gemm3_fits<Direct, false, true>(g)
                    : ks == 0 ? gemm3_fits<Direct>(g) : false;
  return fits ? g.M / Direct::WTM : 0;
}
int gemm2_nt_splitk(int cfg, const GemmArgs& g) {
  return cfg == G2_256x256 ? gemm2_effective_splitk<NtBig>(g) : gemm2_effective_splitk<NtMid>(g);
}
}  // namespace dion
