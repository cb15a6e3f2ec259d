// Variant dispatch shared by the GEMM translation units.
#pragma once
#include "internal.hpp"

#define DION_DISPATCH_VARIANT(BF16, ASRC, BSRC, GBF16, EPI, DUAL)                                          \
  switch (variant) {                                                                                       \
    case VAR_BIG:                                                                                          \
      return launch_gemm<CfgBig, BF16, ASRC, BSRC, GBF16, EPI, DUAL, false>(g, batch, s);                  \
    case VAR_SMALL:                                                                                        \
      return launch_gemm<CfgSmall, BF16, ASRC, BSRC, GBF16, EPI, DUAL, false>(g, batch, s);                \
    default:                                                                                               \
      return launch_gemm<CfgSmall, BF16, ASRC, BSRC, GBF16, EPI, DUAL, true>(g, batch, s);                 \
  }

#define DION_DISPATCH_TYPES(ASRC, BSRC, EPI, DUAL)                                                         \
  if (bf16) {                                                                                              \
    if (gbf16) { DION_DISPATCH_VARIANT(true, ASRC, BSRC, true, EPI, DUAL) }                                \
    else { DION_DISPATCH_VARIANT(true, ASRC, BSRC, false, EPI, DUAL) }                                     \
  } else {                                                                                                 \
    if (gbf16) { DION_DISPATCH_VARIANT(false, ASRC, BSRC, true, EPI, DUAL) }                               \
    else { DION_DISPATCH_VARIANT(false, ASRC, BSRC, false, EPI, DUAL) }                                    \
  }
