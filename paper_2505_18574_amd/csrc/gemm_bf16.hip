// bf16 GEMM, fp32 accumulate and output: tile selection and launch.
#include "gemm_dtl.hpp"

#include <stdlib.h>

namespace ac {

hipError_t launch_gemm_bf16(const GemmParams& p, hipStream_t stream) {
  const bool aligned = (((uintptr_t)p.A & 15) == 0) && (((uintptr_t)p.B & 15) == 0) && (p.lda % 8 == 0) && (p.ldb % 8 == 0) &&
                       (((uintptr_t)p.C & 15) == 0) && (p.ldc % 4 == 0);
  // direct-to-LDS fast path: additionally K and N in whole 16-byte chunks
  const bool fast = aligned && (p.K % 8 == 0) && (p.N % 8 == 0);
  auto tiles = [&](int t) { return (int64_t)((p.M + t - 1) / t) * ((p.N + t - 1) / t); };
  // a tile much larger than the problem wastes most of its MFMAs: require 3/4 of the tile edge in both dimensions
  const bool ok256 = p.M >= 192 && p.N >= 192, ok128 = p.M >= 96 && p.N >= 96;
  const int tile = (ok256 && tiles(256) >= 192) ? 256 : ((ok128 && tiles(128) >= 192) ? 128 : 64);
  if (fast) {
    // AC_BF16_VARIANT selects an alternative schedule of the large-tile kernel (a tuning aid; default 10:
    // eight waves in ping-pong over four 32 KB LDS stages)
    static const int variant = getenv("AC_BF16_VARIANT") ? atoi(getenv("AC_BF16_VARIANT")) : 10;
    if (tile == 256) {
      switch (variant) {
        case 1: return launch_dtl<TypeBF16, EpilogueF32, 256, 256, 2, 4, 0, 2, 128>(p, stream);
        case 2: return launch_dtl<TypeBF16, EpilogueF32, 256, 256, 4, 2, 0, 2, 128>(p, stream);
        case 3: return launch_dtl<TypeBF16, EpilogueF32, 256, 256, 2, 2, 0, 4, 64>(p, stream);
        case 4: return launch_dtl<TypeBF16, EpilogueF32, 256, 256, 2, 4, 0, 4, 64>(p, stream);
        case 5: return launch_dtl<TypeBF16, EpilogueF32, 256, 128, 2, 2, 0, 3, 128>(p, stream);
        case 6: return launch_dtl<TypeBF16, EpilogueF32, 256, 128, 4, 2, 0, 3, 128>(p, stream);
        case 7: return launch_dtl<TypeBF16, EpilogueF32, 128, 256, 2, 2, 0, 3, 128>(p, stream);
        case 8: return launch_dtl<TypeBF16, EpilogueF32, 256, 128, 2, 2, 0, 6, 64>(p, stream);
        case 9: return launch_dtl<TypeBF16, EpilogueF32, 256, 256, 4, 2, 0, 4, 64>(p, stream);
        case 11: return launch_dtl<TypeBF16, EpilogueF32, 256, 256, 4, 2, 0, 4, 64, true>(p, stream);
        case 13: return launch_dtl<TypeBF16, EpilogueF32, 256, 128, 4, 2, 0, 3, 64, true>(p, stream);
        case 14: return launch_dtl<TypeBF16, EpilogueF32, 256, 128, 4, 2, 0, 3, 64, false>(p, stream);
        case 15: return launch_dtl<TypeBF16, EpilogueF32, 256, 128, 2, 4, 0, 3, 64, true>(p, stream);
        case 16: return launch_dtl<TypeBF16, EpilogueF32, 128, 256, 2, 4, 0, 3, 64, true>(p, stream);
        case 17: return launch_dtl<TypeBF16, EpilogueF32, 256, 128, 2, 2, 0, 3, 64, false>(p, stream);
        case 18: return launch_dtl<TypeBF16, EpilogueF32, 128, 128, 2, 2, 0, 4, 64, false>(p, stream);
        case 12: return launch_dtl<TypeBF16, EpilogueF32, 256, 256, 2, 4, 0, 3, 64, true>(p, stream);
        case 0: return launch_dtl<TypeBF16, EpilogueF32, 256, 256, 2, 2, 0, 2, 128>(p, stream);
        default: return launch_dtl<TypeBF16, EpilogueF32, 256, 256, 2, 4, 0, 4, 64, true>(p, stream);
      }
    }
    if (tile == 128) return launch_dtl<TypeBF16, EpilogueF32, 128, 128, 2, 2, 0, 3>(p, stream);
    return launch_dtl<TypeBF16, EpilogueF32, 64, 64, 2, 2, 0, 4>(p, stream);
  }
#define AC_BF16_LAUNCH(TILE)                                                                        \
  (aligned ? launch_tile<TypeBF16, EpilogueF32, TILE, TILE, 2, 2, 0, true>(p, stream)               \
           : launch_tile<TypeBF16, EpilogueF32, TILE, TILE, 2, 2, 0, false>(p, stream))
  switch (tile) {
    case 256: return AC_BF16_LAUNCH(256);
    case 128: return AC_BF16_LAUNCH(128);
    default: return AC_BF16_LAUNCH(64);
  }
#undef AC_BF16_LAUNCH
}

}  // namespace ac
