// bf16 GEMM, fp32 accumulate and output: tile selection and launch.
#include "gemm_mfma.hpp"

namespace ac {

hipError_t launch_gemm_bf16(const GemmParams& p, hipStream_t stream) {
  const bool aligned = (((uintptr_t)p.A & 15) == 0) && (((uintptr_t)p.B & 15) == 0) && (p.lda % 8 == 0) && (p.ldb % 8 == 0) &&
                       (((uintptr_t)p.C & 15) == 0) && (p.ldc % 4 == 0);
  auto tiles = [&](int t) { return (int64_t)((p.M + t - 1) / t) * ((p.N + t - 1) / t); };
#define AC_BF16_LAUNCH(TILE)                                                                        \
  (aligned ? launch_tile<TypeBF16, EpilogueF32, TILE, TILE, 2, 2, 0, true>(p, stream)               \
           : launch_tile<TypeBF16, EpilogueF32, TILE, TILE, 2, 2, 0, false>(p, stream))
  if (tiles(256) >= 192) return AC_BF16_LAUNCH(256);
  if (tiles(128) >= 192) return AC_BF16_LAUNCH(128);
  return AC_BF16_LAUNCH(64);
#undef AC_BF16_LAUNCH
}

}  // namespace ac
