// int8 GEMM with the accelerator output stage: tile selection and launch.
#include "gemm_dtl.hpp"

namespace ac {

// Pick the square block tile for an M x N x K int8 problem.  The chip has 256
// compute units; a launch wants at least that many workgroups, and a bigger
// tile re-reads less of A and B.  Take the largest tile that still yields
// enough workgroups, else the smallest.
I8Plan plan_gemm_i8(int32_t M, int32_t N, int32_t K, bool have_workspace) {
  (void)K;
  (void)have_workspace;
  auto tiles = [&](int t) { return (int64_t)((M + t - 1) / t) * ((N + t - 1) / t); };
  I8Plan plan;
  plan.splits = 1;
  if (tiles(256) >= 192) plan.tile = 256;
  else if (tiles(128) >= 192) plan.tile = 128;
  else plan.tile = 64;
  return plan;
}

template <int AMODE>
hipError_t dispatch_i8(const GemmParams& p, hipStream_t stream, bool aligned, bool fast) {
  const I8Plan plan = plan_gemm_i8(p.M, p.N, p.K, p.partial != nullptr);
  if (fast) {  // direct-to-LDS kernels
    switch (plan.tile) {
      case 256: return launch_dtl<TypeI8, EpilogueI8, 256, 256, 2, 4, AMODE, 4, 64, true>(p, stream);
      case 128: return launch_dtl<TypeI8, EpilogueI8, 128, 128, 2, 2, AMODE, 3, 128>(p, stream);
      default: return launch_dtl<TypeI8, EpilogueI8, 64, 64, 2, 2, AMODE, 4, 128>(p, stream);
    }
  }
#define AC_I8_CASE(TILE, WM, WN)                                                                         \
  case TILE:                                                                                             \
    return aligned ? launch_tile<TypeI8, EpilogueI8, TILE, TILE, WM, WN, AMODE, true>(p, stream)         \
                   : launch_tile<TypeI8, EpilogueI8, TILE, TILE, WM, WN, AMODE, false>(p, stream);
  switch (plan.tile) {
    AC_I8_CASE(256, 2, 2)
    AC_I8_CASE(128, 2, 2)
    AC_I8_CASE(64, 2, 2)
  }
#undef AC_I8_CASE
  return hipErrorInvalidValue;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

hipError_t launch_gemm_i8(const GemmParams& p, hipStream_t stream) {
  const bool aligned = aligned16(p.A) && aligned16(p.B) && (p.lda % 16 == 0) && (p.ldb % 16 == 0) &&
                       (((uintptr_t)p.C & 3) == 0) && (p.ldc % 4 == 0);
  const bool fast = aligned && (p.K % 16 == 0) && (p.N % 16 == 0);
  return dispatch_i8<0>(p, stream, aligned, fast);
}

hipError_t launch_conv2d_i8(const GemmParams& p, hipStream_t stream) {
  // Fast path: channel counts in multiples of 16 so that a 16-byte K chunk stays inside one kernel tap.
  const bool aligned = aligned16(p.A) && aligned16(p.B) && (p.Cin % 16 == 0) && (p.ldb % 16 == 0) &&
                       (((uintptr_t)p.C & 3) == 0) && (p.ldc % 4 == 0);
  return dispatch_i8<1>(p, stream, aligned, aligned);
}

}  // namespace ac
