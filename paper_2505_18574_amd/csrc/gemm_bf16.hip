// bf16 GEMM, fp32 accumulate and output: tile selection, split-K and launch.
#include <algorithm>

#include "gemm_dtl.hpp"

namespace ac {

// Block tile and K split for an M x N x K bf16 problem.  With more 64 x 64 tiles than the chip holds at once: the
// tile with the lowest time estimate (choose_tile_bf16), unsplit.  With fewer, K is cut into slices that add into
// C (see EpilogueAtomicF32), and tile and slice count come from the cost estimate of plan_few_tiles with constants
// fitted to the plan tables of twenty such shapes (worst miss 18 % over a table's best, against 67 % for a rule
// that only ever slices the 64 x 64 tile): 2 us for the launch that scales C, and 200 fp32 atomic adds per ns.
// Without a workspace the slices add into C with atomics and the last bits then vary from run to run, so K is
// only cut where the estimate, atomics included, is at least a fifth below the best uncut plan's.
GemmPlan plan_gemm_bf16(int32_t M, int32_t N, int32_t K) {
  GemmPlan plan;
  make_plan_bf16(K, 64, 1, &plan);
  if (M < 1 || N < 1) return plan;
  if (many_tiles(M, N, (int64_t)K * 2)) {
    make_plan_bf16(K, choose_tile_bf16(M, N, K), 1, &plan);
    return plan;
  }
  static const SliceModel model = {{40e3, 45e3, 30e3, 25e3}, {0.192, 0.32, 0.44, 0.48}, 2.0, 2e5, 0.8};
  int tile = 64, splits = 1;
  plan_few_tiles(M, N, (int64_t)K * 2, true, model, &tile, &splits);
  make_plan_bf16(K, tile, splits, &plan);
  return plan;
}

// C = beta * C ahead of a split-K launch (beta == 0 stores zeros without reading C).
__global__ void __launch_bounds__(256) scale_c_f32_kernel(float* C, int64_t ldc, int M, int N, float beta) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)M * N) return;
  float* c = C + (i / N) * ldc + (i % N);
  *c = beta == 0.f ? 0.f : beta * *c;
}

// Output stage of a split-K launch through a workspace: C = alpha * (sum of the slices, in slice order) + beta * C.
template <int THREADS>
__global__ void __launch_bounds__(THREADS) splitk_reduce_f32_kernel(const GemmParams p) {
  const int64_t quads_per_row = p.N / 4;  // fast path: N is a multiple of 8
  const int64_t q = (int64_t)blockIdx.x * THREADS + threadIdx.x;
  if (q >= (int64_t)p.M * quads_per_row) return;
  const int m = (int)(q / quads_per_row);
  const int n = (int)(q - (int64_t)m * quads_per_row) * 4;
  const float* part = (const float*)p.partial;
  v4f s = {0.f, 0.f, 0.f, 0.f};
  part += (int64_t)m * p.N + n;
  const int64_t slice = (int64_t)p.M * p.N;
  int k = 0;
  for (; k + 8 <= p.splits; k += 8) {  // eight loads in flight; the sum still runs in slice order
    v4f v[8];
#pragma unroll
    for (int u = 0; u < 8; u++) v[u] = *(const v4f*)(part + (k + u) * slice);
#pragma unroll
    for (int u = 0; u < 8; u++) s += v[u];
  }
  for (; k < p.splits; k++) s += *(const v4f*)(part + k * slice);
  float* dst = (float*)p.C + (int64_t)m * p.ldc + n;
  v4f o = p.alpha * s;
  if (p.beta != 0.f) o += p.beta * *(const v4f*)dst;
  *(v4f*)dst = o;
}

bool gemm_bf16_fast_path(const GemmParams& p) {
  return (((uintptr_t)p.A & 15) == 0) && (((uintptr_t)p.B & 15) == 0) && (p.lda % 8 == 0) && (p.ldb % 8 == 0) &&
         (((uintptr_t)p.C & 15) == 0) && (p.ldc % 4 == 0) && (p.K % 8 == 0) && (p.N % 8 == 0) &&
         lane_offsets_fit(2 * (int64_t)p.lda, 2 * (int64_t)p.ldb);
}

hipError_t launch_gemm_bf16(const GemmParams& p0, hipStream_t stream, const GemmPlan* forced) {
  GemmParams p = p0;
  const bool aligned = (((uintptr_t)p.A & 15) == 0) && (((uintptr_t)p.B & 15) == 0) && (p.lda % 8 == 0) && (p.ldb % 8 == 0) &&
                       (((uintptr_t)p.C & 15) == 0) && (p.ldc % 4 == 0);
  // direct-to-LDS fast path: additionally K and N in whole 16-byte chunks
  const bool fast = gemm_bf16_fast_path(p);
  GemmPlan plan = forced ? *forced : plan_gemm_bf16(p.M, p.N, p.K);
  if (plan.splits > 1 && !fast) {
    if (forced) return hipErrorInvalidValue;
    make_plan_bf16(p.K, choose_tile(p.M, p.N), 1, &plan);  // the generic kernels do not slice K and have square tiles
  }
  p.splits = plan.splits;
  p.kt_per_split = plan.kt_per_split;
  if (fast) {
    if (plan.splits > 1 && p.partial != nullptr) {  // slices through the caller's workspace, summed in a fixed order
      hipError_t e = launch_dtl_tile<TypeBF16, EpiloguePartialF32, 0>(plan.tile, p, stream);
      if (e != hipSuccess) return e;
      // one-wave workgroups for small outputs, as for the int8 combine (64 x 64 x 65536 in 128 slices: 15.3 -> 13.5 us)
      const int64_t quads = (int64_t)p.M * (p.N / 4);
      if (quads <= 32768) hipLaunchKernelGGL(splitk_reduce_f32_kernel<64>, dim3((unsigned)((quads + 63) / 64)), dim3(64), 0, stream, p);
      else hipLaunchKernelGGL(splitk_reduce_f32_kernel<256>, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, p);
      return hipGetLastError();
    }
    if (plan.splits > 1) {  // no workspace: slices add into C with fp32 atomics
      const int64_t n = (int64_t)p.M * p.N;
      hipLaunchKernelGGL(scale_c_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, (float*)p.C, p.ldc, p.M, p.N, p.beta);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      return launch_dtl_tile<TypeBF16, EpilogueAtomicF32, 0>(plan.tile, p, stream);
    }
    return launch_dtl_tile<TypeBF16, EpilogueF32, 0>(plan.tile, p, stream);
  }
#define AC_BF16_LAUNCH(TILE)                                                                        \
  (aligned ? launch_tile<TypeBF16, EpilogueF32, TILE, TILE, 2, 2, 0, true>(p, stream)               \
           : launch_tile<TypeBF16, EpilogueF32, TILE, TILE, 2, 2, 0, false>(p, stream))
  switch (plan.tile) {  // the generic kernel has square tiles only: 192 falls to 128
    case 256: return AC_BF16_LAUNCH(256);
    case 192:
    case 128: return AC_BF16_LAUNCH(128);
    default: return AC_BF16_LAUNCH(64);
  }
#undef AC_BF16_LAUNCH
}

}  // namespace ac
