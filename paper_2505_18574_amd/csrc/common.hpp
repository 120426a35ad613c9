// Shared host/device declarations of the gfx950 kernels: vector types, the
// problem descriptors the host fills in, and the launcher prototypes that the
// C-ABI layer (api.cpp) calls.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace ac {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// x / d by one multiply, exact while x * d < 2^32 (the host checks the ranges it is used on).
struct FastDiv {
  unsigned magic, d;
  __host__ __device__ static FastDiv make(unsigned d) { return FastDiv{d > 1 ? (unsigned)(0x100000000ull / d) + 1u : 0u, d}; }
  __device__ __forceinline__ unsigned div(unsigned x) const { return d == 1 ? x : __umulhi(x, magic); }
};

// Compute units of the device that was current at the first call (256 if the query fails).  A function-local
// static: initialised once, safely under concurrent first calls.  The library serves one GPU per process.
inline int compute_units() {
  static const int cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    return n;
  }();
  return cus;
}

// Raises a kernel's dynamic-LDS limit.
template <class K>
inline hipError_t allow_dynamic_lds(K kern, int bytes) {
  return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}
// The same, once per kernel instantiation: `done` is the launcher's function-local flag.  Only success is
// remembered; a failure goes back to the caller and the next launch tries again.  Concurrent first launches may
// both make the call, which is harmless.
template <class K>
inline hipError_t allow_dynamic_lds_once(std::atomic<bool>& done, K kern, int bytes) {
  if (done.load(std::memory_order_acquire)) return hipSuccess;
  const hipError_t e = allow_dynamic_lds(kern, bytes);
  if (e == hipSuccess) done.store(true, std::memory_order_release);
  return e;
}

// One descriptor serves the int8 GEMM, the int8 implicit-GEMM convolution and
// the bf16 GEMM: all three are C[M][N] = epilogue(A[M][K] . B[K][N]).
struct GemmParams {
  const void* A;        // GEMM: M x K row-major.  Convolution: the NHWC input image.
  const void* B;        // K x N row-major (convolution: [KH][KW][Cin][Cout])
  void* C;              // M x N row-major
  const int32_t* bias;  // int8 paths only; may be null
  int64_t lda, ldb, ldc, bias_ld;  // in elements; bias_ld == 0 broadcasts one row
  int32_t M, N, K;
  int32_t shift, act;   // int8 output stage
  float alpha, beta;    // bf16 epilogue
  // convolution geometry (implicit GEMM: m -> (n, oh, ow), k -> (kh, kw, ci))
  int32_t H, W, Cin, KW, OH, OW, stride, pad;
  int32_t KH;            // kernel rows (K == KH * KW * Cin)
  int32_t a_bytes;       // convolution: bytes of the whole input (Nb * H * W * Cin), the range of the bounds-checked gather
  FastDiv dCin, dKW, dOW, dOH;  // convolution index arithmetic of the direct-to-LDS gather
  // split-K: number of K slices; int8 slices leave int32 partial sums in a workspace, bf16 slices add into C
  int32_t splits;        // number of K slices (1 = no split)
  int32_t kt_per_split;  // K tiles (of the launched kernel's tile depth) per slice
  int32_t* partial;      // int8: [splits][M][N] int32 partial sums when splits > 1
};

struct BatchedParams {
  const float* A;
  const float* B;
  float* C;        // may be null
  const float* x;  // may be null
  const float* d;  // may be null
  float* y;        // non-null iff x is
  int32_t n;
  int64_t batch;
};

struct TinyMpcParams {
  const float* Adyn;  // [nx][nx]
  const float* Bdyn;  // [nx][nu]
  const float* Kinf;  // [nu][nx]
  const float* x0;    // [batch][nx]
  const float* d;     // [batch][horizon][nu]
  float* u;           // [batch][horizon][nu]
  float* x_out;       // [batch][horizon + 1][nx] or null
  int32_t nx, nu, horizon;
  int64_t batch;
};

// Block tile and K split of one GEMM launch.  Chosen by the library from the shape (plan_gemm_*), or named
// by the caller through the planned entry points (make_plan_*), which is what a tuner drives.
struct GemmPlan {
  int tile;          // block tile code: 64, 128, 256 = square tile of that edge; 192 = 256 rows x 128 columns;
                     // 320 / 160 = weight-stationary kernel with 256- / 128-row tiles, 64 columns wide;
                     // 321 / 161 = convolution patch kernel with units of 256 / 128 output pixels
  int ktb;           // K bytes per tile of the kernel that serves this block tile
  int splits;        // K slices (1 = no split)
  int kt_per_split;  // K tiles per slice (0 when splits == 1)
};
// small_kernel: whether the plan may name the one-wave-per-tile kernel (tile code 32): 0 = the operands do not
// qualify for it, 1 = a GEMM that does, 2 = a convolution that does (its alternative is the tiled gather)
GemmPlan plan_gemm_i8(int32_t M, int32_t N, int32_t K, bool have_workspace, int small_kernel);
GemmPlan plan_gemm_bf16(int32_t M, int32_t N, int32_t K);
// Rows / columns of a tile code (false for an unknown code).
bool tile_dims(int32_t tile, int* bm, int* bn);
// Tile code the library picks for an M x N output when nothing else is known (convolutions, fallbacks).
int choose_tile(int32_t M, int32_t N);
// Kernel / tile code for a GEMM with more than 256 tiles of 64 x 64 (more than the chip holds at once), from
// per-code time estimates  t = c0 + rounds * (c1 + c2 * k)  with k = K bytes / 128 and rounds = the number of
// times the code's workgroups fill the chip (tiled codes), or  t = c0 + rounds * (c1 k + c2 r + c3 r k)  with r =
// row tiles per workgroup (the weight-stationary codes, int8 only, where K and the bias layout admit them).  The
// coefficients are least-squares fits to the measured times of every code on some 300 int8 and 200 bf16 shapes
// (M, N 256..16384, K 64..8192); on shapes held out of the fit the chosen code is on average 1 % slower than
// the best one (worst case 24 %), against 10 % (63 %) for thresholds on the tile count alone.
bool many_tiles(int32_t M, int32_t N, int64_t kbytes);
int choose_tile_i8(int32_t M, int32_t N, int32_t K, bool allow_weight_stationary);
int choose_tile_bf16(int32_t M, int32_t N, int32_t K);
// Explicit plans: false when the tile code is unknown, or splits is outside 1 .. number of K tiles.
// Tile and K slices for a problem whose 64 x 64 tiles would leave most of the chip idle: the pair that minimises
//   max(memory term, serial term) + slicing cost, with
//   memory term = max(operand bytes as the tiles request them / min(8 TB/s, W * r),
//                     operand bytes once                       / min(5 TB/s, W * r)),
//                 W workgroups resident, each sustaining r bytes/us on its own (loads in flight over latency);
//   serial term = K tiles per slice * time of one K tile of that kernel with warm operands;
//   slicing     = a fixed cost (the extra launch) + slices * M * N / the rate the partial sums are combined at.
// A bigger tile requests each operand fewer times but offers fewer, slower-starting streams; slicing restores the
// stream count until the traffic of the partial sums outweighs it.  Slices keep at least four K tiles and fit
// the chip in one round.  The constants are fitted to plan tables measured on this chip, one set per data type.
// bf16 slices that add into C with atomics make the last bits of the result vary from run to run, so the bf16
// model cuts K only where that clearly pays (split_margin 0.8); int8 sums are exact in any order (1.0).
struct SliceModel {
  double stream[4];    // r of the tile codes 64, 128, 192, 256 (bytes/us)
  double ktile_us[4];  // time of one K tile of those kernels
  double slice_fix_us, combine_per_us;
  double split_margin;  // a cut plan is taken only if its estimate is below this fraction of the best uncut plan's
};
void plan_few_tiles(int32_t M, int32_t N, int64_t kbytes, bool may_slice, const SliceModel& model, int* tile, int* splits);
bool make_plan_i8(int32_t K, int32_t tile, int32_t splits, GemmPlan* plan);
bool make_plan_bf16(int32_t K, int32_t tile, int32_t splits, GemmPlan* plan);

// Launchers.  `forced` null: the library plans.  A forced plan with splits > 1 needs the fast (direct-to-LDS)
// path; the launcher returns hipErrorInvalidValue when the operands do not qualify for it.
hipError_t launch_tinympc_forward(const TinyMpcParams& p, hipStream_t stream);
hipError_t launch_gemm_i8(const GemmParams& p, hipStream_t stream, const GemmPlan* forced = nullptr);
hipError_t launch_gemm_i8_acc32(const GemmParams& p, hipStream_t stream);
hipError_t launch_gemm_i8_trans(const GemmParams& p, bool trans_a, bool trans_b, hipStream_t stream);
hipError_t launch_conv2d_i8(const GemmParams& p, hipStream_t stream, const GemmPlan* forced = nullptr);
// The direct-to-LDS loaders address a lane's 16-byte chunk as a wave-uniform 64-bit base plus a 32-bit byte offset
// that spans up to 320 rows of A or 128 rows of B.  Row pitches beyond these limits (rows of 13 MB and more) take the
// generic kernels, whose lanes carry 64-bit addresses.
inline bool lane_offsets_fit(int64_t a_pitch_bytes, int64_t b_pitch_bytes) {
  const int64_t span = (1ll << 32) - 65536;
  return a_pitch_bytes * 320 < span && b_pitch_bytes * 128 < span;
}
// True when the weight-stationary kernel behind `tile` (320 / 160) can run p: bias absent or a row, K resident.
bool wstat_eligible(const GemmParams& p, int tile);
// True when the convolution patch kernel behind `tile` (321 / 161) can run the convolution described by p.
bool conv_halo_eligible(const GemmParams& p, int tile);
hipError_t launch_gemm_bf16(const GemmParams& p, hipStream_t stream, const GemmPlan* forced = nullptr);
// Size of the partial-sum buffer that lives in the code object (AC_STATIC_SCRATCH_BYTES of the C header), and the
// device address of the current GPU's copy of it (resolved on the first call per GPU, kept afterwards).
constexpr size_t STATIC_SCRATCH_BYTES = 16u << 20;
hipError_t static_scratch(void** ptr);
hipError_t launch_batched_f32(const BatchedParams& p, hipStream_t stream);
bool gemm_i8_fast_path(const GemmParams& p);
bool conv_i8_fast_path(const GemmParams& p);
bool gemm_bf16_fast_path(const GemmParams& p);

}  // namespace ac
