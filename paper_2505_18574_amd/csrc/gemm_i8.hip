// int8 GEMM / implicit-GEMM convolution with the accelerator output stage: tile selection, split-K and launch.
#include "conv_halo.hpp"
#include "gemm_small.hpp"
#include "gemm_wstat.hpp"

#include <algorithm>
#include <mutex>

namespace ac {

// Partial-sum buffer of ac_gemm_i8_static, the entry point for callers that cannot allocate device memory.  It
// lives in the code object: every GPU that loads the library holds its own copy, at its own address, until the
// process ends.  In host code the name below is only a handle for hipGetSymbolAddress; the device address it
// resolves to (one per GPU) is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

hipError_t static_scratch(void** ptr) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex lock;
  static void* resolved[MAX_DEVICES] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> guard(lock);
  if (resolved[dev] == nullptr) {  // first call on this GPU (it is the current one): resolve its copy's address
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    resolved[dev] = p;
  }
  *ptr = resolved[dev];
  return hipSuccess;
}

static int ktb_of_tile(int tile) { return tile == 256 || tile == 32 ? 64 : 128; }  // K bytes per tile of the kernel behind a tile code

bool tile_dims(int32_t tile, int* bm, int* bn) {
  switch (tile) {
    case 32: *bm = *bn = 32; return true;    // one wave per tile (gemm_small.hpp), int8 GEMM only
    case 64: *bm = *bn = 64; return true;
    case 128: *bm = *bn = 128; return true;
    case 192: *bm = 256; *bn = 128; return true;
    case 256: *bm = *bn = 256; return true;
    case 320: *bm = 256; *bn = 64; return true;  // weight-stationary kernel
    case 160: *bm = 128; *bn = 64; return true;
    case 321: *bm = 256; *bn = 64; return true;  // convolution patch kernel
    case 161: *bm = 128; *bn = 64; return true;
    default: return false;
  }
}

// Shared by both GEMM types: the largest tile that still gives most compute units a workgroup (thresholds from
// exhaustive plan tables on this chip).  A tile much wider or taller than the problem wastes most of its MFMAs,
// so a tile needs 3/4 of its edge in both dimensions.
int choose_tile(int32_t M, int32_t N) {
  auto tiles = [&](int bm, int bn) { return (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
  if (M >= 192 && N >= 192 && tiles(256, 256) >= 192) return 256;
  if (M >= 192 && N >= 96 && tiles(256, 128) >= 192) return 192;
  if (M >= 96 && N >= 96 && tiles(128, 128) >= 128) return 128;
  return 64;
}

namespace {
// The plan tables and fits below were measured on the 256 compute units of an MI355X, and the planners are pure host
// arithmetic (the workspace size they imply must not depend on which device happens to be current): they count
// rounds and slots for that chip.  On another compute-unit count the plans stay valid and are merely untuned; the
// launchers size their grids from the device's own count.
constexpr int PLAN_CUS = 256;
struct TiledCost { double c0, per_round, per_round_k; };
struct StationaryCost { double c0, per_k, per_row_tile, per_row_tile_k; };
// time estimate (us) of a tiled code: bm x bn tiles, per_cu workgroups resident per compute unit
double tiled_estimate(const TiledCost& c, int bm, int bn, int per_cu, int32_t M, int32_t N, int64_t k128) {
  const int64_t tiles = (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn), slots = PLAN_CUS * per_cu;
  const double rounds = (double)((tiles + slots - 1) / slots);
  return c.c0 + rounds * (c.per_round + c.per_round_k * (double)k128);
}
// ... of a weight-stationary code: every column block of 64 gets the same number of persistent workgroups
double stationary_estimate(const StationaryCost& c, int bm, int32_t M, int32_t N, int64_t k128) {
  const int64_t nblk = (N + 63) / 64, tm = (M + bm - 1) / bm;
  int64_t wgs = nblk <= PLAN_CUS ? PLAN_CUS / nblk : 1;
  if (wgs > tm) wgs = tm;
  if (wgs < 1) wgs = 1;
  const double per = (double)((tm + wgs - 1) / wgs), rounds = (double)((wgs * nblk + PLAN_CUS - 1) / PLAN_CUS);
  return c.c0 + rounds * (c.per_k * (double)k128 + c.per_row_tile * per + c.per_row_tile_k * per * (double)k128);
}
int cheapest_tiled(const TiledCost (&c)[4], int32_t M, int32_t N, int64_t k128, double* cost) {
  static const int codes[4] = {64, 128, 192, 256}, per_cu[4] = {2, 1, 1, 1};
  int best = 64;
  // from three rounds of 256 x 256 tiles on, only that tile: the fits stop at 8192 x 8192 outputs, and beyond
  // them the smaller tiles' estimates grow too slowly (32768 x 32768 x 32 bf16: 814 us against 1006 us on 128 x 128)
  const bool huge = (int64_t)((M + 255) / 256) * ((N + 255) / 256) >= 768;
  for (int i = huge ? 3 : 0; i < 4; i++) {
    int bm, bn;
    tile_dims(codes[i], &bm, &bn);
    const double t = tiled_estimate(c[i], bm, bn, per_cu[i], M, N, k128);
    if (i == 0 || huge || t < *cost) *cost = t, best = codes[i];
  }
  return best;
}
}  // namespace

// Which of the two estimates plans a GEMM: the per-code one (unsplit) from 257 tiles of 64 x 64 on, except that up
// to 512 tiles (one round of that kernel) a K of 4096 bytes or more still goes to plan_few_tiles, which may slice
// it.  Exhaustive tile x slice tables of 43 shapes with 257 .. 2048 tiles and K 1024 .. 32768: up to 512 tiles the
// unsplit choice misses by up to 2.06x at K = 32768 and 1.4x at 8192 where plan_few_tiles misses by at most 1.13x;
// from 576 tiles on the unsplit choice is the table's best on every shape and plan_few_tiles misses by up to 1.26x.
bool many_tiles(int32_t M, int32_t N, int64_t kbytes) {
  const int64_t tiles64 = (int64_t)((M + 63) / 64) * ((N + 63) / 64);
  return tiles64 > 512 || (tiles64 > 256 && kbytes < 4096);
}

int choose_tile_i8(int32_t M, int32_t N, int32_t K, bool allow_weight_stationary) {
  static const TiledCost tiled[4] = {{1.298, 1.791, 0.3930}, {1.564, 3.370, 0.4437}, {1.075, 6.635, 0.7549}, {-1.198, 10.768, 1.0961}};
  static const StationaryCost st160 = {2.414, 0.0705, 1.0672, 0.4786}, st320 = {2.397, 0.0043, 1.2743, 0.6840};
  const int64_t k128 = ((int64_t)K + 127) / 128;
  double cost = 0.0;
  int best = cheapest_tiled(tiled, M, N, k128, &cost);
  if (allow_weight_stationary && K >= 16) {
    if (k128 <= wstat_max_kt(160)) {
      const double t = stationary_estimate(st160, 128, M, N, k128);
      if (t < cost) cost = t, best = 160;
    }
    if (k128 <= wstat_max_kt(320)) {
      const double t = stationary_estimate(st320, 256, M, N, k128);
      if (t < cost) cost = t, best = 320;
    }
  }
  return best;
}

int choose_tile_bf16(int32_t M, int32_t N, int32_t K) {
  static const TiledCost tiled[4] = {{1.944, 1.630, 0.3737}, {1.479, 3.315, 0.4174}, {-0.530, 7.057, 0.6704}, {-6.486, 15.278, 0.9995}};
  double cost = 0.0;
  return cheapest_tiled(tiled, M, N, ((int64_t)K * 2 + 127) / 128, &cost);
}

// The weight-stationary kernel takes direct-to-LDS operands (checked by the caller), no bias or a bias row, and a
// K whose 64-column block of B fits in LDS beside the ring of A stages.
bool wstat_eligible(const GemmParams& p, int tile) {
  int bm;
  if (!wstat_tile_rows(tile, &bm)) return false;
  const int nkt = (p.K + 127) / 128;
  return p.K >= 1 && nkt <= wstat_max_kt(tile) && (p.bias == nullptr || p.bias_ld == 0);
}

bool conv_halo_eligible(const GemmParams& p, int tile) {
  int bm;
  ConvHaloParams h;
  size_t lds = 0;
  return halo_tile_rows(tile, &bm) && conv_halo_plan(p, bm, &h, &lds);
}

// Kernel / tile and K split for an M x N x K int8 problem.  With more 64 x 64 tiles than the chip holds at once:
// the code with the lowest time estimate (choose_tile_i8), unsplit.  With fewer: tile and K slices together from
// the cost estimate of plan_few_tiles (slicing needs the caller's workspace for the int32 partial sums).
GemmPlan plan_gemm_i8(int32_t M, int32_t N, int32_t K, bool have_workspace, int small_kernel) {
  GemmPlan plan;
  plan.splits = 1;
  plan.kt_per_split = 0;
  plan.tile = 64;
  plan.ktb = ktb_of_tile(plan.tile);
  if (M < 1 || N < 1) return plan;
  // Launches of a few microseconds: the one-wave-per-tile kernel, where a sweep of 33 outputs (4 to 6272 tiles of
  // 32 x 32) x 14 depths on this chip has it ahead of every tiled plan with operands in the caches and level with
  // them with operands in HBM: the fewer the tiles, the deeper the K that a lone wave per tile still wins with (at
  // 1024 tiles the 64 x 64 tiles share operands through LDS and win from K = 512).  Warm margins: 256^3 2.9 vs
  // 3.6 us, 512 x 768 x 768 3.9 vs 4.6, 128 x 1024 x 1024 3.9 vs 4.5, 2048 x 1024 x 192 4.2 vs 4.6.  Between 1024
  // and 2048 tiles K = 256 .. 320 is ahead by 2-4 % on most shapes and behind by up to 20 % on some (1024 x 1744 x
  // 320: 7.2 against 6.0 us), so the rule stops at 192 there.  Deeper K with few tiles is also ahead warm (128 x
  // 1024 x 3072: 6.8 vs 8.8 us for a cut K) but well behind from HBM (14.5 vs 10.6 us: a cut K has eight times the
  // loads in flight), and 784 x 512 x 1152 gives from HBM what it gains warm (7.9 vs 7.0, 4.6 vs 5.0): both stay on
  // the tiled plans.  Against the convolution gather of the 64 x 64 tiles it stays ahead further: 8 images of
  // 56 x 56 x 64 -> 64 (1568 tiles, K = 576) 5.7 against 6.5 us warm, 6.5 against 6.9 from HBM; not at 3136 tiles
  // (11.9 against 8.0).
  if (small_kernel != 0 && K >= SMALL_KTB && K % SMALL_KTB == 0) {
    const int64_t tiles32 = (int64_t)((M + 31) / 32) * ((N + 31) / 32);
    int kmax = tiles32 <= 512 ? 1024 : tiles32 <= 1024 ? 384 : tiles32 <= 2048 ? 192 : 0;
    if (small_kernel == 2 && tiles32 <= 2048 && kmax < 640) kmax = 640;
    if (K <= kmax) {
      make_plan_i8(K, 32, 1, &plan);
      return plan;
    }
  }
  if (many_tiles(M, N, K)) {
    plan.tile = choose_tile_i8(M, N, K, true);
    plan.ktb = ktb_of_tile(plan.tile);
    return plan;
  }
  {
    // Constants from the plan tables of 23 int8 shapes (worst miss 38 % over a table's best; the rule this replaces,
    // eight slices of the 64 x 64 tile from 64 K tiles on, missed by up to 3.8x on deep K).  The slices' int32
    // partial sums go through the caller's workspace and a second launch combines them.  The tables are timed on
    // warm operands, where that second launch costs 7 us; the fixed cost used here is 5 us, which moves one
    // boundary case: 49 x 2048 x 4608 (9.4 MB of weights behind 32 tiles) takes four slices, 9.3 us instead of
    // 7.9 us on warm operands but 12.7 instead of 22.2 us when the weights come from HBM, as they do whenever
    // anything else ran since the last call (a compute unit sustains only some 50 GB/s of cold misses, so few
    // workgroups cannot stream weights however deep their prefetch).  For the same reason the stream rate of a
    // 64 x 64 workgroup is the cold one (its four 16 KB stages in flight over some 2 us of HBM latency: 32 GB/s;
    // the warm tables gave 60): over eighteen further few-tile shapes the library's choices then take 214 us in
    // sum on operands from HBM against 260 us, and 152 against 158 us on operands from the caches.
    static const SliceModel model = {{32e3, 45e3, 40e3, 25e3}, {0.066, 0.132, 0.198, 0.24}, 5.0, 4e5, 1.0};
    int tile = 64, splits = 1;
    plan_few_tiles(M, N, K, have_workspace, model, &tile, &splits);
    make_plan_i8(K, tile, splits, &plan);
  }
  return plan;
}

// Shared by the int8 and bf16 explicit plans: `splits` slices of ceil(nkt / splits) K tiles each.
static bool make_plan(int64_t kbytes, int tile, int ktb, int splits, GemmPlan* plan) {
  const int64_t nkt = (kbytes + ktb - 1) / ktb;
  if (splits < 1 || (splits > 1 && splits > nkt)) return false;
  plan->tile = tile;
  plan->ktb = ktb;
  plan->splits = 1;
  plan->kt_per_split = 0;
  if (splits > 1) {
    const int per = (int)((nkt + splits - 1) / splits);
    plan->kt_per_split = per;
    plan->splits = (int)((nkt + per - 1) / per);  // slices that actually hold K tiles
    if (plan->splits <= 1) {
      plan->splits = 1;
      plan->kt_per_split = 0;
    }
  }
  return true;
}

bool make_plan_i8(int32_t K, int32_t tile, int32_t splits, GemmPlan* plan) {
  int bm, bn;
  if (!tile_dims(tile, &bm, &bn)) return false;
  if ((wstat_tile_rows(tile, &bm) || halo_tile_rows(tile, &bm)) && splits != 1) return false;  // these kernels keep all of K resident
  if (tile == 32 && (K < SMALL_KTB || K % SMALL_KTB != 0)) return false;                           // whole K tiles of 64 bytes
  return make_plan(K, tile, ktb_of_tile(tile), splits, plan);
}

bool make_plan_bf16(int32_t K, int32_t tile, int32_t splits, GemmPlan* plan) {
  int bm, bn;
  if (!tile_dims(tile, &bm, &bn) || tile == 32 || wstat_tile_rows(tile, &bm) || halo_tile_rows(tile, &bm)) return false;
  return make_plan((int64_t)K * 2, tile, ktb_of_tile(tile), splits, plan);
}

void plan_few_tiles(int32_t M, int32_t N, int64_t kbytes, bool may_slice, const SliceModel& model, int* tile, int* splits) {
  static const int codes[4] = {64, 128, 192, 256};
  static const int per_cu[4] = {2, 1, 1, 1};  // workgroups of that kernel a compute unit holds (LDS)
  const double once = (double)kbytes * ((double)M + N);
  double best = 0.0, best_uncut = 0.0;
  int tile_uncut = 64;
  *tile = 64, *splits = 1;
  if (M < 1 || N < 1 || kbytes < 1) return;
  if ((int64_t)((M + 63) / 64) * ((N + 63) / 64) > 512) return;  // more than one round of 64 x 64 tiles: outside the fitted range
  for (int c = 0; c < 4; c++) {
    int bm, bn;
    tile_dims(codes[c], &bm, &bn);
    const int ktb = ktb_of_tile(codes[c]);
    const int64_t tm = (M + bm - 1) / bm, tn = (N + bn - 1) / bn;
    const int64_t nkt = (kbytes + ktb - 1) / ktb, slots = PLAN_CUS * per_cu[c];
    const double requested = (double)kbytes * ((double)tm * bm * tn + (double)tn * bn * tm);
    for (int s = 1; s <= PLAN_CUS; s *= 2) {
      const int64_t items = tm * tn * s;
      if (s > 1 && (!may_slice || items > slots || (int64_t)s * 4 > nkt)) break;
      const double rate = (double)(items < slots ? items : slots) * model.stream[c];
      const double mem = std::max(requested / std::min(8e6, rate), once / std::min(5e6, rate));
      const double serial = (double)((items + slots - 1) / slots) * (double)((nkt + s - 1) / s) * model.ktile_us[c];
      const double est = std::max(mem, serial) + (s > 1 ? model.slice_fix_us + (double)s * M * N / model.combine_per_us : 0.0);
      if ((c == 0 && s == 1) || est < best) best = est, *tile = codes[c], *splits = s;
      if (s == 1 && (c == 0 || est < best_uncut)) best_uncut = est, tile_uncut = codes[c];
    }
  }
  if (*splits > 1 && best > model.split_margin * best_uncut) *tile = tile_uncut, *splits = 1;
}

// Output stage of a split-K launch: sum the K slices, then bias / shift / saturate / ReLU, 4 outputs per thread.
template <int THREADS>
__global__ void __launch_bounds__(THREADS) splitk_reduce_i8_kernel(const GemmParams p) {
  const int64_t quads_per_row = p.N / 4;  // split-K is only used on the fast path: N is a multiple of 16
  const int64_t q = (int64_t)blockIdx.x * THREADS + threadIdx.x;
  if (q >= (int64_t)p.M * quads_per_row) return;
  const int m = (int)(q / quads_per_row);
  const int n = (int)(q - (int64_t)m * quads_per_row) * 4;
  v4i s = {0, 0, 0, 0};
  const int32_t* part = p.partial + (int64_t)m * p.N + n;
  const int64_t slice = (int64_t)p.M * p.N;
  int k = 0;
  for (; k + 8 <= p.splits; k += 8) {  // eight loads in flight: the slices of one output are a latency chain otherwise
    v4i v[8];
#pragma unroll
    for (int u = 0; u < 8; u++) v[u] = *(const v4i*)(part + (k + u) * slice);
#pragma unroll
    for (int u = 0; u < 8; u++) s += v[u];
  }
  for (; k < p.splits; k++) s += *(const v4i*)(part + k * slice);
  int a4[4] = {s[0], s[1], s[2], s[3]};
  EpilogueI8::store4<true>(p, m, n, a4);
}

// One-wave workgroups for small outputs: the kernel is a chain of latencies, and four times the workgroups spread
// it over four times the compute units (49 x 2048 x 4608 in 8 slices: 8.7 -> 7.3 us for the whole call, 32 x 2048 x
// 2048 7.8 -> 6.6; level or within 0.3 us on nine other shapes; from 50176 outputs of four on, 256 threads again).
static hipError_t launch_splitk_reduce_i8(const GemmParams& p, hipStream_t stream) {
  const int64_t quads = (int64_t)p.M * (p.N / 4);
  if (quads <= 32768) hipLaunchKernelGGL(splitk_reduce_i8_kernel<64>, dim3((unsigned)((quads + 63) / 64)), dim3(64), 0, stream, p);
  else hipLaunchKernelGGL(splitk_reduce_i8_kernel<256>, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, p);
  return hipGetLastError();
}

template <int AMODE>
hipError_t dispatch_i8(GemmParams p, hipStream_t stream, bool aligned, bool fast, const GemmPlan* forced) {
  // the one-wave-per-tile kernel is planned only for operands it takes
  GemmPlan plan = forced ? *forced : plan_gemm_i8(p.M, p.N, p.K, fast && p.partial != nullptr, fast && small_i8_eligible(p) ? 1 + AMODE : 0);
  int ws_bm;
  if (!forced && wstat_tile_rows(plan.tile, &ws_bm) && !(fast && wstat_eligible(p, plan.tile))) {
    plan.tile = choose_tile_i8(p.M, p.N, p.K, false);  // operands the weight-stationary kernel does not take: the tiled kernels
    plan.ktb = ktb_of_tile(plan.tile);
  }
  p.splits = plan.splits;
  p.kt_per_split = plan.kt_per_split;
  if (plan.splits > 1 && (!fast || p.partial == nullptr)) return hipErrorInvalidValue;
  if (wstat_tile_rows(plan.tile, &ws_bm)) {
    if (!fast || !wstat_eligible(p, plan.tile)) return hipErrorInvalidValue;
    return launch_wstat_tile<AMODE>(plan.tile, p, stream);
  }
  if (plan.tile == 32) {
    if (!fast || !small_i8_eligible(p)) return hipErrorInvalidValue;
    const hipError_t e = launch_small_i8<AMODE>(p, stream);
    if (e != hipSuccess || plan.splits <= 1) return e;
    return launch_splitk_reduce_i8(p, stream);
  }
  if (halo_tile_rows(plan.tile, &ws_bm)) {
    ConvHaloParams h;
    size_t lds = 0;
    if (AMODE != 1 || !fast || !conv_halo_plan(p, ws_bm, &h, &lds)) return hipErrorInvalidValue;
    return ws_bm == 256 ? launch_conv_halo<256>(p, h, lds, stream) : launch_conv_halo<128>(p, h, lds, stream);
  }
  if (fast) {  // direct-to-LDS kernels
    if (plan.splits > 1) {
      hipError_t e = launch_dtl_tile<TypeI8, EpiloguePartialI32, AMODE>(plan.tile, p, stream);
      if (e != hipSuccess) return e;
      return launch_splitk_reduce_i8(p, stream);
    }
    return launch_dtl_tile<TypeI8, EpilogueI8, AMODE>(plan.tile, p, stream);
  }
#define AC_I8_CASE(TILE, WM, WN)                                                                         \
  case TILE:                                                                                             \
    return aligned ? launch_tile<TypeI8, EpilogueI8, TILE, TILE, WM, WN, AMODE, true>(p, stream)         \
                   : launch_tile<TypeI8, EpilogueI8, TILE, TILE, WM, WN, AMODE, false>(p, stream);
  switch (plan.tile == 192 ? 128 : plan.tile) {  // the generic kernel has square tiles only
    AC_I8_CASE(256, 2, 2)
    AC_I8_CASE(128, 2, 2)
    AC_I8_CASE(64, 2, 2)
  }
#undef AC_I8_CASE
  return hipErrorInvalidValue;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// Fast (direct-to-LDS) path: 16-byte aligned operands and pitches, K and N in whole 16-byte chunks.
bool gemm_i8_fast_path(const GemmParams& p) {
  return aligned16(p.A) && aligned16(p.B) && (p.lda % 16 == 0) && (p.ldb % 16 == 0) && (((uintptr_t)p.C & 3) == 0) &&
         (p.ldc % 4 == 0) && (p.K % 16 == 0) && (p.N % 16 == 0) && lane_offsets_fit(p.lda, p.ldb);
}

// Raw int32 accumulator output: same kernels, epilogue without the output stage (no split-K).
hipError_t launch_gemm_i8_acc32(const GemmParams& p0, hipStream_t stream) {
  GemmParams p = p0;
  p.splits = 1;
  p.kt_per_split = 0;
  const bool aligned = aligned16(p.A) && aligned16(p.B) && (p.lda % 16 == 0) && (p.ldb % 16 == 0) && aligned16(p.C) && (p.ldc % 4 == 0);
  const bool fast = aligned && (p.K % 16 == 0) && (p.N % 16 == 0) && lane_offsets_fit(p.lda, p.ldb);
  if (fast) return launch_dtl_tile<TypeI8, EpilogueRawI32, 0>(choose_tile(p.M, p.N), p, stream);  // 4-byte output: its own regime, thresholds kept
  return aligned ? launch_tile<TypeI8, EpilogueRawI32, 64, 64, 2, 2, 0, true>(p, stream)
                 : launch_tile<TypeI8, EpilogueRawI32, 64, 64, 2, 2, 0, false>(p, stream);
}

hipError_t launch_gemm_i8(const GemmParams& p, hipStream_t stream, const GemmPlan* forced) {
  const bool aligned = aligned16(p.A) && aligned16(p.B) && (p.lda % 16 == 0) && (p.ldb % 16 == 0) &&
                       (((uintptr_t)p.C & 3) == 0) && (p.ldc % 4 == 0);
  return dispatch_i8<0>(p, stream, aligned, gemm_i8_fast_path(p), forced);
}

// Direct-to-LDS path of the convolution: channel counts in multiples of 16 so that a 16-byte K chunk stays inside
// one kernel tap, at most 32 taps (one validity bit each), and index ranges that the one-multiply divisions of the
// gather cover (K * Cin, M * OW and (M / OW) * OH below 2^32).
bool conv_i8_fast_path(const GemmParams& p) {
  const bool aligned = aligned16(p.A) && aligned16(p.B) && (p.Cin % 16 == 0) && (p.ldb % 16 == 0) &&
                       (((uintptr_t)p.C & 3) == 0) && (p.ldc % 4 == 0);
  const int64_t lim = 1ll << 32;
  return aligned && p.KH >= 1 && p.KH * p.KW <= 32 && (int64_t)p.K * p.Cin < lim && (int64_t)p.M * p.OW < lim &&
         ((int64_t)p.M / (p.OW > 0 ? p.OW : 1) + 1) * p.OH < lim && p.a_bytes > 0 && lane_offsets_fit(0, p.ldb);
}

hipError_t launch_conv2d_i8(const GemmParams& p, hipStream_t stream, const GemmPlan* forced) {
  if (!forced && p.KH == 1 && p.KW == 1 && p.stride == 1 && p.pad == 0) {
    // a 1 x 1 convolution over every pixel is the GEMM (pixels x Cin) . (Cin x Cout): the plain operand loaders and
    // the GEMM planner (1 x 1, 256 -> 64 on 256 images of 56 x 56: 42 us against 71 us through the gather)
    GemmParams g = p;
    g.lda = p.Cin;
    return launch_gemm_i8(g, stream, nullptr);
  }
  const bool aligned = aligned16(p.A) && aligned16(p.B) && (p.Cin % 16 == 0) && (p.ldb % 16 == 0) &&
                       (((uintptr_t)p.C & 3) == 0) && (p.ldc % 4 == 0);
  const bool fast = conv_i8_fast_path(p);
  if (!forced && fast) {
    // The patch kernel (weights and the image patch of a unit both in LDS) as soon as the 64 x 64 tiles would
    // need a second round on the chip (more than two per compute unit), or the convolution has a unit of 256
    // output pixels per compute unit and column block.  Plan tables, 56 x 56 x 64 -> 64: 10 images (490 tiles)
    // 6.5 us tiled against 7.5 us, 12 images (588 tiles) 9.2 against 7.5, 16 images 10.0 against 7.6, 64 images
    // 28 against 17; 56 x 56 x 64 -> 128 at 8 images 10.0 against 7.7.  Below that the fixed cost of filling LDS
    // once per workgroup makes the 64 x 64 tiles the faster choice.
    ConvHaloParams h;
    size_t lds = 0;
    GemmParams q = p;
    q.splits = 1;
    q.kt_per_split = 0;
    const int64_t nblk = (p.N + 63) / 64, tiles64 = (int64_t)((p.M + 63) / 64) * nblk;
    // a single kernel tap reuses nothing of a patch: such a convolution (1 x 1 with a stride) is a gather GEMM and
    // is planned as one (64 -> 256 on 64 images of 56 x 56, stride 2: 13.1 us weight-stationary, 21.3 us patch kernel)
    const bool taps = p.KH * p.KW > 1;
    if (taps && conv_halo_plan(p, 256, &h, &lds)) {
      if (h.units * nblk >= 256 || tiles64 > 512) return launch_conv_halo<256>(q, h, lds, stream);
    } else if (taps && conv_halo_plan(p, 128, &h, &lds)) {
      // the patch of 256 pixels does not fit, that of 128 does (28 x 28 x 128 -> 128: 64 images 18.7 us against
      // 18.5 us on the best tiled kernel, 128 images 29.6 against 33.6)
      if (h.units * nblk >= 512) return launch_conv_halo<128>(q, h, lds, stream);
    } else {
      return dispatch_i8<1>(p, stream, aligned, fast, forced);
    }
    // a convolution the patch kernel could take but that is too small for it: the tiled kernels (or one wave per
    // tile, by the GEMM's rule: 56 x 56 x 64 -> 64, one image, 4.4 us against 5.4; K = 1152 gains 0.5 us with the
    // input in the caches and loses up to 1 us with it in HBM, as for the GEMM), never the weight-stationary
    // kernel, whose gather loses to both (28 x 28 x 128 -> 128, 32 images: 13.9 us against 10.2)
    GemmPlan plan = plan_gemm_i8(p.M, p.N, p.K, p.partial != nullptr, small_i8_eligible(p) ? 2 : 0);
    int ws_bm;
    if (wstat_tile_rows(plan.tile, &ws_bm)) make_plan_i8(p.K, choose_tile(p.M, p.N), 1, &plan);  // unsplit: no workspace needed
    return dispatch_i8<1>(p, stream, aligned, fast, &plan);
  }
  return dispatch_i8<1>(p, stream, aligned, fast, forced);
}

}  // namespace ac
