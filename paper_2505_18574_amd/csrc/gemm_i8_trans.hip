// int8 GEMM with transposed operands (the A_transpose / B_transpose fields of the accelerator's config_ex,
// Appendix C Fig. 14): A may be given as A^T (K x M row-major) and B as B^T (N x K row-major).
//
// Either operand of the product is, in memory, "K-contiguous" (a row holds consecutive k: plain A, transposed
// B) or "K-strided" (a row holds consecutive m or n: transposed A, plain B).  The kernel stages each operand
// tile in LDS in its memory order and picks the fragment read that matches: a 16-byte ds_read_b128 along a
// K-contiguous row, or the transposing ds_read_b64_tr_b8 pair down a K-strided tile.  Both deliver the same
// MFMA operand (row or column l % 32, 16 bytes of K selected by l / 32), so the four combinations share one
// body.  Register-staged double buffering, guarded loads: any alignment and any M, N, K.
//
// Operands that qualify for the direct-to-LDS kernels (16-byte aligned bases and pitches, M, N and K in whole
// 16-byte chunks) run on those instead, with the transposed operand in the other operand's LDS role (TA / TB of
// gemm_dtl_kernel): the same tiles, pipeline and output stage as the untransposed product.
#include <algorithm>

#include "gemm_dtl.hpp"

namespace ac {

template <int TILE>
struct TransGeometry {
  static constexpr int KT = 64;        // K bytes per step
  static constexpr int THREADS = 256;  // 2 x 2 waves
  static constexpr int WT = TILE / 2;  // wave tile edge
  static constexpr int T32 = WT / 32;  // 32x32 MFMA tiles per wave edge
  // K-contiguous tile: [TILE rows][KT + 16]; 4 chunks of 16 bytes per row
  static constexpr int KC_STRIDE = KT + 16;
  static constexpr int KC_BYTES = TILE * KC_STRIDE;
  static constexpr int KC_ROWS_PER_PASS = THREADS / 4;
  static constexpr int KC_IT = TILE / KC_ROWS_PER_PASS;
  // K-strided tile: [KT k-rows][TILE + 16]
  static constexpr int KS_STRIDE = TILE + 16;
  static constexpr int KS_BYTES = KT * KS_STRIDE;
  static constexpr int KS_CPR = TILE / 16;
  static constexpr int KS_ROWS_PER_PASS = THREADS / KS_CPR;
  static constexpr int KS_IT = KT / KS_ROWS_PER_PASS;
  static constexpr int OP_BYTES = KC_BYTES > KS_BYTES ? KC_BYTES : KS_BYTES;
  static constexpr int LDS_BYTES = 2 * 2 * OP_BYTES;  // two operands, two stages
  static constexpr int MAX_IT = KC_IT > KS_IT ? KC_IT : KS_IT;
  static_assert(KC_IT >= 1 && KS_IT >= 1 && T32 >= 1, "tile / thread mismatch");
};

// One operand of the product.  KSTRIDED: memory rows run along the tile's own dimension (m or n) and K
// advances by `ld` per row; otherwise memory rows run along K.  `origin` is the tile's first m (or n),
// `extent` is M (or N).
template <int TILE, bool KSTRIDED, bool ALIGNED>
struct TransOperand {
  using G = TransGeometry<TILE>;
  const unsigned char* base;
  int64_t ld;
  int origin, extent, K;
  v4i reg[G::MAX_IT];

  __device__ __forceinline__ void load(int k0, int t) {
    if constexpr (KSTRIDED) {
      const int cc = t % G::KS_CPR, r0 = t / G::KS_CPR;
      const int col = origin + cc * 16;
#pragma unroll
      for (int i = 0; i < G::KS_IT; i++) {
        const int k = k0 + r0 + i * G::KS_ROWS_PER_PASS;
        reg[i] = k < K ? load16<ALIGNED>(base + (int64_t)k * ld + col, extent - col) : (v4i){0, 0, 0, 0};
      }
    } else {
      const int cc = t & 3, r0 = t >> 2;
      const int kb = k0 + cc * 16;
#pragma unroll
      for (int i = 0; i < G::KC_IT; i++) {
        const int row = origin + r0 + i * G::KC_ROWS_PER_PASS;
        reg[i] = row < extent ? load16<ALIGNED>(base + (int64_t)row * ld + kb, K - kb) : (v4i){0, 0, 0, 0};
      }
    }
  }
  __device__ __forceinline__ void store(unsigned char* tile, int t) const {
    if constexpr (KSTRIDED) {
      const int cc = t % G::KS_CPR, r0 = t / G::KS_CPR;
#pragma unroll
      for (int i = 0; i < G::KS_IT; i++) *(v4i*)(tile + (r0 + i * G::KS_ROWS_PER_PASS) * G::KS_STRIDE + cc * 16) = reg[i];
    } else {
      const int cc = t & 3, r0 = t >> 2;
#pragma unroll
      for (int i = 0; i < G::KC_IT; i++) *(v4i*)(tile + (r0 + i * G::KC_ROWS_PER_PASS) * G::KC_STRIDE + cc * 16) = reg[i];
    }
  }
  // MFMA operand of the 32 rows (columns) starting at `off` inside the tile, K bytes kb .. kb + 15
  static __device__ __forceinline__ v4i fragment(const unsigned char* tile, int off, int kb, int lane) {
    if constexpr (KSTRIDED) return TypeI8::read_col(tile, G::KS_STRIDE, kb, off + 16 * ((lane >> 4) & 1), lane);
    else return *(const v4i*)(tile + (off + (lane & 31)) * G::KC_STRIDE + kb);
  }
};

template <int TILE, bool TRA, bool TRB, bool ALIGNED>
__global__ void __launch_bounds__(256) gemm_i8_trans_kernel(const GemmParams p, const int tiles_m, const int tiles_n) {
  using G = TransGeometry<TILE>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int tm, tn;
  tile_coords(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
  const int m0 = tm * TILE, n0 = tn * TILE;

  TransOperand<TILE, TRA, ALIGNED> opa;    // transposed A is K-strided
  TransOperand<TILE, !TRB, ALIGNED> opb;   // plain B is K-strided
  opa.base = (const unsigned char*)p.A; opa.ld = p.lda; opa.origin = m0; opa.extent = p.M; opa.K = p.K;
  opb.base = (const unsigned char*)p.B; opb.ld = p.ldb; opb.origin = n0; opb.extent = p.N; opb.K = p.K;

  v16i acc[G::T32][G::T32];
#pragma unroll
  for (int i = 0; i < G::T32; i++)
#pragma unroll
    for (int j = 0; j < G::T32; j++) acc[i][j] = TypeI8::zero();

  auto stage_a = [&](int buf) { return smem + buf * 2 * G::OP_BYTES; };
  auto stage_b = [&](int buf) { return smem + buf * 2 * G::OP_BYTES + G::OP_BYTES; };
  const int nkt = (p.K + G::KT - 1) / G::KT;
  if (nkt > 0) {
    opa.load(0, t);
    opb.load(0, t);
    opa.store(stage_a(0), t);
    opb.store(stage_b(0), t);
  }
  __syncthreads();
  for (int kt = 0; kt < nkt; kt++) {
    const bool more = kt + 1 < nkt;
    if (more) {
      opa.load((kt + 1) * G::KT, t);
      opb.load((kt + 1) * G::KT, t);
    }
    const unsigned char* As = stage_a(kt & 1);
    const unsigned char* Bs = stage_b(kt & 1);
#pragma unroll
    for (int ks = 0; ks < G::KT / 32; ks++) {
      const int kb = ks * 32 + (lane >> 5) * 16;
      v4i af[G::T32], bf[G::T32];
#pragma unroll
      for (int i = 0; i < G::T32; i++) af[i] = decltype(opa)::fragment(As, wm * G::WT + i * 32, kb, lane);
#pragma unroll
      for (int j = 0; j < G::T32; j++) bf[j] = decltype(opb)::fragment(Bs, wn * G::WT + j * 32, kb, lane);
#pragma unroll
      for (int i = 0; i < G::T32; i++)
#pragma unroll
        for (int j = 0; j < G::T32; j++) acc[i][j] = TypeI8::mfma(bf[j], af[i], acc[i][j]);
    }
    if (more) {
      opa.store(stage_a((kt + 1) & 1), t);
      opb.store(stage_b((kt + 1) & 1), t);
    }
    __syncthreads();
  }

  // lane holds, per 32x32 tile and per q, row m and columns n .. n+3 (operands swapped as in the main kernels)
#pragma unroll
  for (int i = 0; i < G::T32; i++) {
    const int m = m0 + wm * G::WT + i * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < G::T32; j++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int n = n0 + wn * G::WT + j * 32 + 8 * q + 4 * (lane >> 5);
        int a4[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        if (ALIGNED) EpilogueI8::store4<true>(p, m, n, a4);
        else EpilogueI8::store4<false>(p, m, n, a4);
      }
  }
}

template <int TILE, bool TRA, bool TRB>
static hipError_t launch_trans(const GemmParams& p, hipStream_t stream, bool aligned) {
  using G = TransGeometry<TILE>;
  const int tiles_m = (p.M + TILE - 1) / TILE, tiles_n = (p.N + TILE - 1) / TILE;
  const dim3 grid((unsigned)(tiles_m * tiles_n));
  if (aligned) hipLaunchKernelGGL((gemm_i8_trans_kernel<TILE, TRA, TRB, true>), grid, dim3(256), G::LDS_BYTES, stream, p, tiles_m, tiles_n);
  else hipLaunchKernelGGL((gemm_i8_trans_kernel<TILE, TRA, TRB, false>), grid, dim3(256), G::LDS_BYTES, stream, p, tiles_m, tiles_n);
  return hipGetLastError();
}

template <bool TA, bool TB>
static hipError_t launch_trans_dtl(const GemmParams& p0, hipStream_t stream) {
  GemmParams p = p0;
  p.splits = 1;
  p.kt_per_split = 0;
  switch (choose_tile_i8(p.M, p.N, p.K, false)) {  // square tiles only: the 256 x 128 code falls to 128
    case 256: return launch_dtl<TypeI8, EpilogueI8, 256, 256, 2, 4, 0, 4, 64, true, TA, TB>(p, stream);
    case 192:
    case 128: return launch_dtl<TypeI8, EpilogueI8, 128, 128, 2, 4, 0, 3, 128, false, TA, TB>(p, stream);
    default: return launch_dtl<TypeI8, EpilogueI8, 64, 64, 2, 2, 0, 4, 128, false, TA, TB>(p, stream);
  }
}

// A is K x M when trans_a, B is N x K when trans_b (both row-major with their own leading dimension).
hipError_t launch_gemm_i8_trans(const GemmParams& p, bool trans_a, bool trans_b, hipStream_t stream) {
  if (!trans_a && !trans_b) return launch_gemm_i8(p, stream);
  // direct-to-LDS kernels: whole 16-byte chunks along every contiguous dimension, and row pitches that keep a lane's
  // offset from its tile's first row in 32 bits (a K-contiguous operand spans up to 320 rows, a K-strided one 128)
  const int64_t pitch_kc = std::max<int64_t>(trans_a ? 0 : p.lda, trans_b ? p.ldb : 0);
  const int64_t pitch_ks = std::max<int64_t>(trans_a ? p.lda : 0, trans_b ? 0 : p.ldb);
  const bool fast = (((uintptr_t)p.A | (uintptr_t)p.B) & 15) == 0 && p.lda % 16 == 0 && p.ldb % 16 == 0 && ((uintptr_t)p.C & 3) == 0 &&
                    p.ldc % 4 == 0 && p.K % 16 == 0 && p.N % 16 == 0 && (!trans_a || p.M % 16 == 0) && p.K > 0 &&
                    lane_offsets_fit(pitch_kc, pitch_ks);
  if (fast) {
    if (trans_a && trans_b) return launch_trans_dtl<true, true>(p, stream);
    if (trans_a) return launch_trans_dtl<true, false>(p, stream);
    return launch_trans_dtl<false, true>(p, stream);
  }
  // 16-byte vector loads and 4-byte packed stores need aligned bases and pitches
  const bool aligned = (((uintptr_t)p.A | (uintptr_t)p.B) & 15) == 0 && p.lda % 16 == 0 && p.ldb % 16 == 0 &&
                       ((uintptr_t)p.C & 3) == 0 && p.ldc % 4 == 0;
  // 128 x 128 tiles once they fill the chip, 64 x 64 otherwise
  const bool big = (int64_t)((p.M + 127) / 128) * ((p.N + 127) / 128) >= 256;
#define AC_TRANS(TRA, TRB) (big ? launch_trans<128, TRA, TRB>(p, stream, aligned) : launch_trans<64, TRA, TRB>(p, stream, aligned))
  if (trans_a && trans_b) return AC_TRANS(true, true);
  if (trans_a) return AC_TRANS(true, false);
  return AC_TRANS(false, true);
#undef AC_TRANS
}

}  // namespace ac
