// Weight-stationary int8 GEMM / implicit-GEMM convolution for gfx950: a 64-column block of B (all of K) stays
// resident in LDS for the life of a workgroup while tiles of A stream past it.
//
// The paper's best schedule for its accelerator does the same thing with the scratchpad (Appendix D.1: B
// resident, A tiles double-buffered, output stage fused into the accumulator read); here it is the shape of
// kernel that suits problems with a short K and a narrow N (the first ResNet-50 layers: K = 576, N = 64), where
// a tile-at-a-time kernel spends its time filling and draining its pipeline once per output tile and re-reads B
// for every tile.
//
// One workgroup = eight waves (two per SIMD, so one wave's output stage overlaps the other's MFMAs), laid out
// 4 x 2 over a BM x 64 tile (wave tile BM/4 x 32).  The workgroup owns column block nb and the row tiles
// wg, wg + wgs, ...; their K tiles form ONE stream of steps (tile 0: K tiles 0..nkt-1, tile 1: ...), which runs
// through a ring of LDS stages without a break at tile boundaries: while the last K tiles of one row tile are
// multiplied, the first K tiles of the next are already in flight.  Accumulators start from the bias row, and a
// row tile's output stage (shift, saturate, ReLU, pack, store) runs right after its last K step.
//
// LDS: [nkt][128 k-rows][64 B] resident B (same swizzle as a B tile of the tiled kernel), then STAGES stages of
// A [BM][128 B] (same swizzle as its A tile).  Preconditions (host): operands qualify for the direct-to-LDS
// path, bias absent or a row vector, nkt * 8 KB + ring <= 160 KB.
#pragma once
#include "gemm_dtl.hpp"

namespace ac {

template <int BM, int STAGES>
struct WstatGeometry {
  static constexpr int KTB = 128, BN = 64, WAVES = 8, WAVES_M = 4, WAVES_N = 2, THREADS = 512;
  static constexpr int A_STAGE = BM * KTB;
  static constexpr int B_TILE = KTB * BN;
  static constexpr int A_INSTR = A_STAGE / 1024 / WAVES;  // direct-to-LDS instructions per wave per step
  static constexpr int WTM = BM / WAVES_M, TM = WTM / 32;
  static constexpr int RING = STAGES * A_STAGE;
  static constexpr int MAX_KT = (160 * 1024 - RING) / B_TILE;  // K tiles of B that fit beside the ring
  static_assert(A_INSTR >= 2 && A_INSTR % 2 == 0, "the swizzle variant of a load is its index parity");
  static_assert(TM >= 1 && STAGES >= 2 && MAX_KT >= 1, "geometry");
  static_assert((STAGES - 1) * A_INSTR <= 63, "vmcnt is a 6-bit counter");
};

template <int BM, int AMODE, int STAGES>
__global__ void __launch_bounds__(512) gemm_i8_wstat_kernel(const GemmParams p, const int tiles_m, const int n_blocks) {
  using G = WstatGeometry<BM, STAGES>;
  using T = TypeI8;
  using EPI = EpilogueI8;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned lds0 = (unsigned)(uintptr_t)AC_LDS(unsigned char, smem);

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int nb = blockIdx.x % n_blocks, wg = blockIdx.x / n_blocks, wgs = gridDim.x / n_blocks;
  const int n0 = nb * G::BN;
  const int nkt = (p.K + G::KTB - 1) / G::KTB;
  const int ks_last = (p.K - (nkt - 1) * G::KTB + 31) / 32;  // MFMA K-steps that hold data in the last K tile
  const int my_tiles = wg < tiles_m ? (tiles_m - wg + wgs - 1) / wgs : 0;
  const int nsteps = my_tiles * nkt;
  if (nsteps <= 0) return;  // the same for every wave of the workgroup
  const unsigned ldsA = lds0 + nkt * G::B_TILE;
  const unsigned char* zero = (const unsigned char*)g_zero16;

  // bias of this lane's 16 columns (requested first: it is the oldest vector-memory operation of the wave)
  typename EPI::Pre pre;
  EPI::prefetch(p, n0 + wn * 32, lane, pre);

  // ---- resident B: wave w fills k-rows 16 w .. 16 w + 15 of every K tile (one instruction per K tile) ----
  {
    const int r_in = wave * 16 + (lane >> 2);  // k-row inside the K tile; the swizzle term has period 8 rows
    const int ls = BSwizzle<1, G::BN>::slot(lane & 3, r_in);
    const int colb = n0 + ls * 16;
    const unsigned char* src = (const unsigned char*)p.B + (int64_t)r_in * p.ldb + (colb < p.N ? colb : n0);
    for (int kt = 0; kt < nkt; kt++) {
      load_to_lds16(kt * G::KTB + r_in < p.K ? src : zero, lds0 + kt * G::B_TILE + wave * 1024);
      src += (int64_t)G::KTB * p.ldb;
    }
  }

  // ---- A loader: wave instruction j = wave * A_INSTR + i fills tile rows 8 j .. 8 j + 7; lane l -> row
  // 8 j + l / 8, physical slot l % 8, which holds logical chunk (l % 8) ^ ((4 (j & 1) + l / 16) & 7) --------
  int a_chunk[2];
#pragma unroll
  for (int v = 0; v < 2; v++) a_chunk[v] = (lane & 7) ^ ((4 * v + (lane >> 4)) & 7);
  int l_mt = wg, l_kt = 0, l_stage = 0;  // loader position: row tile, K tile, ring stage
  // GEMM: wave-uniform row-tile base + per-lane 32-bit offsets (rows beyond M clamped to the last row)
  const unsigned char* a_base = (const unsigned char*)p.A;
  unsigned a_voff[G::A_INSTR];
  // convolution: output pixel of each of the lane's rows, kept incrementally from one row tile to the next
  int px_ow[G::A_INSTR], px_oh[G::A_INSTR], px_img[G::A_INSTR];
  int px_base[G::A_INSTR], px_ih0[G::A_INSTR], px_iw0[G::A_INSTR];
  bool px_ok[G::A_INSTR];
  int d_ow = 0, d_oh = 0, d_img = 0;  // (image, oh, ow) step of wgs * BM rows
  int c_kh[2], c_kw[2], c_ci[2], c_off[2], c0_kh[2], c0_kw[2], c0_ci[2], c0_off[2];

  auto derive_pixels = [&](int m0) {
#pragma unroll
    for (int i = 0; i < G::A_INSTR; i++) {
      const int row = (wave * G::A_INSTR + i) * 8 + (lane >> 3);
      px_ok[i] = m0 + row < p.M;
      px_ih0[i] = px_oh[i] * p.stride - p.pad;
      px_iw0[i] = px_ow[i] * p.stride - p.pad;
      px_base[i] = ((px_img[i] * p.H + px_ih0[i]) * p.W + px_iw0[i]) * p.Cin;
    }
  };
  auto setup_rows_gemm = [&](int m0) {
    a_base = (const unsigned char*)p.A + (int64_t)m0 * p.lda;
#pragma unroll
    for (int i = 0; i < G::A_INSTR; i++) {
      const int row = (wave * G::A_INSTR + i) * 8 + (lane >> 3);
      const int rclamp = m0 + row < p.M ? row : p.M - 1 - m0;
      a_voff[i] = (unsigned)rclamp * (unsigned)p.lda + a_chunk[i & 1] * 16;
    }
  };
  if constexpr (AMODE == 0) {
    setup_rows_gemm(wg * BM);
#pragma unroll
    for (int v = 0; v < 2; v++) c_kh[v] = c_kw[v] = c_ci[v] = c_off[v] = c0_kh[v] = c0_kw[v] = c0_ci[v] = c0_off[v] = 0;
#pragma unroll
    for (int i = 0; i < G::A_INSTR; i++) px_ow[i] = px_oh[i] = px_img[i] = px_base[i] = px_ih0[i] = px_iw0[i] = 0, px_ok[i] = false;
  } else {
#pragma unroll
    for (int i = 0; i < G::A_INSTR; i++) {
      a_voff[i] = 0;
      const int m = wg * BM + (wave * G::A_INSTR + i) * 8 + (lane >> 3);
      px_ow[i] = m % p.OW;
      const int q = m / p.OW;
      px_oh[i] = q % p.OH;
      px_img[i] = q / p.OH;
    }
    derive_pixels(wg * BM);
    const int dm = wgs * BM;
    d_ow = dm % p.OW;
    d_oh = (dm / p.OW) % p.OH;
    d_img = (dm / p.OW) / p.OH;
#pragma unroll
    for (int v = 0; v < 2; v++) {  // (kh, kw, ci) of the lane's chunk in K tile 0; c_off = its element offset from the window origin
      const int kb = a_chunk[v] * 16;
      const int tap = kb / p.Cin;
      c0_ci[v] = kb - tap * p.Cin;
      c0_kh[v] = tap / p.KW;
      c0_kw[v] = tap - c0_kh[v] * p.KW;
      c0_off[v] = (c0_kh[v] * p.W + c0_kw[v]) * p.Cin + c0_ci[v];
      c_kh[v] = c0_kh[v], c_kw[v] = c0_kw[v], c_ci[v] = c0_ci[v], c_off[v] = c0_off[v];
    }
  }

  // Issues the loads of the loader's current step and moves it on by one step.  Steps are issued strictly in
  // stream order.
  auto issue_step = [&]() {
    const unsigned As = ldsA + l_stage * G::A_STAGE;
    const int kbase = l_kt * G::KTB;
    const bool full = kbase + G::KTB <= p.K;  // wave-uniform
    if (AMODE == 0 && full) {
#pragma unroll
      for (int i = 0; i < G::A_INSTR; i++) load_to_lds16_so(a_base, a_voff[i], As + (wave * G::A_INSTR + i) * 1024);
    } else {
#pragma unroll
      for (int i = 0; i < G::A_INSTR; i++) {
        const int v = i & 1;
        const int kb = kbase + a_chunk[v] * 16;
        const unsigned char* src = zero;
        if constexpr (AMODE == 0) {
          if (kb < p.K) src = a_base + a_voff[i];
        } else {
          const int ih = px_ih0[i] + c_kh[v], iw = px_iw0[i] + c_kw[v];
          if (px_ok[i] && kb < p.K && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
            src = (const unsigned char*)p.A + px_base[i] + c_off[v];
        }
        load_to_lds16(src, As + (wave * G::A_INSTR + i) * 1024);
      }
    }
    l_stage = l_stage + 1 == STAGES ? 0 : l_stage + 1;
    if (++l_kt == nkt) {  // on to the next row tile of this workgroup
      l_kt = 0;
      l_mt += wgs;
      if constexpr (AMODE == 0) {
        if (l_mt < tiles_m) setup_rows_gemm(l_mt * BM);
      } else {
#pragma unroll
        for (int i = 0; i < G::A_INSTR; i++) {
          int ow = px_ow[i] + d_ow;
          const int c1 = ow >= p.OW;
          ow -= c1 ? p.OW : 0;
          int oh = px_oh[i] + d_oh + c1;
          const int c2 = oh >= p.OH;
          oh -= c2 ? p.OH : 0;
          px_ow[i] = ow, px_oh[i] = oh, px_img[i] += d_img + c2;
        }
        derive_pixels(l_mt * BM);
#pragma unroll
        for (int v = 0; v < 2; v++) c_kh[v] = c0_kh[v], c_kw[v] = c0_kw[v], c_ci[v] = c0_ci[v], c_off[v] = c0_off[v];
      }
    } else {
      a_base += G::KTB;
      if constexpr (AMODE == 1) {  // advance the tap decode by one K tile
#pragma unroll
        for (int v = 0; v < 2; v++) {
          c_ci[v] += G::KTB;
          c_off[v] += G::KTB;
          while (c_ci[v] >= p.Cin) {
            c_ci[v] -= p.Cin;
            if (++c_kw[v] == p.KW) {
              c_kw[v] = 0;
              ++c_kh[v];
              c_off[v] += (p.W - p.KW) * p.Cin;
            }
          }
        }
      }
    }
  };

  // ---- fragments: lane's A row inside a 32-row MFMA tile is lane & 31 ------------------------------------
  struct Frag {
    v4i a[G::TM], b;
  };
  const int a_swz = ((lane & 31) >> 1) & 7;
  const int a_lane_off = (wm * G::WTM + (lane & 31)) * G::KTB;
  auto read_frags = [&](int stage, int kt, int ks, Frag& f) {
    const unsigned char* As = smem + nkt * G::B_TILE + stage * G::A_STAGE;
    const unsigned char* Bs = smem + kt * G::B_TILE;
    const int chunk = 2 * ks + (lane >> 5);
#pragma unroll
    for (int i = 0; i < G::TM; i++) f.a[i] = *(const v4i*)(As + a_lane_off + i * 32 * G::KTB + ((chunk ^ a_swz) << 4));
    f.b = dtl_read_col_i8<G::BN>(Bs, chunk * 16, wn, lane);
  };

  // ---- prologue: fill the ring ---------------------------------------------------------------------------
#pragma unroll
  for (int s = 0; s < STAGES; s++)
    if (s < nsteps) issue_step();
  if (STAGES - 1 < nsteps) wait_vm<(STAGES - 1) * G::A_INSTR>();
  else wait_vm<0>();
  block_sync();  // resident B and step 0 are visible
  Frag fr[4];
#pragma unroll
  for (int ks = 0; ks < 4; ks++) read_frags(0, 0, ks, fr[ks]);

  // accumulators start from the bias row: register 4 q + e of a tile is column 8 q + 4 (lane / 32) + e
  typename T::accv acc[G::TM];
  auto start_acc = [&]() {
#pragma unroll
    for (int i = 0; i < G::TM; i++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][r] = pre.bias[r >> 2][r & 3];
  };
  start_acc();

  // ---- the stream ----------------------------------------------------------------------------------------
  // Step g sits in stage g % STAGES; its fragments were read during step g - 1 (rolling refill: as soon as the
  // MFMAs of K-step s are issued, set s takes K-step s of the next step).  The barrier at the top of step g
  // therefore finds every wave holding step g in registers: the stage can take step g + STAGES, and step g + 1,
  // whose loads each wave has just waited for, is visible to all.
  int c_mt = wg, c_kt = 0, c_stage = 0;
  for (int g = 0; g < nsteps; g++) {
    if (g + STAGES - 1 < nsteps) wait_vm<(STAGES - 2) * G::A_INSTR>();
    else wait_vm<0>();
    block_sync();
    if (g + STAGES < nsteps) issue_step();
    const bool tile_end = c_kt == nkt - 1;
    const int nks = tile_end ? ks_last : 4;
    const int n_stage = c_stage + 1 == STAGES ? 0 : c_stage + 1;
    const int n_kt = tile_end ? 0 : c_kt + 1;
    const bool more = g + 1 < nsteps;
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {
      if (ks < nks) {
#pragma unroll
        for (int i = 0; i < G::TM; i++) acc[i] = T::mfma(fr[ks].b, fr[ks].a[i], acc[i]);
      }
      __builtin_amdgcn_sched_barrier(0);  // keep the refill behind the MFMAs that still read the old fragments
      if (more) read_frags(n_stage, n_kt, ks, fr[ks]);
    }
    if (tile_end) {
      EPI::template wave_column<true>(p, c_mt * BM + wm * G::WTM, n0 + wn * 32, acc, lane, pre);
      start_acc();
      c_mt += wgs;
    }
    c_kt = n_kt;
    c_stage = n_stage;
  }
}

template <int BM, int AMODE, int STAGES>
static hipError_t launch_wstat(const GemmParams& p, hipStream_t stream) {
  using G = WstatGeometry<BM, STAGES>;
  auto kern = gemm_i8_wstat_kernel<BM, AMODE, STAGES>;
  static std::atomic<bool> configured{false};
  if (const hipError_t e = allow_dynamic_lds_once(configured, kern, 160 * 1024)) return e;
  const int nkt = (p.K + G::KTB - 1) / G::KTB;
  if (nkt < 1 || nkt > G::MAX_KT) return hipErrorInvalidValue;
  const int cus = compute_units();
  const int tiles_m = (p.M + BM - 1) / BM, n_blocks = (p.N + G::BN - 1) / G::BN;
  // one workgroup per compute unit (its LDS holds B and the ring); every column block gets the same number
  int wgs = cus / n_blocks;
  if (wgs < 1) wgs = 1;
  if (wgs > tiles_m) wgs = tiles_m;
  const size_t lds = (size_t)nkt * G::B_TILE + G::RING;
  hipLaunchKernelGGL(kern, dim3((unsigned)(wgs * n_blocks)), dim3(G::THREADS), lds, stream, p, tiles_m, n_blocks);
  return hipGetLastError();
}

// Tile codes of the weight-stationary kernel: 320 = 256-row tiles, 160 = 128-row tiles (both 64 columns wide).
static inline bool wstat_tile_rows(int tile, int* bm) {
  if (tile == 320) return *bm = 256, true;
  if (tile == 160) return *bm = 128, true;
  return false;
}
// K tiles (128 bytes of K) the kernel behind a tile code can hold resident, with its deepest ring that fits.
static inline int wstat_max_kt(int tile) { return tile == 320 ? WstatGeometry<256, 2>::MAX_KT : WstatGeometry<128, 2>::MAX_KT; }

template <int AMODE>
static hipError_t launch_wstat_tile(int tile, const GemmParams& p, hipStream_t stream) {
  const int nkt = (p.K + 127) / 128;
  if (tile == 320) {
    if (nkt <= WstatGeometry<256, 3>::MAX_KT) return launch_wstat<256, AMODE, 3>(p, stream);
    return launch_wstat<256, AMODE, 2>(p, stream);
  }
  if (nkt <= WstatGeometry<128, 4>::MAX_KT) return launch_wstat<128, AMODE, 4>(p, stream);
  return launch_wstat<128, AMODE, 2>(p, stream);
}

}  // namespace ac
