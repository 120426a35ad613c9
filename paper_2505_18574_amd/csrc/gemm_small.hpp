// int8 GEMM and convolution for launches that last a few microseconds (the accelerator-sized layers of Sections
// 4.4.1 and 4.4.2): one wave per 32 x 32 output tile, one to four independent waves per workgroup.
//
// At that size a launch is a chain of latencies, not of throughput: a workgroup of the tiled kernels spends
// about 1.3 us in some 500 instructions of addressing before its first operand arrives (a wave issues one
// instruction every 4-5 cycles), 0.5 us in a K loop with two barriers per tile and 0.7 us in the output stage.
// Here a wave owns its tile alone, so there is no barrier anywhere and no tile-order, K-slice or persistence
// logic ahead of the first load; the operands stream through a ring of private LDS stages (64 or 128 bytes of K
// each) and the fragments of the next K tile are read while the MFMAs of the current one run.
//
// The ring bounds the waves a compute unit holds (160 KB of LDS), and the workgroup size decides over how many
// compute units a small grid spreads, so the launcher picks among a few (stage width, stages, waves per workgroup)
// combinations by K and tile count; see launch_small_i8.
//
// Operands as for the direct-to-LDS kernels (16-byte aligned, K and N in whole 16-byte chunks), and K a multiple
// of 64; anything else stays on the tiled kernels.
#pragma once
#include "gemm_dtl.hpp"

namespace ac {

constexpr int SMALL_KTB = 64;  // K bytes per stage at least; 128 where K is a multiple of that (half the bookkeeping per byte)

// KTB: bytes of K per stage, S: stages of a wave's ring, SMALL_WAVES: independent waves (tiles) per workgroup,
// AMODE 0: A is the M x K matrix; 1: A is gathered from the NHWC input of a convolution (the per-lane window
// origin and one validity bit per kernel tap of gemm_dtl_kernel; a chunk outside the image gets the offset
// 0xffffffff and the bounds check of the buffer load writes its zeros).  SPLIT: a wave owns (tile, K slice): slice s
// covers K tiles s * kt_per_split ... and leaves its int32 sums in p.partial[s][M][N] for splitk_reduce_i8_kernel
// (with few tiles and a deep K, slices are what puts enough loads in flight; ntiles then counts tiles, not items).
template <int KTB, int S, int SMALL_WAVES, int AMODE, bool SPLIT>
__global__ void __launch_bounds__(64 * SMALL_WAVES) gemm_i8_small_kernel(const GemmParams p, const int tiles_n, const int ntiles, const unsigned tn_magic) {
  using T = TypeI8;
  using EPI = EpilogueI8;
  using G = DtlGeometry<T, 32, 32, 1, 1, S, KTB>;
  constexpr int NA = G::A_INSTR, NB = G::B_INSTR, KS = G::KSTEPS;
  static_assert(NA == KTB / 32 && NB == KTB / 32 && KS == KTB / 32 && G::TM == 1 && G::TN == 1 && G::STAGE == 64 * KTB && S >= 3, "geometry");
  constexpr int PER_TILE = NA + NB;
  static_assert((S - 1) * PER_TILE <= 63, "vmcnt is a 6-bit counter");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int item = blockIdx.x * SMALL_WAVES + wave;
  if (item >= (SPLIT ? ntiles * p.splits : ntiles)) return;  // whole waves leave; no wave of this kernel ever waits for another
  const int split = SPLIT ? item / ntiles : 0;
  const int tile = item - split * ntiles;
  const int kt0 = split * p.kt_per_split;  // first K tile of this slice
  const int tm = tn_magic ? (int)__umulhi((unsigned)tile, tn_magic) : tile / tiles_n;
  const int tn = tile - tm * tiles_n;
  const int m0 = tm * 32, n0 = tn * 32;
  unsigned char* win = smem + wave * (S * G::STAGE);
  const unsigned lds0 = (unsigned)(uintptr_t)AC_LDS(unsigned char, win);

  // source offsets of the loads of a K tile (same lane roles as gemm_dtl_kernel, with one wave)
  constexpr int NVAR = KTB == 128 ? 2 : 1;  // distinct swizzle terms of a lane over the A instructions
  unsigned a_voff[NA], b_voff[NB];
  int g_base[NA];
  unsigned g_mask[NA], g_kb[NVAR];
  v4i a_rsrc = {0, 0, 0, 0};
  if constexpr (AMODE == 1) {
    const uint64_t ab = (uint64_t)(uintptr_t)p.A;
    a_rsrc[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)ab);
    a_rsrc[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(ab >> 32));
    a_rsrc[2] = __builtin_amdgcn_readfirstlane(p.a_bytes);
    a_rsrc[3] = 0x00020000;
  }
#pragma unroll
  for (int i = 0; i < NA; i++) {
    const int row = i * G::A_ROWS_PER_INSTR + lane / G::A_SPR;
    const int a_chunk = (lane % G::A_SPR) ^ G::a_xor(row);
    g_base[i] = 0, g_mask[i] = 0u, a_voff[i] = 0u;
    if constexpr (AMODE == 0) {
      const int rclamp = m0 + row < p.M ? row : p.M - 1 - m0;
      a_voff[i] = (unsigned)rclamp * (unsigned)p.lda + a_chunk * 16;
    } else {
      if (i < NVAR) g_kb[i] = (unsigned)(kt0 * KTB + a_chunk * 16);  // a_xor(row) repeats with period NVAR over the instructions
      const int m = m0 + row;
      const unsigned mm = m < p.M ? (unsigned)m : 0u;
      const unsigned q = p.dOW.div(mm), img = p.dOH.div(q);
      const int ow = (int)(mm - q * p.OW), oh = (int)(q - img * p.OH);
      const int ih0 = oh * p.stride - p.pad, iw0 = ow * p.stride - p.pad;
      g_base[i] = (((int)img * p.H + ih0) * p.W + iw0) * p.Cin;
      auto span = [](int first, int n, int extent) {  // bits k = 0 .. n-1 with 0 <= first + k < extent
        const int lo = first < 0 ? -first : 0, hi = extent - first < n ? extent - first : n;
        if (hi <= lo) return 0u;
        return (hi >= 32 ? ~0u : (1u << hi) - 1u) & ~((1u << lo) - 1u);
      };
      const unsigned rows = span(ih0, p.KH, p.H), cols = span(iw0, p.KW, p.W);
      unsigned mask = 0u;
      for (int kh = 0; kh < p.KH; kh++)
        if ((rows >> kh) & 1u) mask |= cols << (kh * p.KW);
      g_mask[i] = m < p.M ? mask : 0u;
    }
    const int brow = i * G::B_ROWS_PER_INSTR + lane / G::B_SPR;
    const int slot = lane % G::B_SPR;
    b_voff[i] = (unsigned)brow * (unsigned)p.ldb + (n0 + slot * 16 < p.N ? slot * 16 : 0);
  }
  const int64_t b_step = (int64_t)G::BK * p.ldb;
  const unsigned char* a_base = (const unsigned char*)p.A + (AMODE == 0 ? (int64_t)m0 * p.lda : 0) + (int64_t)kt0 * KTB;
  const unsigned char* b_base = (const unsigned char*)p.B + n0 + kt0 * b_step;
  const int nkt_total = p.K / KTB;
  const int nkt = SPLIT ? (nkt_total - kt0 < p.kt_per_split ? nkt_total - kt0 : p.kt_per_split) : nkt_total;

  // the bias row is requested ahead of the operand loads, so that the counted waits on those see nothing else
  EPI::Pre pre;
  if constexpr (!SPLIT) EPI::prefetch(p, n0, lane, pre);

  int wr = 0;  // stage that the next requested tile goes to
  auto issue = [&]() {
    const unsigned st = lds0 + wr * G::STAGE;
    if constexpr (AMODE == 1) {
      // the lane's chunk sits at K byte g_kb: tap g_kb / Cin, channel g_kb % Cin (K is in whole stages: never beyond K)
      unsigned g_off[NVAR], g_tap[NVAR];
#pragma unroll
      for (int v = 0; v < NVAR; v++) {
        const unsigned tap = p.dCin.div(g_kb[v]), ci = g_kb[v] - tap * p.Cin;
        const unsigned kh = p.dKW.div(tap), kw = tap - kh * p.KW;
        g_off[v] = (kh * p.W + kw) * p.Cin + ci;
        g_tap[v] = tap;
        g_kb[v] += KTB;
      }
#pragma unroll
      for (int i = 0; i < NA; i++) {
        const unsigned inside = (g_mask[i] >> (g_tap[i & (NVAR - 1)] & 31u)) & 1u;
        buffer_to_lds16(a_rsrc, ((unsigned)g_base[i] + g_off[i & (NVAR - 1)]) | (inside - 1u), st + i * 1024);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NA; i++) load_to_lds16_so(a_base, a_voff[i], st + i * 1024);
    }
#pragma unroll
    for (int i = 0; i < NB; i++) load_to_lds16_so(b_base, b_voff[i], st + G::A_BYTES + i * 1024);
    a_base += KTB;
    b_base += b_step;
    wr = wr + 1 == S ? 0 : wr + 1;
  };
#pragma unroll
  for (int s = 0; s < S - 1; s++)
    if (s < nkt) issue();

  // fragment addresses: the lane's A row is lane & 31, its 16 K-bytes of K-step ks sit in chunk 2 ks + lane / 32
  const int a_swz = G::a_xor(lane & 31);
  int a_fo[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) a_fo[ks] = (lane & 31) * G::KTB + (((2 * ks + (lane >> 5)) ^ a_swz) << 4);
  const int b_fo = G::A_BYTES + dtl_col_off<T, G::B_ROW>((lane >> 5) * 16, 0, lane);
  constexpr int KS_B = 32 * G::B_ROW;  // bytes between the B rows of consecutive K-steps

  struct Frag {
    v4i a[KS], b[KS];
  };
  int rd = 0;  // stage of the next tile to be read
  auto read_frags = [&](Frag& f) {
    const unsigned char* st = win + rd * G::STAGE;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      f.a[ks] = *(const v4i*)(st + a_fo[ks]);
      f.b[ks] = dtl_read_col_at<T, G::B_ROW>(st + b_fo + ks * KS_B);
    }
    rd = rd + 1 == S ? 0 : rd + 1;
  };

  typename T::accv acc = T::zero();
  Frag f[2];
  if (nkt > 0) {
    if (S - 1 <= nkt) wait_vm<(S - 2) * PER_TILE>();
    else wait_vm<0>();
    read_frags(f[0]);
  }
  // Tile kt: request tile kt + S - 1 into the stage tile kt - 1 has left (its fragments were waited for before its
  // MFMAs), wait for this wave's loads of tile kt + 1, read its fragments, then the MFMAs of tile kt.
  auto step = [&](int kt, Frag& cur, Frag& nxt) {
    if (kt + 1 < nkt) {
      if (kt + S - 1 < nkt) {
        issue();
        wait_vm<(S - 2) * PER_TILE>();
      } else {
        wait_vm<0>();  // the last S - 2 tiles: everything that is still in flight
      }
      read_frags(nxt);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ks++) acc = T::mfma(cur.b[ks], cur.a[ks], acc);  // EPI::SWAP operand order
  };
  int kt = 0;
  for (; kt + 1 < nkt; kt += 2) {
    step(kt, f[0], f[1]);
    step(kt + 1, f[1], f[0]);
  }
  if (kt < nkt) step(kt, f[0], f[1]);

  if constexpr (SPLIT) {
    // With the swapped operand order, registers 4 g .. 4 g + 3 of a lane are columns 8 g + 4 (lane / 32) + 0 .. 3 of
    // row lane % 32: one 16-byte store each (N is a multiple of 16 on this path: a group of four is inside or outside).
    const int m = m0 + (lane & 31);
    int32_t* row = p.partial + ((int64_t)split * p.M + m) * p.N;
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const int n = n0 + 8 * g + 4 * (lane >> 5);
      if (m < p.M && n < p.N) *(v4i*)(row + n) = v4i{acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
    }
  } else {
    EPI::tile(p, m0, n0, acc, lane, 0, pre);
  }
}

// Whether the small kernel can run p (a GEMM or a convolution on direct-to-LDS operands, see gemm_i8_fast_path and
// conv_i8_fast_path, checked by the caller).
static inline bool small_i8_eligible(const GemmParams& p) {
  const int64_t tiles = (int64_t)((p.M + 31) / 32) * ((p.N + 31) / 32);
  return p.K >= SMALL_KTB && p.K % SMALL_KTB == 0 && tiles * (p.splits > 1 ? p.splits : 1) <= INT32_MAX;
}

template <int KTB, int S, int SMALL_WAVES, int AMODE, bool SPLIT = false>
static hipError_t launch_small_i8_cfg(const GemmParams& p, hipStream_t stream) {
  constexpr int LDS = SMALL_WAVES * S * 64 * KTB;
  static std::atomic<bool> configured{false};
  if (const hipError_t e = allow_dynamic_lds_once(configured, gemm_i8_small_kernel<KTB, S, SMALL_WAVES, AMODE, SPLIT>, LDS)) return e;
  const int tiles_m = (p.M + 31) / 32, tiles_n = (p.N + 31) / 32;
  const int ntiles = tiles_m * tiles_n;
  const unsigned tn_magic = (uint64_t)ntiles * (unsigned)tiles_n < (1ull << 32) ? FastDiv::make((unsigned)tiles_n).magic : 0u;
  const int64_t items = (int64_t)ntiles * (SPLIT ? p.splits : 1);
  hipLaunchKernelGGL((gemm_i8_small_kernel<KTB, S, SMALL_WAVES, AMODE, SPLIT>), dim3((unsigned)((items + SMALL_WAVES - 1) / SMALL_WAVES)), dim3(64 * SMALL_WAVES), LDS, stream, p,
                     tiles_n, ntiles, tn_magic);
  return hipGetLastError();
}

// Measured (us, warm, per launch; four waves per workgroup over 24 KB rings first, then the choice below):
// 256^3 3.32 -> 2.92, 3136x64x576 3.83 -> 3.48, 512x768x768 4.63 -> 3.86, 128x1024x1024 5.20 -> 3.94,
// 6272x256x64 4.36 -> 3.36.  With 24 KB per wave and four waves a compute unit holds one
// workgroup, four waves; smaller workgroups pack six waves, and up to 256 one-wave workgroups land on compute
// units of their own.  One or two K tiles per wave need no deep ring: 12 KB rings and four waves per workgroup
// (twelve waves per compute unit, a quarter of the workgroups to launch).  Deeper rings (up to eight stages), and
// a tile order that keeps an XCD's tiles in one block of the output so that its L2 fetches less of A and B, were
// measured too, with operands in the caches and in HBM: no gain on any shape the planner sends here.
template <int AMODE>
static hipError_t launch_small_i8(const GemmParams& p, hipStream_t stream) {
  // K slices (64-byte K tiles, as the plan counts them): the caller launches the kernel that sums them
  if (p.splits > 1) return launch_small_i8_cfg<64, 4, 2, AMODE, true>(p, stream);
  const int64_t ntiles = (int64_t)((p.M + 31) / 32) * ((p.N + 31) / 32);
  if (p.K <= 128) return launch_small_i8_cfg<64, 3, 4, AMODE>(p, stream);
  // 16 KB rings in pairs: ten waves per compute unit, 2560 tiles at once (the 24 KB rings hold 1536)
  if (p.K % 128 != 0 || ntiles > 1536) return launch_small_i8_cfg<64, 4, 2, AMODE>(p, stream);
  return ntiles <= 256 ? launch_small_i8_cfg<128, 3, 1, AMODE>(p, stream) : launch_small_i8_cfg<128, 3, 2, AMODE>(p, stream);
}

}  // namespace ac
