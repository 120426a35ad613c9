// int8 convolution for gfx950 that keeps BOTH operands of its implicit GEMM on chip: a 64-column block of the
// weights (all of K) is resident in LDS, and the input enters LDS as the image patch that a block of output
// pixels needs (rows with their halo), once, instead of as im2col rows in which every input pixel appears
// KH * KW times.
//
// Why: with 64 output channels the im2col stream through the vector L1 (64 B / clock / CU) costs as many cycles
// as the MFMAs themselves, and building one gather address per 16 bytes costs more vector-ALU time than that.
// A patch is a handful of contiguous row segments: a fifth of the bytes (3 x 3, stride 1), one address per
// kilobyte, and -- since the whole patch of a unit is on chip before its first MFMA -- no barrier inside the K
// loop.  (The paper's best schedules get their speed the same way: operands resident in the scratchpad,
// Appendix D.1.)
//
// Work unit: BM consecutive output pixels (row-major over oh, ow) of one image, times one 64-column block.
// Eight waves, 4 x 2 over the BM x 64 tile.  A wave always works on the same 32 columns, so for the usual K
// depths (template parameter NKS = K / 32) it keeps its weight fragments for ALL of K in registers, read from
// LDS once: the K loop then reads only the A fragments, which halves the LDS traffic per MFMA.
// The two waves of a SIMD belong to two groups that run half a unit apart (group 1 does the output stage of
// unit t - 1 while group 0 multiplies unit t, then the roles swap), so the vector-ALU work of the output stage
// runs under the other group's MFMAs.
//
// LDS: [nkt][128][64 B] weights (B-tile swizzle of the tiled kernels) | patch buffer 0 | patch buffer 1.
// Patch layout: pixel P = ihl * ROWP + (iwl % stride) * WQ + iwl / stride, where (ihl, iwl) counts from the
// top-left corner of the patch including padding, WQ = ceil(WP / stride), ROWP = stride * WQ; a pixel takes
// Cin + 16 bytes (the odd number of 16-byte slots makes the A-fragment reads of 16 consecutive pixels
// conflict-free).  For output pixel (ohl, ow) of the unit and tap (kh, kw) the input pixel is
//   P = [ohl * stride * ROWP + ow] + [kh * ROWP + (kw % stride) * WQ + kw / stride],
// a per-lane term plus a wave-uniform term: the K loop adds one scalar to a fixed per-lane address.
// Preconditions (host, conv_halo_plan): direct-to-LDS operands, Cin a multiple of 32, LDS budget.
#pragma once
#include "gemm_dtl.hpp"

namespace ac {

// A pointer the compiler must keep in scalar registers (it is the same in every lane by construction).
static __device__ __forceinline__ const unsigned char* uniform_ptr(const unsigned char* q) {
  const uint64_t v = (uint64_t)(uintptr_t)q;
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v), hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
  return (const unsigned char*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

struct ConvHaloParams {
  int32_t KH, WQ, ROWP, SP, PITCH;  // kernel rows; patch geometry (pixels per plane row / per patch row; 16-byte slots and bytes per pixel)
  int32_t HB;                       // bytes of one patch buffer (whole kilobytes)
  int32_t U;                        // units per image
  int32_t units;                    // Nb * U
  int32_t nks;                      // MFMA K-steps (32 bytes of K each) = K / 32, at most 64
  int32_t PPI, CPR;                 // pixels per patch-load instruction (64 / SP); instructions per patch row
  int32_t RIN;                      // patch rows a buffer holds
  int32_t NPAD_R;                   // padding columns to the right of the image that the patch includes
  FastDiv dWQ, dOW, dU, dPADC, dCC, dS, dCIN, dKW;  // dPADC: padding slots per patch row; dCC: data slots per pixel
};

// TM 32 x 32 accumulator tiles, 32 rows apart (sums already include the bias) -> int8 outputs of rows m < m_end.
// Register 4 q + e of lane l is row l % 32, column 8 q + 4 (l / 32) + e of a tile.  What the tiles have in common
// (whole 32-column block or its 16-column remainder, which rounding) is decided once for all of them.
template <int TM, class ACC>
static __device__ __forceinline__ void halo_store_tiles(const GemmParams& p, int m0, int m_end, int ncol0, const ACC (&acc)[TM], int lane) {
  using EPI = EpilogueI8;
  if (ncol0 >= p.N) return;  // wave-uniform
  int8_t* C = (int8_t*)p.C;
  if (ncol0 + 32 <= p.N) {
    auto blocks = [&](auto quant) {
#pragma unroll
      for (int i = 0; i < TM; i++) {
        const int m = m0 + 32 * i;
        int t[16];
#pragma unroll
        for (int r = 0; r < 16; r++) t[r] = acc[i][r];
        const v4i o = quant(t);
        if (m < m_end) *(v4i*)(C + (int64_t)m * p.ldc + ncol0 + 16 * (lane >> 5)) = o;
      }
    };
    if (p.shift >= 1 && p.shift <= 23) {
      const EPI::FastQuant f = EPI::fast_quant(p.shift, p.act);
      if (p.shift <= 17) blocks([&](const int* t) { return EPI::quant16<true>(t, f); });
      else blocks([&](const int* t) { return EPI::quant16<false>(t, f); });
    } else {
      blocks([&](const int* t) { return EPI::quant16(t, p.shift, p.act); });
    }
  } else {  // the 16-column remainder of the last block
#pragma unroll
    for (int i = 0; i < TM; i++) {
      const int m = m0 + 32 * i;
      if (m >= m_end) continue;
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int n = ncol0 + 8 * q + 4 * (lane >> 5);
        if (n + 3 < p.N) {
          int v[4];
#pragma unroll
          for (int e = 0; e < 4; e++) v[e] = EPI::requant(acc[i][4 * q + e], p.shift, p.act);
          *(unsigned*)(C + (int64_t)m * p.ldc + n) = EPI::pack4(v[0], v[1], v[2], v[3]);
        }
      }
    }
  }
}

template <int BM, int NKS>
__global__ void __launch_bounds__(512) conv_i8_halo_kernel(const GemmParams p, const ConvHaloParams h, const int n_blocks) {
  using T = TypeI8;
  using EPI = EpilogueI8;
  constexpr int WTM = BM / 4, TM = WTM / 32, B_TILE = 128 * 64;
  constexpr int NB = NKS > 0 ? NKS : 1;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned lds0 = (unsigned)(uintptr_t)AC_LDS(unsigned char, smem);

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int grp = wave >> 2, wm = wave & 3, wn = grp;  // waves w and w + 4 share a SIMD: one of each group
  const int nb = blockIdx.x % n_blocks, wg = blockIdx.x / n_blocks, wgs = gridDim.x / n_blocks;
  const int n0 = nb * 64;
  const int nkt = (p.K + 127) / 128;
  const int my_units = wg < h.units ? (h.units - wg + wgs - 1) / wgs : 0;
  if (my_units <= 0) return;  // the same for every wave of the workgroup
  const unsigned ldsP = lds0 + nkt * B_TILE;  // patch buffers
  const unsigned char* zero = (const unsigned char*)g_zero16;
  const int npix = p.OH * p.OW;  // output pixels per image
  const int nks = NKS > 0 ? NKS : h.nks;

  typename EPI::Pre pre;
  EPI::prefetch(p, n0 + wn * 32, lane, pre);

  // ---- weights -> LDS: wave w fills k-rows 16 w .. 16 w + 15 of every K tile -----------------------------
  {
    const int r_in = wave * 16 + (lane >> 2);
    const int ls = BSwizzle<1, 64>::slot(lane & 3, r_in);
    const int colb = n0 + ls * 16;
    const unsigned char* src = (const unsigned char*)p.B + (int64_t)r_in * p.ldb + (colb < p.N ? colb : n0);
    for (int kt = 0; kt < nkt; kt++) {
      load_to_lds16(kt * 128 + r_in < p.K ? src : zero, lds0 + kt * B_TILE + wave * 1024);
      src += (int64_t)128 * p.ldb;
    }
  }

  // first output row and patch rows of unit u (u counts over images and their units)
  struct Unit {
    int img, q0, oh_first, rin;
  };
  auto unit_of = [&](int u) {
    Unit w;
    w.img = (int)h.dU.div((unsigned)u);
    w.q0 = (u - w.img * h.U) * BM;
    w.oh_first = (int)h.dOW.div((unsigned)w.q0);
    const int qlast = w.q0 + BM - 1 < npix ? w.q0 + BM - 1 : npix - 1;
    w.rin = ((int)h.dOW.div((unsigned)qlast) - w.oh_first) * p.stride + h.KH;
    return w;
  };

  // Patch of unit `w` -> buffer `buf`.  A wave takes whole patch rows (row r -> wave r % 8), one instruction per
  // run of PPI pixels: per row only the wave-uniform row base changes (a row outside the image is fetched from the
  // block of zeros, offset 0 for every lane), and from one run to the next a lane's image column and byte offset
  // advance by constants.  Lanes that hold a pad slot, lie beyond the run or the row, or fall on a padding column
  // are switched off; the padding columns are cleared once, below, and nothing else ever writes them.
  const int lane_px = lane / h.SP, lane_part = lane - lane_px * h.SP;
  const bool lane_on = lane_px < h.PPI && lane_part < h.SP - 1;
  {  // one thread per 16-byte slot of a padding column (both buffers, every row): image columns -pad .. -1 and W ..
    const int npad_l = p.pad, npad = npad_l + h.NPAD_R, cc = h.SP - 1;
    for (int z = t; z < 2 * h.RIN * npad * cc; z += 512) {
      const int rowz = (int)h.dPADC.div((unsigned)z), rem = z - rowz * npad * cc;
      const int idx = (int)h.dCC.div((unsigned)rem), part = rem - idx * cc;
      const int iwl = idx < npad_l ? idx : p.W + idx;  // patch column, counted from image column -pad
      const int q = (int)h.dS.div((unsigned)iwl), pp = (iwl - q * p.stride) * h.WQ + q;
      const int bz = rowz >= h.RIN, row = rowz - bz * h.RIN;
      *(v4i*)(smem + nkt * B_TILE + bz * h.HB + ((row * h.ROWP + pp) * h.PITCH + part * 16)) = (v4i){0, 0, 0, 0};
    }
  }
  // stride 1: image column and byte offset of the lane in run 0; a lane that is off gets a column no test passes
  const int iw_run0 = lane_on ? lane_px - p.pad : 0x40000000;
  const int off_run0 = (lane_px - p.pad) * p.Cin + lane_part * 16;
  const int iw_lim = p.W < h.ROWP - p.pad ? p.W : h.ROWP - p.pad;  // columns of this row that exist in the image
  // Stride 1 with at most MAXC runs per patch row: which lanes load in run c, and from which byte of the row, is
  // the same for every row of every unit, so both are kept (a lane mask and an offset per run) and a row is MAXC
  // predicated loads in a straight line.  As a loop over the runs with the tests inside, a row cost some hundred
  // instructions and a dozen taken branches for its five loads.
  constexpr int MAXC = 6;
  const bool short_rows = p.stride == 1 && h.CPR <= MAXC;  // wave-uniform
  unsigned run_off[MAXC];
  bool run_on[MAXC];
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    run_on[c] = short_rows && c < h.CPR && (unsigned)(iw_run0 + c * h.PPI) < (unsigned)iw_lim;
    run_off[c] = (unsigned)(off_run0 + c * h.PPI * p.Cin);
  }
  auto issue_patch = [&](const Unit& w, int buf, int row_first, int row_step) {
    const int ih_base = w.oh_first * p.stride - p.pad;
    const unsigned char* img_base = (const unsigned char*)p.A + (int64_t)w.img * p.H * p.W * p.Cin;
    for (int row = row_first; row < w.rin; row += row_step) {
      const int ih = ih_base + row;
      const bool row_ok = (unsigned)ih < (unsigned)p.H;
      const unsigned char* sbase = uniform_ptr(row_ok ? img_base + (int64_t)ih * p.W * p.Cin : zero);
      unsigned dst = ldsP + buf * h.HB + row * h.ROWP * h.PITCH;
      if (short_rows) {
        const unsigned keep = row_ok ? ~0u : 0u;  // a row outside the image: every lane reads the block of zeros at offset 0
#pragma unroll
        for (int c = 0; c < MAXC; c++)
          if (run_on[c]) load_to_lds16_so(sbase, run_off[c] & keep, (unsigned)__builtin_amdgcn_readfirstlane((int)(dst + c * h.PPI * h.PITCH)));
      } else if (p.stride == 1) {
        int iw = iw_run0, off = off_run0;
        for (int c = 0; c < h.CPR; c++) {
          if ((unsigned)iw < (unsigned)iw_lim) load_to_lds16_so(sbase, row_ok ? (unsigned)off : 0u, (unsigned)__builtin_amdgcn_readfirstlane((int)dst));
          iw += h.PPI, off += h.PPI * p.Cin, dst += h.PPI * h.PITCH;
        }
      } else {
        for (int c = 0; c < h.CPR; c++) {
          const int pp = c * h.PPI + lane_px;  // position in the patch row, plane-major
          const int plane = (int)h.dWQ.div((unsigned)pp);
          const int iw = (pp - plane * h.WQ) * p.stride + plane - p.pad;
          if (lane_on && pp < h.ROWP && (unsigned)iw < (unsigned)p.W)
            load_to_lds16_so(sbase, row_ok ? (unsigned)(iw * p.Cin + lane_part * 16) : 0u, (unsigned)__builtin_amdgcn_readfirstlane((int)dst));
          dst += h.PPI * h.PITCH;
        }
      }
    }
  };

  // Patch offset of K-step k (32 bytes of K: tap (kh, kw), byte cib inside the tap):
  // (kh * ROWP + (kw % stride) * WQ + kw / stride) * PITCH + cib.
  auto tap_offset = [&](int k) {
    const int kbyte = k * 32;
    const int tap = (int)h.dCIN.div((unsigned)kbyte), cib = kbyte - tap * p.Cin;
    const int kh = (int)h.dKW.div((unsigned)tap), kw = tap - kh * p.KW;
    const int kwq = (int)h.dS.div((unsigned)kw), kwr = kw - kwq * p.stride;
    return (kh * h.ROWP + kwr * h.WQ + kwq) * h.PITCH + cib;
  };
  const int tap_tbl = tap_offset(lane < nks ? lane : 0);  // lane k: K-step k (the K loop of unknown depth reads it with v_readlane)

  // B fragment of K-step k: k-rows 32 k + 16 (lane / 32) + ..., whose swizzle term does not depend on k
  const int b_off0 = [&]() {
    const int i = lane & 15, g1 = (lane >> 4) & 1;
    const int r = (lane >> 5) * 16 + (i >> 1);
    return r * 64 + ((wn ^ BSwizzle<1, 64>::seg_xor(r)) << 5) + g1 * 16 + 8 * (i & 1);
  }();
  auto read_b = [&](int k) {
    const unsigned char* bp = smem + b_off0 + k * 2048;
    const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32(AC_LDS(v2i, bp));
    const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32(AC_LDS(v2i, bp + 8 * 64));
    return (v4i){lo[0], lo[1], hi[0], hi[1]};
  };

  int a_addr[TM];  // LDS offset of the lane's output pixel in the current patch buffer, per 32-row MFMA tile
  struct FragA {
    v4i a[TM];
  };
  int tap_v[NB];  // NKS > 0: the tap offsets, one register each (the same value in every lane)
  if constexpr (NKS > 0) {
#pragma unroll
    for (int k = 0; k < NKS; k++) tap_v[k] = tap_offset(k);
  }
  auto read_a = [&](int k, FragA& f) {  // k wave-uniform, < nks (a compile-time constant when NKS > 0)
    int so;
    if constexpr (NKS > 0) so = tap_v[k];
    else so = __builtin_amdgcn_readlane(tap_tbl, k);
#pragma unroll
    for (int i = 0; i < TM; i++) f.a[i] = *(const v4i*)(smem + (a_addr[i] + so));
  };

  typename T::accv acc[TM], bias_acc;  // register 4 q + e of a tile is column 8 q + 4 (lane / 32) + e: bias_acc is the bias row in that order
#pragma unroll
  for (int r = 0; r < 16; r++) bias_acc[r] = pre.bias[r >> 2][r & 3];

  // The K loop of unit w on patch buffer buf.  A fragments: four sets in rotation, three K-steps read ahead (a
  // wave has only TM MFMAs per K-step, far less than the latency of an LDS read).
  v4i bw[NB];  // NKS > 0: this wave's weight fragments of every K-step
  auto multiply = [&](const Unit& w, int buf) {
#pragma unroll
    for (int i = 0; i < TM; i++) {
      int q = w.q0 + wm * WTM + i * 32 + (lane & 31);
      q = q < npix ? q : npix - 1;  // rows past the image end compute on a valid pixel and are never stored
      const int oh = (int)h.dOW.div((unsigned)q), ow = q - oh * p.OW;
      a_addr[i] = ((oh - w.oh_first) * p.stride * h.ROWP + ow) * h.PITCH + (lane >> 5) * 16 + nkt * B_TILE + buf * h.HB;
    }
    const int last = nks - 1;
    FragA f[4];
#pragma unroll
    for (int j = 0; j < 3; j++) read_a(j < last ? j : last, f[j]);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (NKS > 0) {
#pragma unroll
      for (int k = 0; k < NKS; k++) {
        if (k + 3 < NKS) read_a(k + 3, f[(k + 3) & 3]);
        __builtin_amdgcn_sched_barrier(0);  // the read-ahead stays ahead: the scheduler would sink each read to its use
#pragma unroll
        for (int i = 0; i < TM; i++) acc[i] = T::mfma(bw[k], f[k & 3].a[i], k == 0 ? bias_acc : acc[i]);  // sums start from the bias row
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < TM; i++) acc[i] = bias_acc;
      v4i fb[4];
#pragma unroll
      for (int j = 0; j < 3; j++) fb[j] = read_b(j < last ? j : last);
      int k = 0;
      for (; k + 7 <= nks; k += 4) {  // steps k .. k + 3 multiply while steps k + 3 .. k + 6 are read: all exist
#pragma unroll
        for (int j = 0; j < 4; j++) {
          read_a(k + j + 3, f[(j + 3) & 3]);
          fb[(j + 3) & 3] = read_b(k + j + 3);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < TM; i++) acc[i] = T::mfma(fb[j], f[j].a[i], acc[i]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      for (; k < nks; k += 4) {  // the last few steps: reads past the end repeat the last step and are not used
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const int kk = k + j + 3 < last ? k + j + 3 : last;
          read_a(kk, f[(j + 3) & 3]);
          fb[(j + 3) & 3] = read_b(kk);
          __builtin_amdgcn_sched_barrier(0);
          if (k + j < nks) {
#pragma unroll
            for (int i = 0; i < TM; i++) acc[i] = T::mfma(fb[j], f[j].a[i], acc[i]);
          }
        }
      }
    }
  };

  // ---- units, in half steps ------------------------------------------------------------------------------
  // Group g multiplies unit t in half step 2 t + g and runs its output stage in half step 2 t + g + 1; a barrier
  // follows every odd half step.  The patch of unit t + 1 is requested ahead of the output stages: by group 1 at
  // the start of half step 2 t and by group 0 at the start of half step 2 t + 1, each wave its own rows, so that
  // the request runs beside the other group's MFMAs (requested by all eight waves at once it was a stretch of a
  // microsecond per unit in which no wave of the compute unit multiplied, and requested by group 1 alone that
  // group's half steps were a microsecond longer than group 0's).  At the barrier both groups are done reading
  // patch t (group 0 since half step 2 t, group 1 just now) and every wave has waited for its own loads of patch
  // t + 1 (group 1 after its multiply, group 0 after its output stage), so patch t + 1 is complete and the buffer
  // of patch t is free for patch t + 2.
  issue_patch(unit_of(wg), 0, wave, 8);
  wait_vm<0>();
  block_sync();  // weights and the first patch are visible
  asm volatile("" ::"v"(bias_acc));  // the bias row is needed from here on: its wait belongs before the unit loop, not in it
  if constexpr (NKS > 0) {
#pragma unroll
    for (int k = 0; k < NKS; k++) bw[k] = read_b(k);
  }
  for (int hs = 0; hs <= 2 * my_units; hs++) {
    if ((hs & 1) != grp && (hs >> 1) + 1 < my_units) issue_patch(unit_of(wg + ((hs >> 1) + 1) * wgs), ((hs >> 1) + 1) & 1, wave, 8);
    const int rel = hs - grp;
    if (rel >= 0 && (rel >> 1) < my_units) {
      const Unit w = unit_of(wg + (rel >> 1) * wgs);
      if (!(rel & 1)) {
        multiply(w, (rel >> 1) & 1);
        wait_vm<0>();  // this wave's share of the next patch has landed (and its earlier stores have drained)
      } else {
        const int mrow0 = w.img * npix + w.q0 + wm * WTM + (lane & 31);
        const int m_end = (w.img + 1) * npix;  // rows of the unit past the end of its image belong to nobody
        halo_store_tiles(p, mrow0, m_end, n0 + wn * 32, acc, lane);
        if (grp == 0) wait_vm<0>();  // group 0's share of the next patch was requested at the top of this half step
      }
    }
    if (hs & 1) block_sync();
  }
}

// Geometry of the patch kernel for a convolution, or false when the convolution does not fit it.
static inline bool conv_halo_plan(const GemmParams& p, int bm, ConvHaloParams* h, size_t* lds_bytes) {
  if (p.Cin < 32 || p.Cin % 32 != 0 || p.Cin > 1008 || p.N % 16 != 0 || p.K < 32 || p.KW < 1 || p.stride < 1) return false;
  if (p.bias != nullptr && p.bias_ld != 0) return false;
  if ((((uintptr_t)p.C) & 15) != 0 || p.ldc % 16 != 0) return false;  // whole 16-byte output stores
  const int KH = p.K / (p.KW * p.Cin);
  if (KH < 1 || KH * p.KW * p.Cin != p.K) return false;
  const int64_t npix = (int64_t)p.OH * p.OW;
  if (npix < 1 || npix > (1 << 24) || p.M % npix != 0) return false;
  const int nkt = (p.K + 127) / 128;
  const int WP = (p.OW - 1) * p.stride + p.KW;  // patch width in input pixels, padding included
  const int WQ = (WP + p.stride - 1) / p.stride;
  const int ROWP = p.stride * WQ;
  const int SP = p.Cin / 16 + 1;
  int span = (bm + p.OW - 2) / p.OW + 1;  // output rows that bm consecutive pixels can touch
  if (span > p.OH) span = p.OH;
  const int rin_max = (span - 1) * p.stride + KH;
  const int64_t hb = (((int64_t)rin_max * ROWP * SP * 16) + 1023) / 1024 * 1024;
  const int64_t lds = (int64_t)nkt * 8192 + 2 * hb;
  if (lds > 160 * 1024) return false;
  if ((int64_t)rin_max * ROWP * SP >= (1 << 20) || (int64_t)p.H * p.W * p.Cin >= (1ll << 31)) return false;
  h->KH = KH, h->WQ = WQ, h->ROWP = ROWP, h->SP = SP, h->PITCH = SP * 16;
  h->HB = (int32_t)hb;
  h->U = (int32_t)((npix + bm - 1) / bm);
  const int64_t units = (p.M / npix) * h->U;
  if (units > (1 << 24)) return false;
  h->units = (int32_t)units;
  h->nks = p.K / 32;
  if (h->nks > 64) return false;  // one lane of the tap table per K-step
  h->PPI = 64 / SP;
  h->CPR = (ROWP + h->PPI - 1) / h->PPI;
  h->RIN = rin_max;
  h->NPAD_R = WP - p.pad - p.W > 0 ? WP - p.pad - p.W : 0;
  if (p.pad > WP) return false;
  h->dWQ = FastDiv::make(WQ), h->dOW = FastDiv::make(p.OW), h->dU = FastDiv::make(h->U);
  h->dPADC = FastDiv::make((p.pad + h->NPAD_R) * (SP - 1) > 0 ? (p.pad + h->NPAD_R) * (SP - 1) : 1), h->dCC = FastDiv::make(SP - 1);
  h->dS = FastDiv::make(p.stride), h->dCIN = FastDiv::make(p.Cin), h->dKW = FastDiv::make(p.KW);
  *lds_bytes = (size_t)lds;
  return true;
}

template <int BM, int NKS>
static hipError_t launch_conv_halo_nks(const GemmParams& p, const ConvHaloParams& h, size_t lds, hipStream_t stream) {
  auto kern = conv_i8_halo_kernel<BM, NKS>;
  static std::atomic<bool> configured{false};
  if (const hipError_t e = allow_dynamic_lds_once(configured, kern, 160 * 1024)) return e;
  const int cus = compute_units();
  const int n_blocks = (p.N + 63) / 64;
  int wgs = cus / n_blocks;
  if (wgs < 1) wgs = 1;
  if (wgs > h.units) wgs = h.units;
  hipLaunchKernelGGL(kern, dim3((unsigned)(wgs * n_blocks)), dim3(512), lds, stream, p, h, n_blocks);
  return hipGetLastError();
}

// K depths with a register-resident-weights instantiation: 3 x 3 taps of 32 / 64 channels, 1 x 1 of 64 .. 256.
// Any other depth (up to 64 K-steps) runs the variant that reads its weight fragments from LDS in the K loop.
template <int BM>
static hipError_t launch_conv_halo(const GemmParams& p, const ConvHaloParams& h, size_t lds, hipStream_t stream) {
  switch (h.nks) {
    case 2: return launch_conv_halo_nks<BM, 2>(p, h, lds, stream);
    case 4: return launch_conv_halo_nks<BM, 4>(p, h, lds, stream);
    case 8: return launch_conv_halo_nks<BM, 8>(p, h, lds, stream);
    case 9: return launch_conv_halo_nks<BM, 9>(p, h, lds, stream);
    case 18: return launch_conv_halo_nks<BM, 18>(p, h, lds, stream);
    default: return launch_conv_halo_nks<BM, 0>(p, h, lds, stream);
  }
}

// Tile codes of the patch kernel: 321 = units of 256 output pixels, 161 = units of 128.
static inline bool halo_tile_rows(int tile, int* bm) {
  if (tile == 321) return *bm = 256, true;
  if (tile == 161) return *bm = 128, true;
  return false;
}

}  // namespace ac
