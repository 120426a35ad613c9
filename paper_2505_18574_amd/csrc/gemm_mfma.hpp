// Tiled MFMA GEMM for gfx950 (CDNA4), shared by the int8 GEMM, the int8
// implicit-GEMM convolution and the bf16 GEMM.
//
// One workgroup owns a BM x BN tile of C.  Per K step of 128 bytes of A-row:
//   global (16 B per lane, coalesced) -> registers -> LDS (double buffered)
//   LDS -> MFMA operands: A rows by ds_read_b128 (K is contiguous in A);
//   B columns by the gfx950 transposing LDS reads (ds_read_b64_tr_b8/_b16),
//   because B is K x N row-major and the matrix unit wants K contiguous per lane.
//   32x32 MFMA tiles (i32_32x32x32_i8 / f32_32x32x16_bf16), accumulators in registers.
// The two MFMA source operands are swapped (B^T tile as the row operand, A tile
// as the column operand) so that each lane ends up holding 4 consecutive n of one
// row m: the epilogue can then requantise in registers and store 4 packed int8
// (or a float4) without an LDS transpose.
#pragma once
#include "common.hpp"
#include <type_traits>

namespace ac {

#define AC_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))

struct TypeI8 {
  static constexpr int EB = 1;  // element bytes
  using accv = v16i;
  static __device__ __forceinline__ accv zero() {
    accv z;
#pragma unroll
    for (int r = 0; r < 16; r++) z[r] = 0;
    return z;
  }
  static __device__ __forceinline__ accv mfma(v4i rowop, v4i colop, accv c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(rowop, colop, c, 0, 0, 0);
  }
  // 16 consecutive k (bytes) of one B column, gathered from K-major LDS rows.
  // Within a 16-lane group lane i supplies the address of 8 bytes of row i/2 and
  // receives 8 k-values of column i.
  static __device__ __forceinline__ v4i read_col(const unsigned char* tile, int stride, int k0, int ncol_bytes, int lane) {
    int i = lane & 15;
    const unsigned char* p = tile + (k0 + (i >> 1)) * stride + ncol_bytes + 8 * (i & 1);
    v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32(AC_LDS(v2i, p));
    v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32(AC_LDS(v2i, p + 8 * stride));
    return (v4i){lo[0], lo[1], hi[0], hi[1]};
  }
};

struct TypeBF16 {
  static constexpr int EB = 2;
  using accv = v16f;
  static __device__ __forceinline__ accv zero() {
    accv z;
#pragma unroll
    for (int r = 0; r < 16; r++) z[r] = 0.f;
    return z;
  }
  static __device__ __forceinline__ accv mfma(v4i rowop, v4i colop, accv c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, rowop), __builtin_bit_cast(v8bf, colop), c, 0, 0, 0);
  }
  // 8 consecutive k of one B column: lane i of a 16-lane group addresses 4
  // elements of row i/4 and receives 4 k-values of column i.
  static __device__ __forceinline__ v4i read_col(const unsigned char* tile, int stride, int k0, int ncol_bytes, int lane) {
    int i = lane & 15;
    const unsigned char* p = tile + (k0 + (i >> 2)) * stride + ncol_bytes + 8 * (i & 3);
    v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(AC_LDS(v4s, p));
    v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(AC_LDS(v4s, p + 4 * stride));
    v2i l2 = __builtin_bit_cast(v2i, lo), h2 = __builtin_bit_cast(v2i, hi);
    return (v4i){l2[0], l2[1], h2[0], h2[1]};
  }
};

// 16 bytes from p, of which only the first `valid` (may be <= 0 or >= 16) exist.
static __device__ __forceinline__ v4i load16_bytes(const unsigned char* p, int valid) {
  unsigned int w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int e = 0; e < 16; e++)
    if (e < valid) w[e >> 2] |= (unsigned int)p[e] << (8 * (e & 3));
  return (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
}

// Without the 16-byte guarantee a whole chunk at a 4-byte aligned address is still four dword loads rather than
// sixteen byte loads (a row pitch that is a multiple of 4 but not of 16, say N = 1000, keeps every chunk there).
template <bool ALIGNED>
static __device__ __forceinline__ v4i load16(const unsigned char* p, int valid) {
  if (valid <= 0) return (v4i){0, 0, 0, 0};
  if (ALIGNED && valid >= 16) return *(const v4i*)p;
  if (!ALIGNED && valid >= 16 && (((uintptr_t)p) & 3) == 0) {
    const int* q = (const int*)p;
    return (v4i){q[0], q[1], q[2], q[3]};
  }
  return load16_bytes(p, valid);
}

// XCD-aware tile order.  Workgroups are dealt round-robin to the 8 XCDs (each
// with its own L2), so workgroup b runs on XCD b % 8.  Give every XCD one
// contiguous run of logical tile ids, and lay those ids out in bands of GROUP_M
// tile-rows so that a run is a compact rectangle sharing A rows and B columns.
static __device__ __forceinline__ void tile_coords(int b, int nblocks, int tiles_m, int tiles_n, int& tm, int& tn) {
  constexpr int XCDS = 8, GROUP_M = 4;
  int q = nblocks / XCDS, r = nblocks % XCDS;
  int xcd = b % XCDS, idx = b / XCDS;
  int id = xcd * q + (xcd < r ? xcd : r) + idx;
  int group_size = GROUP_M * tiles_n;
  int group = id / group_size;
  int first_m = group * GROUP_M;
  int gsz = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
  int in_group = id - group * group_size;
  tm = first_m + in_group % gsz;
  tn = in_group / gsz;
}

// Epilogue policies -----------------------------------------------------------
// store4(): for one lane, 4 accumulators of row m at columns n .. n+3 (the generic kernel, which always swaps
// the MFMA operands).  tile(): one 32x32 accumulator tile of the direct-to-LDS kernel, whose operand order the
// policy chooses with SWAP:
//   SWAP (B^T tile as the row operand): register r of lane l is row l % 32, column 8 (r/4) + 4 (l/32) + r % 4:
//     a lane owns runs of 4 consecutive columns of one row.  Right for 1-byte outputs, which pack 4 (and, after
//     a lane exchange, 16) of them per store.
//   !SWAP: register r of lane l is row 8 (r/4) + 4 (l/32) + r % 4, column l % 32: the 32 lanes of a half-wave
//     own 32 consecutive columns of one row, so a 4-byte-per-lane store writes a whole 128-byte row segment.
//     Right for 4-byte outputs: with the swapped order a store instruction scatters 32-byte pieces over 32
//     rows, which the memory system drains at half the rate (measured on a store-bound GEMM).
// tile() receives the tile origin (mrow0, ncol0).

// Applies f(r, m, n) to the 16 accumulators of an unswapped tile: r = register, (m, n) = its coordinates.
template <class F>
static __device__ __forceinline__ void for_each_unswapped(int mrow0, int ncol0, int lane, F f) {
#pragma unroll
  for (int r = 0; r < 16; r++) f(r, mrow0 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3), ncol0 + (lane & 31));
}

// An epilogue that can take a whole wave tile at once declares WAVE_TILE.
template <class E, class = void>
struct has_wave_tile : std::false_type {};
template <class E>
struct has_wave_tile<E, std::void_t<decltype(E::WAVE_TILE)>> : std::true_type {};

// int8 output stage: bias, v / 2^shift to nearest (halves to even), saturate, ReLU.
struct EpilogueI8 {
  static constexpr bool SWAP = true;
  static constexpr bool LDS_STAGED = false;
  static __device__ __forceinline__ int requant(int v, int shift, int act) {
    int fl = v >> shift;
    unsigned int rem = (unsigned int)v & ((1u << shift) - 1u);
    unsigned int half = shift > 0 ? (1u << (shift - 1)) : 0u;
    int inc = (shift > 0) && (rem > half || (rem == half && (fl & 1)));
    int q = fl + inc;
    q = q > 127 ? 127 : q;
    q = q < -128 ? -128 : q;
    if (act) q = q < 0 ? 0 : q;
    return q;
  }
  template <bool VEC, bool ADD_BIAS = true>
  static __device__ __forceinline__ void store4(const GemmParams& p, int m, int n, const int* a, int = 0) {
    if (m >= p.M || n >= p.N) return;
    int8_t* C = (int8_t*)p.C;
    int v[4];
    const bool full = n + 3 < p.N;
#pragma unroll
    for (int e = 0; e < 4; e++) {
      int b = 0;
      if (ADD_BIAS && p.bias && (full || n + e < p.N)) b = p.bias_ld == 0 ? p.bias[n + e] : p.bias[(int64_t)m * p.bias_ld + n + e];
      v[e] = requant(a[e] + b, p.shift, p.act);
    }
    int8_t* dst = C + (int64_t)m * p.ldc + n;
    if (VEC && full) {
      unsigned int w = (unsigned int)(v[0] & 0xff) | ((unsigned int)(v[1] & 0xff) << 8) | ((unsigned int)(v[2] & 0xff) << 16) | ((unsigned int)(v[3] & 0xff) << 24);
      *(unsigned int*)dst = w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; e++)
        if (n + e < p.N) dst[e] = (int8_t)v[e];
    }
  }

  // ---- tile-level interface of the direct-to-LDS kernels ----------------------------------------------
  // One 32x32 MFMA tile: lane l holds row m = row0 + l % 32 and, for q = 0..3, columns
  // ncol0 + 8q + 4 (l / 32) + 0..3.
  struct Pre {
    v4i bias[4];  // bias of this lane's 16 columns (row-vector bias only), fetched before the K loop
  };
  // The bias row is read through a bounds-checked buffer of N int32 (no row bias: zero records), so the four
  // loads carry no branches: columns beyond N, and every column when there is no row bias, come back as zeros.
  static __device__ __forceinline__ void prefetch(const GemmParams& p, int ncol0, int lane, Pre& pre) {
    const bool row_bias = p.bias != nullptr && p.bias_ld == 0;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)p.bias, 0, row_bias && p.N < (1 << 29) ? p.N * 4 : 0, 0x00020000);
    const int off = (ncol0 + 4 * (lane >> 5)) * 4;
    if (p.N < (1 << 29)) {  // wave-uniform; byte offsets fit the signed 32-bit buffer arithmetic
#pragma unroll
      for (int q = 0; q < 4; q++) pre.bias[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off + 32 * q, 0, 0);
    } else {
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int n = ncol0 + 8 * q + 4 * (lane >> 5);
        pre.bias[q] = (v4i){0, 0, 0, 0};
        if (row_bias && n + 3 < p.N) pre.bias[q] = (v4i){p.bias[n], p.bias[n + 1], p.bias[n + 2], p.bias[n + 3]};
      }
    }
  }
  // Fast form of requant() for 1 <= shift <= 23: floor((t + 2^(shift-1) - 1 + bit) / 2^shift) with bit = bit
  // `shift` of t rounds halves to even.  The rounding shift is monotone, so the output clamp is taken on the way
  // in: t is clamped to [lo, hi] with hi = 127 * 2^shift + 2^(shift-1) - 1, the largest t that still rounds to
  // 127, and lo = -128 * 2^shift, which rounds to -128 exactly (0 with ReLU: every negative t ends as 0), which
  // also keeps the rounding add inside int32 and makes both activations the same code.
  struct FastQuant {
    int shift, rnd, lo, hi;
    float scale, lo_f, hi_f;  // 2^-shift and the bounds as fp32 (exact for shifts up to 17)
  };
  static __device__ __forceinline__ FastQuant fast_quant(int shift, int act) {
    const int rnd = (1 << (shift - 1)) - 1, lo = act ? 0 : -128 * (1 << shift), hi = (127 << shift) + rnd;
    return {shift, rnd, lo, hi, __builtin_ldexpf(1.f, -shift), (float)lo, (float)hi};
  }
  // FLOAT_ROUND (shift <= 17): the bounds are at most 2^24 in magnitude, so they and everything between them are
  // exact in fp32, and the conversion of a sum outside them (rounded, but monotone) stays outside them: the sum is
  // converted first and clamped as a float (one median instruction), and one fused multiply-add
  // c * 2^-shift + 1.5 * 2^23 rounds the quotient to an integer, halves to even (the result lies in [2^23, 2^24),
  // where fp32 steps by 1 and the constant is even): the low byte of its bit pattern is the two's-complement
  // output.  Three VALU instructions per value; only the low byte of the returned word is meaningful.
  // Otherwise (shifts 18..23): clamp (a maximum and a minimum: with bounds that are not constants the compiler
  // cannot form the integer median), bit extract, three-operand add, shift.
  template <bool FLOAT_ROUND = false>
  static __device__ __forceinline__ int requant_fast(int t, const FastQuant& f) {
    if constexpr (FLOAT_ROUND) {
      const float c = __builtin_amdgcn_fmed3f((float)t, f.lo_f, f.hi_f);
      return __builtin_bit_cast(int, __builtin_fmaf(c, f.scale, 12582912.f));
    } else {
      int c = t < f.lo ? f.lo : t;
      c = c > f.hi ? f.hi : c;
      const int bit = (int)__builtin_amdgcn_ubfe((unsigned)c, (unsigned)f.shift, 1u);
      return (c + bit + f.rnd) >> f.shift;
    }
  }
  // The low bytes of four words in one dword (v0 lowest).
  static __device__ __forceinline__ unsigned pack4(int v0, int v1, int v2, int v3) {
    const unsigned lo = __builtin_amdgcn_perm((unsigned)v1, (unsigned)v0, 0x0c0c0400u);
    const unsigned hi = __builtin_amdgcn_perm((unsigned)v3, (unsigned)v2, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
  }
  // The 16 values of one lane (accumulator + bias), quantised and packed four to a dword -> 16 output bytes in
  // column order after the lane exchange: lanes l and l + 32 hold interleaved 4-byte pieces of the same row.
  // Swapping the upper half of d[0] (d[1]) with the lower half of d[2] (d[3]) leaves 16 consecutive bytes in every
  // lane: columns 0..15 in lanes 0..31, columns 16..31 in lanes 32..63, so a row leaves as two whole 16-byte stores.
  static __device__ __forceinline__ v4i exchange16(const unsigned* d) {
    typedef unsigned v2u __attribute__((ext_vector_type(2)));
    const v2u s02 = __builtin_amdgcn_permlane32_swap(d[0], d[2], false, false);
    const v2u s13 = __builtin_amdgcn_permlane32_swap(d[1], d[3], false, false);
    return (v4i){(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
  }
  // Any shift / activation (requant).
  static __device__ __forceinline__ v4i quant16(const int* t, int shift, int act) {
    unsigned d[4];
#pragma unroll
    for (int q = 0; q < 4; q++) d[q] = pack4(requant(t[4 * q], shift, act), requant(t[4 * q + 1], shift, act), requant(t[4 * q + 2], shift, act), requant(t[4 * q + 3], shift, act));
    return exchange16(d);
  }
  // Fast form.
  template <bool FLOAT_ROUND = false>
  static __device__ __forceinline__ v4i quant16(const int* t, const FastQuant& f) {
    unsigned d[4];
#pragma unroll
    for (int q = 0; q < 4; q++)
      d[q] = pack4(requant_fast<FLOAT_ROUND>(t[4 * q], f), requant_fast<FLOAT_ROUND>(t[4 * q + 1], f), requant_fast<FLOAT_ROUND>(t[4 * q + 2], f), requant_fast<FLOAT_ROUND>(t[4 * q + 3], f));
    return exchange16(d);
  }
  // Fast form, the rounding picked by the shift (wave-uniform).
  static __device__ __forceinline__ v4i quant16_by_shift(const int* t, const FastQuant& f) {
    return f.shift <= 17 ? quant16<true>(t, f) : quant16<false>(t, f);
  }
  // The whole wave tile, TM x TN blocks of 32 x 32, when every block takes 16-byte stores, the bias is a row or
  // absent and the shift has the fast form: one decision per wave tile and straight-line code for its blocks (as
  // separate calls of tile() every block carries the whole decision tree, and the output stage of a 256 x 256
  // tile ran through some 90 KB of code).  BIASED as in tile().
  static constexpr bool WAVE_TILE = true;
  // acc_of(i, j) and pre_of(j) give block (i, j)'s accumulators and column block j's prefetched bias.
  template <bool BIASED, int TM, int TN, class ACC_OF, class PRE_OF>
  static __device__ __forceinline__ void wave_blocks(const GemmParams& p, int mrow0, int ncol0, ACC_OF acc_of, int lane, int esplit, PRE_OF pre_of) {
    int8_t* C = (int8_t*)p.C;
    const bool fast = ncol0 + 32 * TN <= p.N && (p.ldc & 15) == 0 && (((uintptr_t)C) & 15) == 0 && (p.bias == nullptr || p.bias_ld == 0) && p.shift >= 1 && p.shift <= 23;
    if (fast) {  // wave-uniform
      const FastQuant f = fast_quant(p.shift, p.act);
      auto blocks = [&](auto float_round) {
#pragma unroll
        for (int i = 0; i < TM; i++) {
          const int m = mrow0 + 32 * i + (lane & 31);
          int8_t* dst = C + (int64_t)m * p.ldc + ncol0 + 16 * (lane >> 5);
#pragma unroll
          for (int j = 0; j < TN; j++) {
            int t[16];
#pragma unroll
            for (int r = 0; r < 16; r++) t[r] = BIASED ? acc_of(i, j)[r] : acc_of(i, j)[r] + pre_of(j).bias[r >> 2][r & 3];  // no bias: the prefetch returned zeros
            const v4i o = quant16<decltype(float_round)::value>(t, f);
            if (m < p.M) *(v4i*)(dst + 32 * j) = o;
          }
        }
      };
      if (p.shift <= 17) blocks(std::true_type{});
      else blocks(std::false_type{});
    } else {
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++) tile<BIASED>(p, mrow0 + 32 * i, ncol0 + 32 * j, acc_of(i, j), lane, esplit, pre_of(j));
    }
  }
  template <bool BIASED = false, int TM, int TN, class ACC>
  static __device__ __forceinline__ void wave_tile(const GemmParams& p, int mrow0, int ncol0, const ACC (&acc)[TM][TN], int lane, int esplit, const Pre (&pre)[TN]) {
    wave_blocks<BIASED, TM, TN>(p, mrow0, ncol0, [&](int i, int j) -> const ACC& { return acc[i][j]; }, lane, esplit, [&](int j) -> const Pre& { return pre[j]; });
  }
  // A column of TM blocks with one bias block.
  template <bool BIASED = false, int TM, class ACC>
  static __device__ __forceinline__ void wave_column(const GemmParams& p, int mrow0, int ncol0, const ACC (&acc)[TM], int lane, const Pre& pre) {
    wave_blocks<BIASED, TM, 1>(p, mrow0, ncol0, [&](int i, int) -> const ACC& { return acc[i]; }, lane, 0, [&](int) -> const Pre& { return pre; });
  }
  // BIASED: the accumulators already hold the bias (a kernel that starts its sums from the bias row).
  template <bool BIASED = false, class ACC>
  static __device__ __forceinline__ void tile(const GemmParams& p, int mrow0, int ncol0, const ACC& acc, int lane, int, const Pre& pre) {
    const int m = mrow0 + (lane & 31);
    if (m >= p.M || ncol0 >= p.N) return;
    int8_t* C = (int8_t*)p.C;
    const bool wide = ncol0 + 32 <= p.N && (p.ldc & 15) == 0 && (((uintptr_t)C) & 15) == 0;
    const bool row_bias = p.bias && p.bias_ld == 0;
    if (wide) {
      int t[16];
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int n = ncol0 + 8 * q + 4 * (lane >> 5);
#pragma unroll
        for (int e = 0; e < 4; e++) {
          int b = 0;
          if constexpr (!BIASED) {
            b = row_bias ? pre.bias[q][e] : 0;
            if (p.bias && !row_bias) b = p.bias[(int64_t)m * p.bias_ld + n + e];
          }
          t[4 * q + e] = acc[4 * q + e] + b;
        }
      }
      const v4i o = p.shift >= 1 && p.shift <= 23 ? quant16_by_shift(t, fast_quant(p.shift, p.act)) : quant16(t, p.shift, p.act);
      *(v4i*)(C + (int64_t)m * p.ldc + ncol0 + 16 * (lane >> 5)) = o;
    } else {
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int n = ncol0 + 8 * q + 4 * (lane >> 5);
        int a4[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        if constexpr (BIASED) store4<true, false>(p, m, n, a4);
        else store4<true>(p, m, n, a4);
      }
    }
  }
};

// Split-K partial sums: raw int32 accumulators of K slice `split` go to partial[split][M][N]; the output stage
// runs in splitk_reduce_i8_kernel once every slice has been written.
struct EpiloguePartialI32 {
  static constexpr bool SWAP = false;
  static constexpr bool LDS_STAGED = true;  // the workspace is 16-byte aligned and N a multiple of 16 on this path
  typedef int StagedValue;
  static __device__ __forceinline__ int staged_in(const GemmParams&, int a) { return a; }
  static __device__ __forceinline__ void staged_out(const GemmParams& p, int m, int n, v4i o, int split) {
    *(v4i*)(p.partial + ((int64_t)split * p.M + m) * p.N + n) = o;
  }
  struct Pre {};
  static __device__ __forceinline__ void prefetch(const GemmParams&, int, int, Pre&) {}
  template <class ACC>
  static __device__ __forceinline__ void tile(const GemmParams& p, int mrow0, int ncol0, const ACC& acc, int lane, int split, const Pre&) {
    for_each_unswapped(mrow0, ncol0, lane, [&](int r, int m, int n) {
      if (m < p.M && n < p.N) p.partial[((int64_t)split * p.M + m) * p.N + n] = acc[r];
    });
  }
};

// Raw accumulator output (the accumulator-type read of the paper's accelerator: no scaling, no activation):
// C32[m][n] = acc + bias, int32, row stride ldc.
struct EpilogueRawI32 {
  static constexpr bool SWAP = false;
  static constexpr bool LDS_STAGED = true;  // C is 16-byte aligned with ldc a multiple of 4 on this path
  typedef int StagedValue;
  static __device__ __forceinline__ int staged_in(const GemmParams&, int a) { return a; }
  static __device__ __forceinline__ void staged_out(const GemmParams& p, int m, int n, v4i o, int) {
    if (p.bias) {
      const int32_t* b = p.bias_ld == 0 ? p.bias + n : p.bias + (int64_t)m * p.bias_ld + n;  // only 4-byte aligned
      o += (v4i){b[0], b[1], b[2], b[3]};
    }
    *(v4i*)((int32_t*)p.C + (int64_t)m * p.ldc + n) = o;
  }
  template <bool VEC>
  static __device__ __forceinline__ void store4(const GemmParams& p, int m, int n, const int* a, int = 0) {
    if (m >= p.M || n >= p.N) return;
    int32_t* dst = (int32_t*)p.C + (int64_t)m * p.ldc + n;
    int v[4];
#pragma unroll
    for (int e = 0; e < 4; e++) {
      int b = 0;
      if (p.bias && n + e < p.N) b = p.bias_ld == 0 ? p.bias[n + e] : p.bias[(int64_t)m * p.bias_ld + n + e];
      v[e] = a[e] + b;
    }
    if (VEC && n + 3 < p.N) {
      *(v4i*)dst = (v4i){v[0], v[1], v[2], v[3]};
    } else {
#pragma unroll
      for (int e = 0; e < 4; e++)
        if (n + e < p.N) dst[e] = v[e];
    }
  }
  struct Pre {};
  static __device__ __forceinline__ void prefetch(const GemmParams&, int, int, Pre&) {}
  template <class ACC>
  static __device__ __forceinline__ void tile(const GemmParams& p, int mrow0, int ncol0, const ACC& acc, int lane, int, const Pre&) {
    for_each_unswapped(mrow0, ncol0, lane, [&](int r, int m, int n) {
      if (m < p.M && n < p.N) {
        int b = 0;
        if (p.bias) b = p.bias_ld == 0 ? p.bias[n] : p.bias[(int64_t)m * p.bias_ld + n];
        ((int32_t*)p.C)[(int64_t)m * p.ldc + n] = acc[r] + b;
      }
    });
  }
};

// fp32 output: C = alpha * acc + beta * C (C read only when beta != 0).
struct EpilogueF32 {
  static constexpr bool SWAP = false;
  // The direct-to-LDS kernels hand over 4-byte outputs through an LDS transpose: staged_in() is applied to every
  // accumulator on its way into LDS, staged_out() receives four consecutive columns of one row.
  static constexpr bool LDS_STAGED = true;
  typedef float StagedValue;
  static __device__ __forceinline__ float staged_in(const GemmParams& p, float a) { return p.alpha * a; }
  static __device__ __forceinline__ void staged_out(const GemmParams& p, int m, int n, v4f o, int) {
    float* dst = (float*)p.C + (int64_t)m * p.ldc + n;
    if (p.beta != 0.f) o += p.beta * *(const v4f*)dst;
    *(v4f*)dst = o;
  }
  template <bool VEC>
  static __device__ __forceinline__ void store4(const GemmParams& p, int m, int n, const float* a, int = 0) {
    if (m >= p.M || n >= p.N) return;
    float* dst = (float*)p.C + (int64_t)m * p.ldc + n;
    const bool full = n + 3 < p.N;
    if (VEC && full) {
      v4f o = {p.alpha * a[0], p.alpha * a[1], p.alpha * a[2], p.alpha * a[3]};
      if (p.beta != 0.f) {
        v4f c = *(const v4f*)dst;
        o += p.beta * c;
      }
      *(v4f*)dst = o;
    } else {
#pragma unroll
      for (int e = 0; e < 4; e++)
        if (n + e < p.N) {
          float o = p.alpha * a[e];
          if (p.beta != 0.f) o += p.beta * dst[e];
          dst[e] = o;
        }
    }
  }
  struct Pre {};
  static __device__ __forceinline__ void prefetch(const GemmParams&, int, int, Pre&) {}
  template <class ACC>
  static __device__ __forceinline__ void tile(const GemmParams& p, int mrow0, int ncol0, const ACC& acc, int lane, int, const Pre&) {
    for_each_unswapped(mrow0, ncol0, lane, [&](int r, int m, int n) {
      if (m < p.M && n < p.N) {
        float* dst = (float*)p.C + (int64_t)m * p.ldc + n;
        float o = p.alpha * acc[r];
        if (p.beta != 0.f) o += p.beta * *dst;
        *dst = o;
      }
    });
  }
};

// Split-K output of the fp32 epilogue: every K slice adds alpha * (its partial product) into C with the
// hardware fp32 atomic add; C was set to beta * C by scale_c_f32_kernel before the slices run.  The order in
// which slices arrive is not fixed, so the last bits of a sum may differ between runs.
struct EpilogueAtomicF32 {
  static constexpr bool SWAP = false;
  static constexpr bool LDS_STAGED = false;
  struct Pre {};
  static __device__ __forceinline__ void prefetch(const GemmParams&, int, int, Pre&) {}
  template <class ACC>
  static __device__ __forceinline__ void tile(const GemmParams& p, int mrow0, int ncol0, const ACC& acc, int lane, int, const Pre&) {
    for_each_unswapped(mrow0, ncol0, lane, [&](int r, int m, int n) {
      if (m < p.M && n < p.N) unsafeAtomicAdd((float*)p.C + (int64_t)m * p.ldc + n, p.alpha * acc[r]);
    });
  }
};

// Split-K partial products in fp32: slice `split` stores its raw accumulators to partial[split][M][N] (the
// int32 workspace pointer reinterpreted); splitk_reduce_f32_kernel sums the slices in slice order and applies
// alpha / beta, so the result does not depend on which slice finishes first.
struct EpiloguePartialF32 {
  static constexpr bool SWAP = false;
  static constexpr bool LDS_STAGED = true;  // the workspace is 16-byte aligned and N a multiple of 8 on this path
  typedef float StagedValue;
  static __device__ __forceinline__ float staged_in(const GemmParams&, float a) { return a; }
  static __device__ __forceinline__ void staged_out(const GemmParams& p, int m, int n, v4f o, int split) {
    *(v4f*)((float*)p.partial + ((int64_t)split * p.M + m) * p.N + n) = o;
  }
  struct Pre {};
  static __device__ __forceinline__ void prefetch(const GemmParams&, int, int, Pre&) {}
  template <class ACC>
  static __device__ __forceinline__ void tile(const GemmParams& p, int mrow0, int ncol0, const ACC& acc, int lane, int split, const Pre&) {
    for_each_unswapped(mrow0, ncol0, lane, [&](int r, int m, int n) {
      if (m < p.M && n < p.N) ((float*)p.partial)[((int64_t)split * p.M + m) * p.N + n] = acc[r];
    });
  }
};

// A-operand addressing ----------------------------------------------------------
// AMODE 0: A is an M x K matrix.  AMODE 1: A(m, k) is gathered from an NHWC image
// (m -> (image, oh, ow), k -> (kh, kw, ci)), zero outside the image.
template <int AMODE>
struct ARow;

template <>
struct ARow<0> {
  const unsigned char* ptr;  // start of the row, null when the row is outside M
  __device__ __forceinline__ void init(const GemmParams& p, int m, int EB) {
    ptr = m < p.M ? (const unsigned char*)p.A + (int64_t)m * p.lda * EB : nullptr;
  }
};

template <>
struct ARow<1> {
  int base;  // element offset of (image, ih0, iw0, 0); may be negative-side of the image, only used when in range
  short ih0, iw0;
  bool ok;
  __device__ __forceinline__ void init(const GemmParams& p, int m, int) {
    ok = m < p.M;
    int mm = ok ? m : 0;
    int ow = mm % p.OW;
    int t = mm / p.OW;
    int oh = t % p.OH;
    int img = t / p.OH;
    ih0 = (short)(oh * p.stride - p.pad);
    iw0 = (short)(ow * p.stride - p.pad);
    base = ((img * p.H + ih0) * p.W + iw0) * p.Cin;
  }
};

template <class T, int BM, int BN, int WAVES_M, int WAVES_N>
struct TileGeometry {
  static constexpr int EB = T::EB;
  static constexpr int KTB = 128;            // bytes of K per A row per step
  static constexpr int BK = KTB / EB;        // elements of K per step
  static constexpr int THREADS = 64 * WAVES_M * WAVES_N;
  static constexpr int A_STRIDE = KTB + 16;  // padded LDS row: conflict-free b128 reads
  static constexpr int B_STRIDE = BN * EB + 16;
  static constexpr int A_BYTES = BM * A_STRIDE;
  static constexpr int B_BYTES = BK * B_STRIDE;
  static constexpr int STAGE = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE;
  static constexpr int A_ROWS_PER_PASS = THREADS / 8;
  static constexpr int A_IT = BM / A_ROWS_PER_PASS;
  static constexpr int B_CPR = BN * EB / 16;  // 16-byte chunks per B row
  static constexpr int B_ROWS_PER_PASS = THREADS / B_CPR;
  static constexpr int B_IT = BK / B_ROWS_PER_PASS;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(BM % A_ROWS_PER_PASS == 0 && A_IT >= 1, "A tile / thread mismatch");
  static_assert(THREADS % B_CPR == 0 && BK % B_ROWS_PER_PASS == 0 && B_IT >= 1, "B tile / thread mismatch");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
};

template <class T, class EPI, int BM, int BN, int WAVES_M, int WAVES_N, int AMODE, bool ALIGNED>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) gemm_mfma_kernel(const GemmParams p, const int tiles_m, const int tiles_n) {
  using G = TileGeometry<T, BM, BN, WAVES_M, WAVES_N>;
  constexpr int EB = G::EB;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  int tm, tn;
  tile_coords(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  typename T::accv acc[G::TM][G::TN];
#pragma unroll
  for (int i = 0; i < G::TM; i++)
#pragma unroll
    for (int j = 0; j < G::TN; j++) acc[i][j] = T::zero();

  // ---- per-thread staging assignment
  const int a_cc = t & 7, a_r0 = t >> 3;
  const int b_cc = t % G::B_CPR, b_r0 = t / G::B_CPR;
  ARow<AMODE> arow[G::A_IT];
#pragma unroll
  for (int i = 0; i < G::A_IT; i++) arow[i].init(p, m0 + a_r0 + i * G::A_ROWS_PER_PASS, EB);
  const int kbytes = p.K * EB;               // valid bytes per A row
  const int nbytes = p.N * EB;               // valid bytes per B row
  const int b_col = n0 * EB + b_cc * 16;     // byte column of this thread's B chunks
  const unsigned char* Bp = (const unsigned char*)p.B;

  v4i ra[G::A_IT], rb[G::B_IT];

  auto gload = [&](int kt) {
    const int ka = kt * G::KTB + a_cc * 16;  // byte offset along K of this thread's A chunks
    if constexpr (AMODE == 0) {
#pragma unroll
      for (int i = 0; i < G::A_IT; i++) {
        const unsigned char* rp = arow[i].ptr;
        ra[i] = rp ? load16<ALIGNED>(rp + ka, kbytes - ka) : (v4i){0, 0, 0, 0};
      }
    } else {
      const unsigned char* in = (const unsigned char*)p.A;
      if constexpr (ALIGNED) {  // Cin % 16 == 0: a chunk never straddles a kernel tap
        int tap = ka / p.Cin, ci = ka - tap * p.Cin;
        int kh = tap / p.KW, kw = tap - kh * p.KW;
        int koff = (kh * p.W + kw) * p.Cin + ci;
#pragma unroll
        for (int i = 0; i < G::A_IT; i++) {
          const ARow<1>& r = arow[i];
          int ih = r.ih0 + kh, iw = r.iw0 + kw;
          bool ok = r.ok && ka < kbytes && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
          ra[i] = ok ? *(const v4i*)(in + r.base + koff) : (v4i){0, 0, 0, 0};
        }
      } else {
#pragma unroll
        for (int i = 0; i < G::A_IT; i++) {
          const ARow<1>& r = arow[i];
          unsigned int w[4] = {0u, 0u, 0u, 0u};
          for (int e = 0; e < 16; e++) {
            int k = ka + e;
            if (r.ok && k < kbytes) {
              int tap = k / p.Cin, ci = k - tap * p.Cin;
              int kh = tap / p.KW, kw = tap - kh * p.KW;
              int ih = r.ih0 + kh, iw = r.iw0 + kw;
              if ((unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
                w[e >> 2] |= (unsigned int)in[r.base + (kh * p.W + kw) * p.Cin + ci] << (8 * (e & 3));
            }
          }
          ra[i] = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
        }
      }
    }
#pragma unroll
    for (int i = 0; i < G::B_IT; i++) {
      int k = kt * G::BK + b_r0 + i * G::B_ROWS_PER_PASS;
      rb[i] = k < p.K ? load16<ALIGNED>(Bp + ((int64_t)k * p.ldb) * EB + b_col, nbytes - b_col) : (v4i){0, 0, 0, 0};
    }
  };

  auto lstore = [&](int buf) {
    unsigned char* As = smem + buf * G::STAGE;
    unsigned char* Bs = As + G::A_BYTES;
#pragma unroll
    for (int i = 0; i < G::A_IT; i++) *(v4i*)(As + (a_r0 + i * G::A_ROWS_PER_PASS) * G::A_STRIDE + a_cc * 16) = ra[i];
#pragma unroll
    for (int i = 0; i < G::B_IT; i++) *(v4i*)(Bs + (b_r0 + i * G::B_ROWS_PER_PASS) * G::B_STRIDE + b_cc * 16) = rb[i];
  };

  auto compute = [&](int buf) {
    const unsigned char* As = smem + buf * G::STAGE;
    const unsigned char* Bs = As + G::A_BYTES;
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {  // 4 MFMA K-steps of 32 bytes per tile
      v4i af[G::TM], bf[G::TN];
      const int kb = ks * 32 + (lane >> 5) * 16;  // this lane's 16 bytes of K
#pragma unroll
      for (int i = 0; i < G::TM; i++) af[i] = *(const v4i*)(As + (wm * G::WTM + i * 32 + (lane & 31)) * G::A_STRIDE + kb);
#pragma unroll
      for (int j = 0; j < G::TN; j++)
        bf[j] = T::read_col(Bs, G::B_STRIDE, kb / EB, (wn * G::WTN + j * 32 + 16 * ((lane >> 4) & 1)) * EB, lane);
#pragma unroll
      for (int i = 0; i < G::TM; i++)
#pragma unroll
        for (int j = 0; j < G::TN; j++) acc[i][j] = T::mfma(bf[j], af[i], acc[i][j]);
    }
  };

  const int nkt = (kbytes + G::KTB - 1) / G::KTB;
  if (nkt > 0) {
    gload(0);
    lstore(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nkt; kt++) {
    const bool more = kt + 1 < nkt;
    if (more) gload(kt + 1);
    compute(kt & 1);
    if (more) lstore((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds, per 32x32 tile and per q, row m and columns n..n+3
  const bool vec = ALIGNED;  // host guarantees C alignment / ldc divisibility when ALIGNED
#pragma unroll
  for (int i = 0; i < G::TM; i++) {
    const int m = m0 + wm * G::WTM + i * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < G::TN; j++) {
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int n = n0 + wn * G::WTN + j * 32 + 8 * q + 4 * (lane >> 5);
        decltype(acc[i][j][0] + 0) a4[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        if (vec) EPI::template store4<true>(p, m, n, a4);
        else EPI::template store4<false>(p, m, n, a4);
      }
    }
  }
}

// Host-side launcher for one instantiation.
template <class T, class EPI, int BM, int BN, int WAVES_M, int WAVES_N, int AMODE, bool ALIGNED>
static hipError_t launch_tile(const GemmParams& p, hipStream_t stream) {
  using G = TileGeometry<T, BM, BN, WAVES_M, WAVES_N>;
  auto kern = gemm_mfma_kernel<T, EPI, BM, BN, WAVES_M, WAVES_N, AMODE, ALIGNED>;
  static std::atomic<bool> configured{G::LDS_BYTES <= 64 * 1024};
  if (const hipError_t e = allow_dynamic_lds_once(configured, kern, G::LDS_BYTES)) return e;
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(G::THREADS), G::LDS_BYTES, stream, p, tiles_m, tiles_n);
  return hipGetLastError();
}

}  // namespace ac
