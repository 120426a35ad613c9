// Fast-path tiled MFMA GEMM for gfx950: operands stream global -> LDS directly
// (global_load_lds_dwordx4, no register staging, no ds_write), LDS tiles are
// XOR-swizzled instead of padded, and the K loop is software-pipelined over a
// ring of LDS stages with one workgroup barrier per K tile.
//
// Preconditions (checked by the host launcher; anything else takes the generic
// kernel in gemm_mfma.hpp): all base pointers 16-byte aligned, row pitches of A
// and B multiples of 16 bytes, K and N multiples of 16 bytes' worth of elements,
// C suitably aligned for vector stores.  M, N, K need not be multiples of the
// tile: out-of-range 16-byte chunks are fetched from a 16-byte block of zeros.
//
// LDS layouts (16-byte slots; a direct-to-LDS wave instruction fills 64
// consecutive slots, the source address of each slot is free):
//   A tile  [BM rows][KTB/16 slots]      slot' = slot ^ ((row / rows-per-256B) & (slots-1))
//   B tile  [KTB/EB k-rows][BN*EB/16]    32-column segments XOR-ed with the k-row (BSwizzle)
// chosen so that the ds_read_b128 of an A fragment (32 rows x 16 B) and the
// transposing ds_read_b64_tr of a B fragment (4 or 8 k-rows x 64 or 32 B) touch
// every LDS bank once.
#pragma once
#include <type_traits>
#include <utility>
#include "gemm_mfma.hpp"

namespace ac {

// 16 bytes of zeros in device memory: the source for chunks outside M, N, K and
// for convolution taps that fall in the padding.
__device__ __attribute__((aligned(16))) const int g_zero16[4] = {0, 0, 0, 0};

// One direct-to-LDS wave instruction: lane i copies 16 bytes from gptr to
// lds_base + 16*i.  Issued through inline assembly so that the compiler does not
// serialise later LDS reads against it; ordering is enforced explicitly with
// wait_vm<N>() + a barrier.  The s_nop is the wait state that an LDS-DMA instruction needs after a scalar write
// of M0 (the compiler pads its own such pairs; it cannot see into the assembly).  It costs nothing measurable.
static __device__ __forceinline__ void load_to_lds16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
// Same, with the source given as a wave-uniform base pointer plus a 32-bit byte offset per lane.
static __device__ __forceinline__ void load_to_lds16_so(const void* sbase, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase) : "memory");
}
// The same through a buffer descriptor with a 32-bit byte offset per lane: a lane whose offset lies beyond the
// descriptor's size receives zeros (the hardware bounds check), which is how the convolution gather writes its
// padding: no pointer select, no block of zeros.
static __device__ __forceinline__ void buffer_to_lds16(v4i rsrc, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_base), "v"(voff), "s"(rsrc) : "memory");
}
// Workgroup barrier that waits for this wave's LDS traffic only.  __syncthreads() would also drain every
// outstanding global store, which would serialise one tile's epilogue with the next tile's main loop.
static __device__ __forceinline__ void block_sync() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
template <int N>
static __device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// B-tile swizzle.  A transposing read phase touches R k-rows (4 for bf16, 8 for int8) times one
// SEGB-byte segment (64 / 32 bytes: 32 columns).  With RPW rows per 256-byte bank window, XOR-ing the
// segment index with (row / RPW) & MASK spreads those R segments over all 64 banks.
template <int EB, int B_ROW>
struct BSwizzle {
  static constexpr int R = EB == 2 ? 4 : 8;
  static constexpr int SEGB = EB == 2 ? 64 : 32;
  static constexpr int SEG_SHIFT = EB == 2 ? 6 : 5;
  static constexpr int SEGS = B_ROW / SEGB;
  static constexpr int RPW = B_ROW >= 256 ? 1 : 256 / B_ROW;
  static constexpr int SPAN = R / RPW < SEGS ? R / RPW : SEGS;
  static constexpr int MASK = SPAN - 1;
  static_assert(SEGS >= 1 && (SEGS & (SEGS - 1)) == 0 && SPAN >= 1, "B tile width must be a power of two of 32-column segments");
  static __device__ __forceinline__ int seg_xor(int row) { return (row / RPW) & MASK; }
  // logical 16-byte slot held by physical slot `pslot` of k-row `row` (an involution)
  static __device__ __forceinline__ int slot(int pslot, int row) { return pslot ^ (seg_xor(row) << (SEG_SHIFT - 4)); }
};

// Swizzled B-fragment reads (see TypeI8/TypeBF16::read_col for the lane roles).
// kb: byte offset of this lane's 16 K-bytes inside the 128-byte K tile; seg: index of the 32-column block.
template <int B_ROW>
static __device__ __forceinline__ v4i dtl_read_col_bf16(const unsigned char* Bs, int kb, int seg, int lane) {
  using S = BSwizzle<2, B_ROW>;
  const int i = lane & 15, g1 = (lane >> 4) & 1;
  const int r = (kb >> 1) + (i >> 2);  // k-row; rows r and r + 4 share one swizzle term
  const unsigned char* p = Bs + r * B_ROW + ((seg ^ S::seg_xor(r)) << 6) + g1 * 32 + 8 * (i & 3);
  v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(AC_LDS(v4s, p));
  v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(AC_LDS(v4s, p + 4 * B_ROW));
  v2i l2 = __builtin_bit_cast(v2i, lo), h2 = __builtin_bit_cast(v2i, hi);
  return (v4i){l2[0], l2[1], h2[0], h2[1]};
}
template <int B_ROW>
static __device__ __forceinline__ v4i dtl_read_col_i8(const unsigned char* Bs, int kb, int seg, int lane) {
  using S = BSwizzle<1, B_ROW>;
  const int i = lane & 15, g1 = (lane >> 4) & 1;
  const int r = kb + (i >> 1);  // k-row; rows r and r + 8 share one swizzle term
  const unsigned char* p = Bs + r * B_ROW + ((seg ^ S::seg_xor(r)) << 5) + g1 * 16 + 8 * (i & 1);
  v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32(AC_LDS(v2i, p));
  v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32(AC_LDS(v2i, p + 8 * B_ROW));
  return (v4i){lo[0], lo[1], hi[0], hi[1]};
}
// Byte offset, inside a B tile, of the first of the two transposing reads of dtl_read_col (the second lies
// HI rows further down), and the fragment read at a given address.
template <class T, int B_ROW>
static __device__ __forceinline__ int dtl_col_off(int kb, int seg, int lane) {
  using S = BSwizzle<T::EB, B_ROW>;
  const int i = lane & 15, g1 = (lane >> 4) & 1;
  if constexpr (T::EB == 2) {
    const int r = (kb >> 1) + (i >> 2);
    return r * B_ROW + ((seg ^ S::seg_xor(r)) << 6) + g1 * 32 + 8 * (i & 3);
  } else {
    const int r = kb + (i >> 1);
    return r * B_ROW + ((seg ^ S::seg_xor(r)) << 5) + g1 * 16 + 8 * (i & 1);
  }
}
template <class T, int B_ROW>
static __device__ __forceinline__ v4i dtl_read_col_at(const unsigned char* p) {
  if constexpr (T::EB == 2) {
    v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(AC_LDS(v4s, p));
    v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(AC_LDS(v4s, p + 4 * B_ROW));
    v2i l2 = __builtin_bit_cast(v2i, lo), h2 = __builtin_bit_cast(v2i, hi);
    return (v4i){l2[0], l2[1], h2[0], h2[1]};
  } else {
    v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32(AC_LDS(v2i, p));
    v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32(AC_LDS(v2i, p + 8 * B_ROW));
    return (v4i){lo[0], lo[1], hi[0], hi[1]};
  }
}
template <class T, int B_ROW>
static __device__ __forceinline__ v4i dtl_read_col(const unsigned char* Bs, int kb, int seg, int lane) {
  if constexpr (T::EB == 2) return dtl_read_col_bf16<B_ROW>(Bs, kb, seg, lane);
  else return dtl_read_col_i8<B_ROW>(Bs, kb, seg, lane);
}

// f(integral_constant<0>), f(integral_constant<1>), ...: one call per LDS stage with the stage index a constant.
template <class F, int... I>
static __device__ __forceinline__ void for_each_stage(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}

template <class T, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int KTB_>
struct DtlGeometry {
  static constexpr int EB = T::EB;
  static constexpr int KTB = KTB_;                // K bytes per A row per tile (64 or 128)
  static constexpr int BK = KTB / EB;             // K elements per tile == k-rows of the B tile
  static constexpr int KSTEPS = KTB / 32;         // MFMA K-steps per tile (32 bytes of K each)
  static constexpr int WAVES = WAVES_M * WAVES_N;
  static constexpr int THREADS = 64 * WAVES;
  static constexpr int A_BYTES = BM * KTB;
  static constexpr int A_SPR = KTB / 16;          // slots per A row
  static constexpr int A_RPW = 256 / KTB;         // A rows per 256-byte bank window
  static constexpr int A_ROWS_PER_INSTR = 64 / A_SPR;
  static constexpr int B_ROW = BN * EB;           // bytes per k-row of the B tile
  static constexpr int B_SPR = B_ROW / 16;        // slots per k-row
  static constexpr int B_BYTES = BK * B_ROW;
  static constexpr int STAGE = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = STAGES * STAGE;
  static constexpr int A_INSTR = A_BYTES / 1024 / WAVES;  // direct-to-LDS instructions per wave per tile
  static constexpr int B_INSTR = B_BYTES / 1024 / WAVES;
  static constexpr int B_ROWS_PER_INSTR = 64 / B_SPR;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(KTB == 64 || KTB == 128, "K tile is 64 or 128 bytes");
  static_assert(A_BYTES % (1024 * WAVES) == 0 && B_BYTES % (1024 * WAVES) == 0, "tile must split into whole wave loads");
  static_assert(B_SPR <= 64 && 64 % B_SPR == 0, "B row must divide a wave load");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
  // swizzle term of an A row: rows that share a 256-byte bank window get the same term
  static __device__ __forceinline__ int a_xor(int row) { return (row / A_RPW) & (A_SPR - 1); }
};

// tile_coords() (the XCD-aware tile order) without integer divisions: the band size is divided by with a
// multiplier the host supplies, the band height (1 .. 4 tile rows) by a case split.  Two divisions are some sixty
// scalar and vector instructions ahead of a kernel's first load: 0.07 us of a 4 us launch.
static __device__ __forceinline__ void tile_coords_mul(int b, int nblocks, int tiles_m, int tiles_n, unsigned band_magic, int& tm, int& tn) {
  constexpr int XCDS = 8, GROUP_M = 4;
  const int q = nblocks / XCDS, r = nblocks % XCDS;
  const int xcd = b % XCDS, idx = b / XCDS;
  const int id = xcd * q + (xcd < r ? xcd : r) + idx;
  const int group_size = GROUP_M * tiles_n;
  const int group = band_magic ? (int)__umulhi((unsigned)id, band_magic) : id / group_size;
  const int first_m = group * GROUP_M;
  const int gsz = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
  const int in_group = id - group * group_size;
  int qn;
  if (gsz == 4) qn = in_group >> 2;
  else if (gsz == 3) qn = (int)__umulhi((unsigned)in_group, 0x55555556u);  // exact below 2^31
  else if (gsz == 2) qn = in_group >> 1;
  else qn = in_group;
  tm = first_m + (in_group - qn * gsz);
  tn = qn;
}

// TA / TB (int8 GEMM on square tiles): A is given as A^T (K x M, row pitch lda) / B as B^T (N x K, row pitch ldb).
// A transposed operand takes the other operand's role in LDS: A^T is "K-strided" like B (k-rows of BM bytes, the
// B swizzle, fragments through the transposing reads), B^T is "K-contiguous" like A (rows of KTB bytes, the A
// swizzle, 16-byte fragment reads).  With BM == BN the tiles, the instruction counts and the lane roles of the two
// forms coincide, so only the source offsets, the advance per K tile and the fragment addresses differ.
template <class T, class EPI, int BM, int BN, int WAVES_M, int WAVES_N, int AMODE, int STAGES, int KTB_, bool PINGPONG, bool TA = false, bool TB = false>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) gemm_dtl_kernel(const GemmParams p, const int tiles_m, const int tiles_n, const unsigned band_magic) {
  using G = DtlGeometry<T, BM, BN, WAVES_M, WAVES_N, STAGES, KTB_>;
  constexpr int EB = G::EB;
  static_assert(!(TA || TB) || (BM == BN && AMODE == 0 && EB == 1), "transposed operands: int8 GEMM on square tiles");
  constexpr int AT_ROW = BM * EB, AT_SPR = AT_ROW / 16, AT_RPI = 64 / AT_SPR;  // A^T tile: bytes, slots per k-row, k-rows per instruction
  static_assert(!(TA || TB) || AT_ROW == G::B_ROW, "a transposed operand reuses the other operand's LDS geometry");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned lds0 = (unsigned)(uintptr_t)AC_LDS(unsigned char, smem);

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int kbytes = p.K * EB, nbytes = p.N * EB;
  const unsigned char* zero = (const unsigned char*)g_zero16;
  const int ntiles = tiles_m * tiles_n;
  const int nwork = ntiles * p.splits;

  // Cross-item prefetch (ping-pong GEMM only): a persistent workgroup requests the first STAGES-1 K tiles of its
  // next output tile before it runs the output stage of the current one, so that the pipeline fill of the next
  // tile and the drain of this tile's stores overlap.  Vector-memory operations of a wave complete in issue order,
  // so the waits of the next tile's first trips name the stores that lie between its loads.
  constexpr bool XPF = PINGPONG && AMODE == 0;
  // lower bound of the vector-memory operations one wave issues in the output stage of a FULL tile
  constexpr int EPI_VM = EPI::LDS_STAGED ? G::TM * 2 * (16 / (64 / (G::WTN / 4))) : G::TM * G::TN;
  static_assert(!XPF || (STAGES - 2) * (G::A_INSTR + G::B_INSTR) + EPI_VM <= 63, "vmcnt is a 6-bit counter");

  // ---- item-independent lane roles ---------------------------------------------------------------------
  constexpr int NVAR = G::KTB == 128 ? 2 : 1;
  int a_chunk[NVAR];
#pragma unroll
  for (int v = 0; v < NVAR; v++) a_chunk[v] = (lane % G::A_SPR) ^ G::a_xor(v * G::A_ROWS_PER_INSTR + lane / G::A_SPR);
  const int64_t b_step = (int64_t)G::BK * p.ldb * EB;
  const int64_t a_step_t = (int64_t)G::BK * p.lda * EB;  // A^T: one K tile further down
  v4i a_rsrc = {0, 0, 0, 0};  // buffer descriptor of the input image: base, size in bytes, raw dword format
  if constexpr (AMODE == 1) {
    const uint64_t ab = (uint64_t)(uintptr_t)p.A;
    a_rsrc[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)ab);
    a_rsrc[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(ab >> 32));
    a_rsrc[2] = __builtin_amdgcn_readfirstlane(p.a_bytes);
    a_rsrc[3] = 0x00020000;
  }

  // ---- state of the item whose loads are being issued: per-lane source addressing ------------------------
  // A: wave instruction j (j = wave * A_INSTR + i) fills A_ROWS_PER_INSTR tile rows; lane l -> row
  // j * A_ROWS_PER_INSTR + l / A_SPR, physical slot l % A_SPR, holding logical chunk (l % A_SPR) ^ a_xor(row).
  // The XOR term takes NVAR distinct values per lane as j varies (2 for 128-byte rows, 1 for 64-byte rows).
  // B: wave instruction j fills B_ROWS_PER_INSTR k-rows; lane l -> row j * B_ROWS_PER_INSTR + l / B_SPR,
  // physical slot l % B_SPR.
  // GEMM (AMODE 0): a wave-uniform base pointer per operand that advances by one K tile per issue, plus a
  // constant 32-bit byte offset per lane and instruction.  Rows beyond M and columns beyond N are clamped
  // to valid ones (their products land in accumulators that are never stored); only a partial last K tile
  // needs zeros and takes the slower per-lane pointer path.
  // Convolution (AMODE 1): the row's output pixel gives the byte offset of its window origin in the image
  // (g_base, possibly "negative": only ever used together with an in-range tap) and one bit per kernel tap that
  // says whether the tap falls inside the image (g_mask, bit kh * KW + kw; the host keeps KH * KW <= 32).  A
  // load then costs an add, a bit test and an OR: a lane whose tap is padding, whose row is beyond M or whose K
  // position is beyond K gets the offset 0xffffffff and the bounds check of the buffer load writes its zeros.
  // The lane's chunk sits at K byte g_kb (the K position of its chunk in the next K tile to be requested), i.e.
  // tap g_kb / Cin, channel g_kb % Cin; both come from two multiply-high divisions per K tile instead of a carried
  // (kh, kw, ci) counter with its loops.
  int split = 0, kt0 = 0, m0 = 0, n0 = 0;
  unsigned a_voff[G::A_INSTR], b_voff[G::B_INSTR];
  int b_krow[G::B_INSTR], a_krow[G::A_INSTR];
  int g_base[G::A_INSTR];
  unsigned g_mask[G::A_INSTR];
  unsigned g_kb[NVAR];
  const unsigned char* a_base = nullptr;
  const unsigned char* b_base = nullptr;

  auto setup = [&](int w) {
    split = p.splits > 1 ? w / ntiles : 0;
    const int tile = w - split * ntiles;
    kt0 = split * p.kt_per_split;  // first K tile of this slice
    int tm, tn;
    tile_coords_mul(tile, ntiles, tiles_m, tiles_n, band_magic, tm, tn);
    m0 = tm * BM, n0 = tn * BN;
#pragma unroll
    for (int i = 0; i < G::A_INSTR; i++) {
      const int row = (wave * G::A_INSTR + i) * G::A_ROWS_PER_INSTR + lane / G::A_SPR;
      const int v = (wave * G::A_INSTR + i) & (NVAR - 1);
      g_base[i] = 0, g_mask[i] = 0u, a_voff[i] = 0, a_krow[i] = 0;
      if constexpr (TA) {
        const int krow = (wave * G::A_INSTR + i) * AT_RPI + lane / AT_SPR;
        const int ls = BSwizzle<EB, AT_ROW>::slot(lane % AT_SPR, krow);
        a_krow[i] = krow;
        a_voff[i] = (unsigned)krow * (unsigned)(p.lda * EB) + ((m0 + ls * 16) * EB < p.M * EB ? ls * 16 : 0);
      } else if constexpr (AMODE == 0) {
        const int rclamp = m0 + row < p.M ? row : p.M - 1 - m0;
        a_voff[i] = (unsigned)rclamp * (unsigned)(p.lda * EB) + a_chunk[v] * 16;
      } else {
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
    }
#pragma unroll
    for (int i = 0; i < G::B_INSTR; i++) {
      if constexpr (TB) {
        const int nrow = (wave * G::B_INSTR + i) * G::A_ROWS_PER_INSTR + lane / G::A_SPR;
        const int rclamp = n0 + nrow < p.N ? nrow : p.N - 1 - n0;
        b_krow[i] = 0;
        b_voff[i] = (unsigned)rclamp * (unsigned)(p.ldb * EB) + a_chunk[(wave * G::B_INSTR + i) & (NVAR - 1)] * 16;
        continue;
      }
      const int row = (wave * G::B_INSTR + i) * G::B_ROWS_PER_INSTR + lane / G::B_SPR;
      const int ls = BSwizzle<EB, G::B_ROW>::slot(lane % G::B_SPR, row);
      b_krow[i] = row;
      b_voff[i] = (unsigned)row * (unsigned)(p.ldb * EB) + (n0 * EB + ls * 16 < nbytes ? ls * 16 : 0);
    }
    if constexpr (TA) a_base = (const unsigned char*)p.A + (int64_t)m0 * EB + kt0 * a_step_t;
    else a_base = (const unsigned char*)p.A + (AMODE == 0 ? (int64_t)m0 * p.lda * EB : 0) + (int64_t)kt0 * G::KTB;
    if constexpr (TB) b_base = (const unsigned char*)p.B + (int64_t)n0 * p.ldb * EB + (int64_t)kt0 * G::KTB;
    else b_base = (const unsigned char*)p.B + (int64_t)n0 * EB + kt0 * b_step;
#pragma unroll
    for (int v = 0; v < NVAR; v++) g_kb[v] = (unsigned)(kt0 * G::KTB + a_chunk[v] * 16);
  };

  // Tiles are issued strictly in order 0, 1, 2, ...: the running bases and tap decode rely on it.
  auto issue_loads = [&](int kt_local, int buf) {
    const unsigned As = lds0 + buf * G::STAGE;
    const unsigned Bs = As + G::A_BYTES;
    const int kt = kt0 + kt_local;
    const int kbase = kt * G::KTB;
    const bool full = kbase + G::KTB <= kbytes;  // wave-uniform
    if constexpr (AMODE == 1) {
      unsigned g_off[NVAR], g_tap[NVAR], g_dead[NVAR];
#pragma unroll
      for (int v = 0; v < NVAR; v++) {
        const unsigned tap = p.dCin.div(g_kb[v]), ci = g_kb[v] - tap * p.Cin;
        const unsigned kh = p.dKW.div(tap), kw = tap - kh * p.KW;
        g_off[v] = (kh * p.W + kw) * p.Cin + ci;
        g_tap[v] = tap;
        g_dead[v] = g_kb[v] < (unsigned)kbytes ? 0u : ~0u;
        g_kb[v] += G::KTB;
      }
#pragma unroll
      for (int i = 0; i < G::A_INSTR; i++) {
        const int v = (wave * G::A_INSTR + i) & (NVAR - 1);
        const unsigned inside = (g_mask[i] >> (g_tap[v] & 31u)) & 1u;
        buffer_to_lds16(a_rsrc, ((unsigned)g_base[i] + g_off[v]) | (inside - 1u) | g_dead[v], As + (wave * G::A_INSTR + i) * 1024);
      }
    } else if (full) {
#pragma unroll
      for (int i = 0; i < G::A_INSTR; i++) load_to_lds16_so(a_base, a_voff[i], As + (wave * G::A_INSTR + i) * 1024);
    } else if constexpr (TA) {
#pragma unroll
      for (int i = 0; i < G::A_INSTR; i++) {
        const int k = kt * G::BK + a_krow[i];
        load_to_lds16(k < p.K ? a_base + a_voff[i] : zero, As + (wave * G::A_INSTR + i) * 1024);
      }
    } else {
#pragma unroll
      for (int i = 0; i < G::A_INSTR; i++) {
        const int v = (wave * G::A_INSTR + i) & (NVAR - 1);
        const int kb = kbase + a_chunk[v] * 16;
        load_to_lds16(kb < kbytes ? a_base + a_voff[i] : zero, As + (wave * G::A_INSTR + i) * 1024);
      }
    }
    if (full) {  // every k-row of the tile exists; columns beyond N were clamped when b_voff was set up
#pragma unroll
      for (int i = 0; i < G::B_INSTR; i++) load_to_lds16_so(b_base, b_voff[i], Bs + (wave * G::B_INSTR + i) * 1024);
    } else if constexpr (TB) {
#pragma unroll
      for (int i = 0; i < G::B_INSTR; i++) {
        const int kb = kbase + a_chunk[(wave * G::B_INSTR + i) & (NVAR - 1)] * 16;
        load_to_lds16(kb < kbytes ? b_base + b_voff[i] : zero, Bs + (wave * G::B_INSTR + i) * 1024);
      }
    } else {
#pragma unroll
      for (int i = 0; i < G::B_INSTR; i++) {
        const int k = kt * G::BK + b_krow[i];
        load_to_lds16(k < p.K ? b_base + b_voff[i] : zero, Bs + (wave * G::B_INSTR + i) * 1024);
      }
    }
    a_base += TA ? a_step_t : (int64_t)G::KTB;
    b_base += TB ? (int64_t)G::KTB : b_step;
  };

  typename T::accv acc[G::TM][G::TN];

  // ---- fragments ---------------------------------------------------------------------------------------
  // the lane's A row within a 32-row MFMA tile is lane & 31; tile origins are multiples of 32 rows and do
  // not change the swizzle term
  const int a_swz = G::a_xor(lane & 31);
  const int a_lane_off = (wm * G::WTM + (lane & 31)) * G::KTB;
  const int b_lane_off_t = (wn * G::WTN + (lane & 31)) * G::KTB;  // B^T: the lane's row of the K-contiguous B tile
  struct Frag {
    v4i a[G::TM], b[G::TN];
  };
  auto read_frags = [&](int buf, int ks, Frag& f) {
    const unsigned char* As = smem + buf * G::STAGE;
    const unsigned char* Bs = As + G::A_BYTES;
    const int chunk = 2 * ks + (lane >> 5);
#pragma unroll
    for (int i = 0; i < G::TM; i++) {
      if constexpr (TA) f.a[i] = dtl_read_col<T, AT_ROW>(As, chunk * 16, wm * G::TM + i, lane);
      else f.a[i] = *(const v4i*)(As + a_lane_off + i * 32 * G::KTB + ((chunk ^ a_swz) << 4));
    }
#pragma unroll
    for (int j = 0; j < G::TN; j++) {
      if constexpr (TB) f.b[j] = *(const v4i*)(Bs + b_lane_off_t + j * 32 * G::KTB + ((chunk ^ a_swz) << 4));
      else f.b[j] = dtl_read_col<T, G::B_ROW>(Bs, chunk * 16, wn * G::TN + j, lane);
    }
  };
  auto mfma_rows = [&](const Frag& f, int i0, int i1) {  // MFMA row tiles i0 .. i1-1 of one K-step
#pragma unroll
    for (int i = i0; i < i1; i++)
#pragma unroll
      for (int j = 0; j < G::TN; j++) acc[i][j] = EPI::SWAP ? T::mfma(f.b[j], f.a[i], acc[i][j]) : T::mfma(f.a[i], f.b[j], acc[i][j]);
  };
  const int nkt_total = (kbytes + G::KTB - 1) / G::KTB;
  constexpr int PER_TILE = G::A_INSTR + G::B_INSTR;  // outstanding vector-memory ops per tile per wave
  static_assert((STAGES - 1) * PER_TILE <= 63, "vmcnt is a 6-bit counter");
  using SW = BSwizzle<EB, G::B_ROW>;
  constexpr int ROWS_PER_CHUNK = 16 / EB;  // k-rows of B that 16 bytes of K span
  static_assert(ROWS_PER_CHUNK % SW::RPW == 0 && ((ROWS_PER_CHUNK / SW::RPW) & SW::MASK) == 0, "the B swizzle term must not depend on the K-step");
  constexpr int KS_B = (32 / EB) * G::B_ROW;  // bytes between the B rows of consecutive K-steps
  // a K-contiguous operand needs one lane address per K-step (row tiles are an immediate apart), a K-strided one
  // one per 32-column block (K-steps are an immediate apart)
  constexpr int NAF = TA ? G::TM : G::KSTEPS, NBF = TB ? G::KSTEPS : G::TN;
  constexpr int KS_A = (32 / EB) * AT_ROW;  // A^T: bytes between the rows of consecutive K-steps
  int a_fo[NAF], b_fo[NBF];
#pragma unroll
  for (int x = 0; x < NAF; x++) {
    if constexpr (TA) a_fo[x] = dtl_col_off<T, AT_ROW>((lane >> 5) * 16, wm * G::TM + x, lane);
    else a_fo[x] = a_lane_off + (((2 * x + (lane >> 5)) ^ a_swz) << 4);
  }
#pragma unroll
  for (int x = 0; x < NBF; x++) {
    if constexpr (TB) b_fo[x] = G::A_BYTES + b_lane_off_t + (((2 * x + (lane >> 5)) ^ a_swz) << 4);
    else b_fo[x] = G::A_BYTES + dtl_col_off<T, G::B_ROW>((lane >> 5) * 16, wn * G::TN + x, lane);
  }
  // The immediate offset of an LDS read has 16 bits: stages that begin 64 KB or more into LDS are read through a
  // second set of lane addresses, 64 KB up (made opaque, or the compiler folds them back into one register per read).
  constexpr bool HI_STAGES = (STAGES - 1) * G::STAGE >= 65536;
  static_assert((STAGES - 1) * G::STAGE < 2 * 65536, "a third set of lane addresses would be needed");
  int a_fo_hi[NAF], b_fo_hi[NBF];
#pragma unroll
  for (int x = 0; x < NAF; x++) {
    a_fo_hi[x] = a_fo[x] + 65536;
    if constexpr (HI_STAGES) asm volatile("" : "+v"(a_fo_hi[x]));
  }
#pragma unroll
  for (int x = 0; x < NBF; x++) {
    b_fo_hi[x] = b_fo[x] + 65536;
    if constexpr (HI_STAGES) asm volatile("" : "+v"(b_fo_hi[x]));
  }
  // K slices keep the general loops; the convolution gather handles a partial last tile itself
  const int nkt_whole = p.splits > 1 ? 0 : (AMODE == 0 ? kbytes / G::KTB : nkt_total);
  auto issue_whole = [&](auto lbufc) {  // the next tile in order, a whole one, into stage LBUF
    constexpr int LBUF = decltype(lbufc)::value;
#pragma unroll
    for (int i = 0; i < G::A_INSTR; i++) load_to_lds16_so(a_base, a_voff[i], lds0 + LBUF * G::STAGE + (wave * G::A_INSTR + i) * 1024);
#pragma unroll
    for (int i = 0; i < G::B_INSTR; i++) load_to_lds16_so(b_base, b_voff[i], lds0 + LBUF * G::STAGE + G::A_BYTES + (wave * G::B_INSTR + i) * 1024);
    a_base += TA ? a_step_t : (int64_t)G::KTB;
    b_base += TB ? (int64_t)G::KTB : b_step;
  };
  auto issue_whole_rt = [&](int lbuf) {  // the same with the stage as a value (constant after unrolling)
#pragma unroll
    for (int i = 0; i < G::A_INSTR; i++) load_to_lds16_so(a_base, a_voff[i], lds0 + lbuf * G::STAGE + (wave * G::A_INSTR + i) * 1024);
#pragma unroll
    for (int i = 0; i < G::B_INSTR; i++) load_to_lds16_so(b_base, b_voff[i], lds0 + lbuf * G::STAGE + G::A_BYTES + (wave * G::B_INSTR + i) * 1024);
    a_base += TA ? a_step_t : (int64_t)G::KTB;
    b_base += TB ? (int64_t)G::KTB : b_step;
  };
  auto read_frags_at = [&](auto bufc, int ks, Frag& f) {  // read_frags with the stage as a constant
    constexpr int BUF = decltype(bufc)::value;
    constexpr bool HI = BUF * G::STAGE >= 65536;
    constexpr int SOFF = BUF * G::STAGE - (HI ? 65536 : 0);
#pragma unroll
    for (int i = 0; i < G::TM; i++) {
      if constexpr (TA) f.a[i] = dtl_read_col_at<T, AT_ROW>(smem + ((HI ? a_fo_hi[i] : a_fo[i]) + (SOFF + ks * KS_A)));
      else f.a[i] = *(const v4i*)(smem + ((HI ? a_fo_hi[ks] : a_fo[ks]) + (SOFF + i * 32 * G::KTB)));
    }
#pragma unroll
    for (int j = 0; j < G::TN; j++) {
      if constexpr (TB) f.b[j] = *(const v4i*)(smem + ((HI ? b_fo_hi[ks] : b_fo[ks]) + (SOFF + j * 32 * G::KTB)));
      else f.b[j] = dtl_read_col_at<T, G::B_ROW>(smem + ((HI ? b_fo_hi[j] : b_fo[j]) + (SOFF + ks * KS_B)));
    }
  };

  // Persistent workgroups: each takes output tiles blockIdx.x, blockIdx.x + gridDim.x, ...  gridDim.x is a multiple
  // of the number of XCDs (or equals ntiles), so a workgroup's tiles all map to its own XCD in tile_coords().
  // With split-K a work item is (tile, K slice): slice s covers K tiles s * kt_per_split ...
  // The launcher never starts more workgroups than work items, so the first pass needs no test.
  int work = blockIdx.x;
  bool started = false;  // the item's addressing is set up and its first STAGES-1 tiles are requested
  bool pf_stores = false;  // ... and EPI_VM stores of a full tile were issued after those requests
  do {
  if (!started) setup(work);
  const int nkt = p.splits > 1 ? (nkt_total - kt0 < p.kt_per_split ? nkt_total - kt0 : p.kt_per_split) : nkt_total;

#pragma unroll
  for (int i = 0; i < G::TM; i++)
#pragma unroll
    for (int j = 0; j < G::TN; j++) acc[i][j] = T::zero();

  // operands of the output stage that do not depend on the product (bias) are requested before the K loop
  typename EPI::Pre pre[G::TN];
#pragma unroll
  for (int j = 0; j < G::TN; j++) EPI::prefetch(p, n0 + wn * G::WTN + j * 32, lane, pre[j]);

  if constexpr (PINGPONG) {
    // ---- ping-pong main loop ---------------------------------------------------------------------------
    // Eight waves, two per SIMD, in two groups of four (one wave of each group on every SIMD).  A wave
    // alternates between a memory phase (issue its share of the direct-to-LDS loads for a later tile, read
    // all fragments of the current tile into registers) and a compute phase (all MFMAs of that tile), with a
    // workgroup barrier after each phase.  Group 1 is held back by one phase, so at any time one wave per
    // SIMD is feeding the matrix pipe while the other fetches:
    //   phase 2t   : group 0 reads tile t      | group 1 computes tile t-1
    //   phase 2t+1 : group 0 computes tile t   | group 1 reads tile t
    // Tile t sits in stage t % STAGES.  In its memory phase of tile t a wave issues the loads of tile
    // t + STAGES - 1 (into the stage of tile t - 1, whose last reader finished one phase earlier) and waits
    // until its own loads of tile t + 1 have landed; the barrier that ends phase 2t+1 therefore publishes tile
    // t + 1 completely before phase 2t+2 reads it.
    static_assert(!PINGPONG || G::WAVES == 8, "ping-pong needs two waves per SIMD");
    static_assert(!PINGPONG || STAGES >= 3, "ping-pong needs at least three LDS stages");
    const int grp = wave >> 2;
    Frag fr[G::KSTEPS];
    if (!started) {
#pragma unroll
      for (int s = 0; s < STAGES - 1; s++)
        if (s < nkt) issue_loads(s, s);
    }
    // tile 0 has landed: the younger tiles (and, after a prefetch, the stores behind them) may still be in flight
    if (XPF && started && pf_stores) wait_vm<(STAGES - 2) * PER_TILE + (XPF ? EPI_VM : 0)>();
    else if (STAGES - 2 < nkt) wait_vm<(STAGES - 2) * PER_TILE>();
    else wait_vm<0>();
    block_sync();                  // tile 0 is visible
    if (grp == 1) block_sync();    // hold group 1 back by one phase
    int buf = 0;
    int kt = 0;
    {
      auto trip = [&](auto bufc, auto extrac) {
        constexpr int BUF = decltype(bufc)::value, LBUF = (BUF + STAGES - 1) % STAGES;
        if constexpr (AMODE == 0) issue_whole(std::integral_constant<int, LBUF>{});
        else issue_loads(kt + BUF + STAGES - 1, LBUF);  // the gather keeps its per-lane addressing; kt is a multiple of STAGES here
#pragma unroll
        for (int ks = 0; ks < G::KSTEPS; ks++) read_frags_at(bufc, ks, fr[ks]);
        wait_vm<(STAGES - 2) * PER_TILE + decltype(extrac)::value>();
        block_sync();
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < G::KSTEPS; ks++) mfma_rows(fr[ks], 0, G::TM);
        __builtin_amdgcn_s_setprio(0);
        block_sync();
      };
      if constexpr (XPF) {
        // first round after a prefetch across full-tile stores: the loads that trips 0 .. STAGES-3 wait for are
        // older than those stores, so their waits name them instead of draining them
        if (started && pf_stores && kt + 2 * STAGES - 2 < nkt_whole && kt + 2 * STAGES - 2 < nkt) {
          for_each_stage([&](auto bc) {
            if constexpr (decltype(bc)::value < STAGES - 2) trip(bc, std::integral_constant<int, EPI_VM>{});
            else trip(bc, std::integral_constant<int, 0>{});
          }, std::make_integer_sequence<int, STAGES>{});
          kt += STAGES;
        }
      }
      // tiles kt + STAGES - 1 .. kt + 2 STAGES - 2, the ones a round of trips requests, are whole
      for (; kt + 2 * STAGES - 2 < nkt_whole && kt + 2 * STAGES - 2 < nkt; kt += STAGES)
        for_each_stage([&](auto bc) { trip(bc, std::integral_constant<int, 0>{}); }, std::make_integer_sequence<int, STAGES>{});
    }
    for (; kt < nkt; kt++) {
      // memory phase
      const int lbuf = buf == 0 ? STAGES - 1 : buf - 1;  // stage of tile kt - 1 == stage of tile kt + STAGES - 1
      if (kt + STAGES - 1 < nkt) issue_loads(kt + STAGES - 1, lbuf);
#pragma unroll
      for (int ks = 0; ks < G::KSTEPS; ks++) read_frags(buf, ks, fr[ks]);
      if (kt + STAGES - 1 < nkt) wait_vm<(STAGES - 2) * PER_TILE>();
      else wait_vm<0>();
      block_sync();
      // compute phase
      __builtin_amdgcn_s_setprio(1);
#pragma unroll
      for (int ks = 0; ks < G::KSTEPS; ks++) mfma_rows(fr[ks], 0, G::TM);
      __builtin_amdgcn_s_setprio(0);
      block_sync();
      buf = buf + 1 == STAGES ? 0 : buf + 1;
    }
    if (grp == 0) block_sync();    // every wave executes the same number of barriers
  } else {
  // Tile t lives in LDS stage t % STAGES.  One fragment set per K-step of a tile stays in registers; as soon
  // as the MFMAs of K-step s of tile kt are issued, the set is refilled with K-step s of tile kt + 1, so an LDS
  // read has the MFMAs of the other K-steps of a tile to land in (with a fragment double buffer per K-step it
  // had one K-step, less than the LDS latency on the small tiles).  One barrier per tile, at the top: past it
  // every wave has received its fragments of tile kt (block_sync waits for the wave's own LDS reads), so the
  // stage of tile kt can take tile kt + STAGES, and tile kt + 1 is visible to everyone.
  Frag fr[G::KSTEPS];
#pragma unroll
  for (int s = 0; s < STAGES; s++)
    if (s < nkt) issue_loads(s, s);
  if (nkt > 0) {
    if (STAGES - 1 < nkt) wait_vm<(STAGES - 1) * PER_TILE>();
    else wait_vm<0>();
    block_sync();
#pragma unroll
    for (int ks = 0; ks < G::KSTEPS; ks++) read_frags(0, ks, fr[ks]);
  }
  int buf = 0;
  int kt = 0;
  {
    auto roll = [&](auto bufc) {
      constexpr int BUF = decltype(bufc)::value;
      wait_vm<(STAGES - 2) * PER_TILE>();
      block_sync();
      if constexpr (AMODE == 0) issue_whole(bufc);  // tile kt + STAGES takes the stage that tile kt has just left
      else issue_loads(kt + BUF + STAGES, BUF);
#pragma unroll
      for (int ks = 0; ks < G::KSTEPS; ks++) {
        mfma_rows(fr[ks], 0, G::TM);
        __builtin_amdgcn_sched_barrier(0);
        read_frags_at(std::integral_constant<int, (BUF + 1) % STAGES>{}, ks, fr[ks]);
      }
    };

    const int lim = nkt < nkt_whole ? nkt : nkt_whole;
    for (; kt + 2 * STAGES - 1 < lim; kt += STAGES) {  // tiles kt + STAGES .. kt + 2 STAGES - 1 are whole
      for_each_stage(roll, std::make_integer_sequence<int, STAGES>{});
    }
  }
  for (; kt + 1 < nkt; kt++) {  // every tile but the last
    const int nbuf = buf + 1 == STAGES ? 0 : buf + 1;
    // tile kt + 1 must have landed: only the (STAGES - 2) younger tiles may still be in flight
    if (kt + STAGES - 1 < nkt) wait_vm<(STAGES - 2) * PER_TILE>();
    else wait_vm<0>();
    block_sync();
    if (kt + STAGES < nkt) issue_loads(kt + STAGES, buf);
#pragma unroll
    for (int ks = 0; ks < G::KSTEPS; ks++) {
      mfma_rows(fr[ks], 0, G::TM);
      __builtin_amdgcn_sched_barrier(0);  // keep the refill behind the MFMAs that still read the old fragments
      read_frags(nbuf, ks, fr[ks]);
    }
    buf = nbuf;
  }
  if (nkt > 0) {  // last tile
#pragma unroll
    for (int ks = 0; ks < G::KSTEPS; ks++) mfma_rows(fr[ks], 0, G::TM);
  }
  }

  // ---- output stage of the finished item; with XPF the next item's first tiles are requested ahead of it ----
  const int em0 = m0, en0 = n0, esplit = split;
  const bool efull = em0 + BM <= p.M && en0 + BN <= p.N;  // wave-uniform: no store of this tile is masked
  started = false;
  if constexpr (XPF) {
    // every item of a launch has the same K range here (no K slices); the fill needs STAGES - 1 whole tiles
    if (work + (int)gridDim.x < nwork && p.splits == 1 && nkt_whole >= STAGES - 1) {
      block_sync();  // every wave has read its last fragments: stages 0 .. STAGES-2 can take the next item's tiles
      setup(work + (int)gridDim.x);
#pragma unroll
      for (int s = 0; s < STAGES - 1; s++) issue_whole_rt(s);
      started = true;
      pf_stores = efull;
    }
  }
  if constexpr (EPI::LDS_STAGED) {
    // 4-byte outputs through LDS: the accumulator layout gives a lane one column of many rows, so straight
    // stores are dwords (one 128-byte row segment per half-wave and instruction, 128 instructions per wave for
    // a 64 x 128 wave tile, each about as slow to issue as a 16-byte one).  Every wave instead transposes 16
    // rows of its tile at a time through a private LDS region and stores 16 bytes per lane, whole 128-byte lines
    // per 8 lanes.  With XPF the region lies in the last LDS stage, which the next item does not fill before its
    // first trip: row pitch WTN values with the two half-rows exchanged in rows 4..7 and 12..15, so that the two
    // half-waves, four rows apart, still hit different banks.  Otherwise: row pitch WTN + 8 from the LDS base.
    using SV = typename EPI::StagedValue;
    typedef SV sv4 __attribute__((ext_vector_type(4)));
    constexpr int PITCH = XPF ? G::WTN : G::WTN + 8;
    constexpr int LPR = G::WTN / 4, RPI = 64 / LPR, NI = 16 / RPI;  // lanes per row, rows per instruction, instructions per 16 rows
    static_assert(G::WAVES * 16 * PITCH * 4 <= (XPF ? G::STAGE : G::LDS_BYTES) && 64 % LPR == 0 && 16 % RPI == 0 && sizeof(SV) == 4, "staging region");
    static_assert(!XPF || (G::WTN % 64 == 0), "the half-row exchange needs rows of whole 32-value halves");
    if (!started) block_sync();  // every wave has read its last fragments: the stages are free
    SV* region = (SV*)(smem + (XPF ? (STAGES - 1) * G::STAGE : 0)) + wave * (16 * PITCH);
    const int h = lane >> 5, c = lane & 31;
    auto body = [&](auto fullc) {
#pragma unroll
    for (int i = 0; i < G::TM; i++) {
#pragma unroll
      for (int hf = 0; hf < 2; hf++) {
#pragma unroll
        for (int j = 0; j < G::TN; j++)
#pragma unroll
          for (int rr = 0; rr < 8; rr++) {
            const int row = 8 * (rr / 4) + 4 * h + rr % 4;
            const int col = XPF ? ((32 * j + c) ^ (h << 5)) : 32 * j + c;  // rows 4 h + ... have bit 2 == h
            region[row * PITCH + col] = EPI::staged_in(p, acc[i][j][hf * 8 + rr]);
          }
#pragma unroll
        for (int q = 0; q < NI; q++) {
          const int row = q * RPI + lane / LPR, col = (lane % LPR) * 4;
          const int pcol = XPF ? (col ^ (((row >> 2) & 1) << 5)) : col;
          const sv4 o = *(const sv4*)(region + row * PITCH + pcol);
          const int m = em0 + wm * G::WTM + i * 32 + hf * 16 + row, n = en0 + wn * G::WTN + col;
          // N is a multiple of 4 on this path: a group of four columns is inside or outside
          if (decltype(fullc)::value || (m < p.M && n < p.N)) EPI::staged_out(p, m, n, o, esplit);
        }
      }
    }
    };
    if (XPF && efull) body(std::true_type{});
    else body(std::false_type{});
  } else if constexpr (has_wave_tile<EPI>::value) {
    EPI::wave_tile(p, em0 + wm * G::WTM, en0 + wn * G::WTN, acc, lane, esplit, pre);
  } else {
#pragma unroll
  for (int i = 0; i < G::TM; i++) {
    const int mrow0 = em0 + wm * G::WTM + i * 32;
#pragma unroll
    for (int j = 0; j < G::TN; j++) EPI::tile(p, mrow0, en0 + wn * G::WTN + j * 32, acc[i][j], lane, esplit, pre[j]);
  }
  }
  block_sync();  // all LDS reads of this tile are done before the next tile refills the LDS stages
  } while ((work += gridDim.x) < nwork);  // tile loop
}

template <class T, class EPI, int BM, int BN, int WAVES_M, int WAVES_N, int AMODE, int STAGES, int KTB_ = 128, bool PINGPONG = false, bool TA = false, bool TB = false>
static hipError_t launch_dtl(const GemmParams& p, hipStream_t stream) {
  using G = DtlGeometry<T, BM, BN, WAVES_M, WAVES_N, STAGES, KTB_>;
  auto kern = gemm_dtl_kernel<T, EPI, BM, BN, WAVES_M, WAVES_N, AMODE, STAGES, KTB_, PINGPONG, TA, TB>;
  static std::atomic<bool> configured{G::LDS_BYTES <= 64 * 1024};
  if (const hipError_t e = allow_dynamic_lds_once(configured, kern, G::LDS_BYTES)) return e;
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const int ntiles = tiles_m * tiles_n;
  // one persistent workgroup per LDS-limited slot of every compute unit
  constexpr int per_cu = (160 * 1024) / (G::LDS_BYTES > 0 ? G::LDS_BYTES : 1);
  int slots = compute_units() * (per_cu < 1 ? 1 : (per_cu > 8 ? 8 : per_cu));
  slots -= slots % 8;
  if (slots < 8) slots = 8;  // fewer than eight compute units: still a grid, the tile order is a bijection for any size
  const int64_t nwork = (int64_t)ntiles * (p.splits > 1 ? p.splits : 1);
  if (nwork > INT32_MAX) return hipErrorInvalidValue;  // the kernel counts (tile, K slice) items in 32 bits
  const int grid = nwork < slots ? (int)nwork : slots;
  // multiplier for the division by the band size of the tile order (0: too many tiles for it, divide)
  const unsigned band = 4u * (unsigned)tiles_n;
  const unsigned band_magic = (uint64_t)ntiles * band < (1ull << 32) ? FastDiv::make(band).magic : 0u;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(G::THREADS), G::LDS_BYTES, stream, p, tiles_m, tiles_n, band_magic);
  return hipGetLastError();
}

// The four direct-to-LDS configurations by tile code.  256: eight waves in ping-pong over four 32 KB stages
// (64 bytes of K per tile; a fifth stage, all of LDS, measured 0.3-1.5 % slower on every large GEMM); 192 (256 x 128), 128 and 64: the rolling-refill loop with 128 bytes of K per tile,
// eight waves of 64 x 64 / 64 x 32 or four waves of 32 x 32 (four stages: six and eight were measured slower on
// every few-tile deep-K shape, 7.9 / 8.3 / 9.3 us on 49 x 2048 x 4608: those loops wait on the barrier, not on loads).
template <class T, class EPI, int AMODE>
static hipError_t launch_dtl_tile(int tile, const GemmParams& p, hipStream_t stream) {
  switch (tile) {
    case 256: return launch_dtl<T, EPI, 256, 256, 2, 4, AMODE, 4, 64, true>(p, stream);
    case 192: return launch_dtl<T, EPI, 256, 128, 4, 2, AMODE, 3, 128>(p, stream);
    case 128: return launch_dtl<T, EPI, 128, 128, 2, 4, AMODE, 3, 128>(p, stream);
    default: return launch_dtl<T, EPI, 64, 64, 2, 2, AMODE, 4, 128>(p, stream);
  }
}

}  // namespace ac
