// Batched small fp32 linear algebra: C_b = A_b . B_b, y_b = C_b . x_b + d_b.
//
// The work is bound by HBM traffic (2 flop per byte), so the kernel is a
// streaming one: a workgroup brings G consecutive items into LDS with fully
// coalesced 16-byte loads, 16 lanes then own one item as a 4 x 4 grid of small
// register blocks of C, the matrix-vector partial sums are combined across the 4
// lanes of a quad with DPP shuffles, and C goes back out through LDS so that the
// stores are coalesced as well.
#include "common.hpp"


namespace ac {

static __device__ __forceinline__ float quad_xor1(float v) {  // lane ^ 1 within a quad
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
}
static __device__ __forceinline__ float quad_xor2(float v) {  // lane ^ 2 within a quad
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
}

// Coalesced copy of `count` floats global -> LDS (VEC: 16-byte granules where whole).
template <bool VEC>
static __device__ __forceinline__ void copy_in(float* dst, const float* src, int count, int t) {
  if (VEC) {
    for (int i = t * 4; i < count; i += 256 * 4) {
      if (i + 3 < count) {
        *(v4f*)(dst + i) = *(const v4f*)(src + i);
      } else {
        for (int e = 0; i + e < count; e++) dst[i + e] = src[i + e];
      }
    }
  } else {
    for (int i = t; i < count; i += 256) dst[i] = src[i];
  }
}

template <bool VEC>
static __device__ __forceinline__ void copy_out(float* dst, const float* src, int count, int t) {
  if (VEC) {
    for (int i = t * 4; i < count; i += 256 * 4) {
      if (i + 3 < count) {
        *(v4f*)(dst + i) = *(const v4f*)(src + i);
      } else {
        for (int e = 0; i + e < count; e++) dst[i + e] = src[i + e];
      }
    }
  } else {
    for (int i = t; i < count; i += 256) dst[i] = src[i];
  }
}

// NFIX > 0: n is the compile-time constant NFIX.  NFIX == 0: n = p.n at run time (1..16).
// G items per workgroup (multiple of 16).  VEC: all pointers are 16-byte aligned.
template <int NFIX, int G, bool VEC>
__global__ void __launch_bounds__(256) batched_f32_kernel(const BatchedParams p) {
  extern __shared__ __attribute__((aligned(16))) float lds_f[];
  const int n = NFIX ? NFIX : p.n;
  const int nn = n * n;
  constexpr int RB = NFIX ? (NFIX + 3) / 4 : 4;  // register block edge: the 4 x 4 lane grid covers 4*RB >= n
  float* As = lds_f;          // [G][n][n]; reused for C on the way out
  float* Bs = As + G * nn;    // [G][n][n]
  float* xs = Bs + G * nn;    // [G][n]
  float* ds = xs + G * n;     // [G][n]

  const int t = threadIdx.x;
  const int64_t b0 = (int64_t)blockIdx.x * G;
  const int64_t left = p.batch - b0;
  const int cnt = left < G ? (int)left : G;

  copy_in<VEC>(As, p.A + b0 * nn, cnt * nn, t);
  copy_in<VEC>(Bs, p.B + b0 * nn, cnt * nn, t);
  if (p.x) copy_in<VEC>(xs, p.x + b0 * n, cnt * n, t);
  if (p.x && p.d) copy_in<VEC>(ds, p.d + b0 * n, cnt * n, t);
  __syncthreads();

  const int sub = t & 15;           // lane within the item's 4 x 4 grid
  const int bi = sub >> 2, bj = sub & 3;
  const int r0 = bi * RB, c0 = bj * RB;
#pragma unroll 1
  for (int item = t >> 4; item < G; item += 16) {
    if (item < cnt) {
      const float* Ai = As + item * nn;
      const float* Bi = Bs + item * nn;
      float c[RB][RB];
#pragma unroll
      for (int i = 0; i < RB; i++)
#pragma unroll
        for (int j = 0; j < RB; j++) c[i][j] = 0.f;
#pragma unroll 4
      for (int k = 0; k < n; k++) {
        float a[RB], b[RB];
#pragma unroll
        for (int i = 0; i < RB; i++) a[i] = (NFIX || r0 + i < n) ? Ai[(r0 + i) * n + k] : 0.f;
#pragma unroll
        for (int j = 0; j < RB; j++) b[j] = (NFIX || c0 + j < n) ? Bi[k * n + c0 + j] : 0.f;
#pragma unroll
        for (int i = 0; i < RB; i++)
#pragma unroll
          for (int j = 0; j < RB; j++) c[i][j] = __builtin_fmaf(a[i], b[j], c[i][j]);
      }
      if (p.x) {
        float xv[RB];
#pragma unroll
        for (int j = 0; j < RB; j++) xv[j] = (NFIX || c0 + j < n) ? xs[item * n + c0 + j] : 0.f;
#pragma unroll
        for (int i = 0; i < RB; i++) {
          float s = 0.f;
#pragma unroll
          for (int j = 0; j < RB; j++) s = __builtin_fmaf(c[i][j], xv[j], s);
          s += quad_xor1(s);  // sum over the 4 column blocks of this row
          s += quad_xor2(s);
          if (bj == 0 && (NFIX || r0 + i < n)) {
            float dv = p.d ? ds[item * n + r0 + i] : 0.f;
            p.y[(b0 + item) * n + r0 + i] = s + dv;
          }
        }
      }
      if (p.C) {
        // all 16 lanes of this item sit in one wavefront and have finished reading Ai
        float* Ci = As + item * nn;
#pragma unroll
        for (int i = 0; i < RB; i++)
#pragma unroll
          for (int j = 0; j < RB; j++)
            if (NFIX || (r0 + i < n && c0 + j < n)) Ci[(r0 + i) * n + c0 + j] = c[i][j];
      }
    }
  }
  if (p.C) {
    __syncthreads();
    copy_out<VEC>(p.C + b0 * nn, As, cnt * nn, t);
  }
}

// ---- 12 x 12 streaming kernel -----------------------------------------------------------------------------
// Each wavefront works alone (no workgroup barrier anywhere): it walks over groups of 4 consecutive items,
// brings a group's A, B, x, d into its private LDS window with direct-to-LDS loads (three windows, the next two
// groups are in flight while the current one is computed), and stores C and y straight from registers.
// 16 lanes own one item: lane (bi, bj) holds rows 3bi..3bi+2 and columns 4bj..4bj+3 of C (bj == 3 idles in the
// product but takes part in the quad reduction), so every store is a whole 16-byte chunk of a C row.
#define AC_LDS3(T, p) ((__attribute__((address_space(3))) T*)(p))
constexpr int B12_ITEM = 12 * 12 * 4;            // bytes of one matrix
constexpr int B12_GROUP = 4;                     // items per wave step
constexpr int B12_MAT = B12_GROUP * B12_ITEM;    // 2304 bytes of A (or B) per group
constexpr int B12_VEC = B12_GROUP * 48;          // 192 bytes of x (or d) per group
constexpr int B12_WIN = 2 * B12_MAT + 2 * B12_VEC + 128;  // one LDS window (5120 bytes)
constexpr int B12_WAVES = 4;                     // waves per workgroup

// Every input byte is read exactly once: the loads carry the non-temporal hint, so that the stream does not claim
// cache lines (the memory-side cache then holds the kernel's output and its neighbours' instead of dead inputs).
static __device__ __forceinline__ void b12_dma(const void* g, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds), "v"(g) : "memory");
}

// The stores of a step are written as instructions as well: the waits below count the vector-memory operations
// between a group's loads and the point of the wait, so that number has to be a property of the source, not of
// how the compiler happens to split or merge stores.  (A store wider than 8 bytes needs wait states before its
// data registers may be overwritten; the compiler pads its own stores and cannot see into the assembly.)
typedef float b12_v3f __attribute__((ext_vector_type(3)));
static __device__ __forceinline__ void b12_store16(float* g, v4f v) {
  asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 1" ::"v"(g), "v"(v) : "memory");
}
static __device__ __forceinline__ void b12_store12(float* g, b12_v3f v) {
  asm volatile("global_store_dwordx3 %0, %1, off\n\ts_nop 1" ::"v"(g), "v"(v) : "memory");
}

__global__ void __launch_bounds__(64 * B12_WAVES) batched12_stream_kernel(const BatchedParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_b[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  unsigned char* win0 = lds_b + wave * 3 * B12_WIN;
  const unsigned win0_addr = (unsigned)(uintptr_t)AC_LDS3(unsigned char, win0);
  const int64_t ngroups = (p.batch + B12_GROUP - 1) / B12_GROUP;
  const int64_t stride = (int64_t)gridDim.x * B12_WAVES;
  const bool has_x = p.x != nullptr, has_d = p.d != nullptr;

  auto issue = [&](int64_t g, int w) {  // group g -> window w
    const unsigned base = win0_addr + w * B12_WIN;
    const int64_t left = p.batch - g * B12_GROUP;
    const int items = left < B12_GROUP ? (int)left : B12_GROUP;
    const int mat_bytes = items * B12_ITEM, vec_bytes = items * 48;
    const unsigned char* Ag = (const unsigned char*)p.A + g * B12_MAT;
    const unsigned char* Bg = (const unsigned char*)p.B + g * B12_MAT;
#pragma unroll
    for (int j = 0; j < 3; j++) {
      const int off = j * 1024 + lane * 16;
      if (off < mat_bytes) {
        b12_dma(Ag + off, base + j * 1024);
        b12_dma(Bg + off, base + B12_MAT + j * 1024);
      }
    }
    if (has_x && lane * 16 < vec_bytes) b12_dma((const unsigned char*)p.x + g * B12_VEC + lane * 16, base + 2 * B12_MAT);
    if (has_d && lane * 16 < vec_bytes) b12_dma((const unsigned char*)p.d + g * B12_VEC + lane * 16, base + 2 * B12_MAT + B12_VEC);
  };

  const int it = lane >> 4, sub = lane & 15, bi = sub >> 2, bj = sub & 3;
  const int cb = bj < 3 ? bj : 2;  // idle lanes shadow column block 2
  // Three windows in rotation: while group g is computed, groups g + stride and g + 2 stride are in flight.
  // Vector-memory operations of a wave complete in issue order, loads and stores alike, so the wait at the end of
  // a step names how many younger operations may still be pending instead of draining everything: the loads of
  // the next group are followed by the stores of the previous step, the loads of the group after, and the stores
  // of this step.  Waiting for the stores themselves would put a write round trip into every step.
  // A full group issues 8 loads (3 + 3 for A and B, x, d) and the step 3 + 1 stores (C rows, y), every one of them
  // an instruction written out above; any other case (a partial last group, absent operands) takes the plain wait
  // for everything.
  constexpr int LOADS = 8, STORES = 4;
  const bool counted = has_x && has_d && p.C != nullptr;
  int64_t g = (int64_t)blockIdx.x * B12_WAVES + wave;
  int w = 0;
  bool first = true;
  if (g < ngroups) issue(g, 0);
  if (g + stride < ngroups) issue(g + stride, 1);
  if (counted && (g + stride + 1) * B12_GROUP <= p.batch) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS) : "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  for (; g < ngroups; g += stride) {
    const int64_t gn = g + 2 * stride;
    const int w2 = w >= 1 ? w - 1 : 2;  // window of group g + 2 stride == window of group g - stride
    if (gn < ngroups) issue(gn, w2);
    const int64_t item = g * B12_GROUP + it;
    if (item < p.batch) {
      const unsigned char* Wn = win0 + w * B12_WIN;
      const float* Ai = (const float*)(Wn + it * B12_ITEM) + 3 * bi * 12;
      const float* Bi = (const float*)(Wn + B12_MAT + it * B12_ITEM) + 4 * cb;
      v4f a[3][3];
#pragma unroll
      for (int i = 0; i < 3; i++)
#pragma unroll
        for (int q = 0; q < 3; q++) a[i][q] = *(const v4f*)(Ai + i * 12 + q * 4);
      v4f c[3] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
      for (int k = 0; k < 12; k++) {
        const v4f b = *(const v4f*)(Bi + k * 12);
#pragma unroll
        for (int i = 0; i < 3; i++) {
          const float av = a[i][k >> 2][k & 3];
#pragma unroll
          for (int e = 0; e < 4; e++) c[i][e] = __builtin_fmaf(av, b[e], c[i][e]);
        }
      }
      if (p.C && bj < 3) {
        float* Cg = p.C + item * 144 + 3 * bi * 12 + 4 * bj;
#pragma unroll
        for (int i = 0; i < 3; i++) b12_store16(Cg + i * 12, c[i]);  // three store instructions
      }
      if (has_x) {
        const v4f xv = *(const v4f*)((const float*)(Wn + 2 * B12_MAT + it * 48) + 4 * cb);
        float s[3];
#pragma unroll
        for (int i = 0; i < 3; i++) {
          float t = 0.f;
#pragma unroll
          for (int e = 0; e < 4; e++) t = __builtin_fmaf(c[i][e], xv[e], t);
          t = bj < 3 ? t : 0.f;
          t += quad_xor1(t);
          t += quad_xor2(t);
          s[i] = t;
        }
        if (bj == 0) {
          const float* dv = (const float*)(Wn + 2 * B12_MAT + B12_VEC + it * 48) + 3 * bi;
          const b12_v3f yv = {s[0] + (has_d ? dv[0] : 0.f), s[1] + (has_d ? dv[1] : 0.f), s[2] + (has_d ? dv[2] : 0.f)};
          b12_store12(p.y + item * 12 + 3 * bi, yv);  // one store instruction
        }
      }
    }
    // the next group's loads must have landed; every LDS read of this window has been consumed above
    if (counted && (gn + 1) * B12_GROUP <= p.batch) {
      if (first) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(LOADS + STORES) : "memory");  // no earlier step, no earlier stores
      else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(STORES + LOADS + STORES) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    }
    first = false;
    w = w == 2 ? 0 : w + 1;
  }
}

hipError_t launch_batched_f32(const BatchedParams& p, hipStream_t stream) {
  auto al = [](const void* q) { return q == nullptr || ((uintptr_t)q & 15) == 0; };
  const bool vec = al(p.A) && al(p.B) && al(p.C) && al(p.x) && al(p.d);
  const int n = p.n;
  if (n == 12 && vec) {
    // streaming kernel: one persistent workgroup of B12_WAVES waves per CU, each wave walking over groups of
    // B12_GROUP items through its own three LDS windows.  More waves per CU were measured slower (4 waves
    // 88 us, 5: 97, 6: 97, 8: 96 for 262144 items; 2 waves: 122): past 4 waves the extra requests in flight only
    // spread the six streams over more DRAM pages.
    constexpr int WGS_PER_CU = 1;
    const int cus = compute_units();
    const int64_t ngroups = (p.batch + B12_GROUP - 1) / B12_GROUP;
    int64_t wgs = (ngroups + B12_WAVES - 1) / B12_WAVES;
    if (wgs > (int64_t)cus * WGS_PER_CU) wgs = (int64_t)cus * WGS_PER_CU;
    hipLaunchKernelGGL(batched12_stream_kernel, dim3((unsigned)wgs), dim3(64 * B12_WAVES), B12_WAVES * 3 * B12_WIN, stream, p);
    return hipGetLastError();
  }
  // LDS-staged kernel: 32 items per workgroup for unaligned 12 x 12 operands (39 KB of LDS), 16 for other n
  const int G = n == 12 ? 32 : 16;
  const size_t lds = (size_t)G * (2 * n * n + 2 * n) * sizeof(float);
  const int64_t blocks = (p.batch + G - 1) / G;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks), block(256);
  if (n == 12) {
    hipLaunchKernelGGL((batched_f32_kernel<12, 32, false>), grid, block, lds, stream, p);
  } else {
    if (vec) hipLaunchKernelGGL((batched_f32_kernel<0, 16, true>), grid, block, lds, stream, p);
    else hipLaunchKernelGGL((batched_f32_kernel<0, 16, false>), grid, block, lds, stream, p);
  }
  return hipGetLastError();
}

}  // namespace ac
