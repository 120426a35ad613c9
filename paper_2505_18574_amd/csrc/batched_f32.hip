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

hipError_t launch_batched_f32(const BatchedParams& p, hipStream_t stream) {
  auto al = [](const void* q) { return q == nullptr || ((uintptr_t)q & 15) == 0; };
  const bool vec = al(p.A) && al(p.B) && al(p.C) && al(p.x) && al(p.d);
  const int n = p.n;
  // items per workgroup: 32 for the 12 x 12 case (39 KB of LDS, 4 workgroups per CU), 16 otherwise
  const int G = n == 12 ? 32 : 16;
  const size_t lds = (size_t)G * (2 * n * n + 2 * n) * sizeof(float);
  const int64_t blocks = (p.batch + G - 1) / G;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks), block(256);
  if (n == 12) {
    if (vec) hipLaunchKernelGGL((batched_f32_kernel<12, 32, true>), grid, block, lds, stream, p);
    else hipLaunchKernelGGL((batched_f32_kernel<12, 32, false>), grid, block, lds, stream, p);
  } else {
    if (vec) hipLaunchKernelGGL((batched_f32_kernel<0, 16, true>), grid, block, lds, stream, p);
    else hipLaunchKernelGGL((batched_f32_kernel<0, 16, false>), grid, block, lds, stream, p);
  }
  return hipGetLastError();
}

}  // namespace ac
