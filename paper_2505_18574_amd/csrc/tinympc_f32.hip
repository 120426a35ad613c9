// Forward pass of the TinyMPC primal update, batched over independent problems:
//   u[i]   = -Kinf . x[i] - d[i]
//   x[i+1] =  Adyn . x[i] + Bdyn . u[i]        i = 0 .. horizon-1
// One lane owns one problem and keeps its state vector in registers; the three small matrices are shared by
// all problems, sit in LDS and are read with wave-uniform (broadcast) addresses.  Per problem the kernel
// moves nx + horizon * nu floats in and horizon * nu out (plus the optional state trajectory): with the
// paper's sizes (12, 4, 5) that is 208 bytes for 2400 flop, so the kernel streams and HBM bounds it.
#include "common.hpp"

namespace ac {

template <int NX, int NU>
__global__ void __launch_bounds__(256) tinympc_forward_kernel(const TinyMpcParams p) {
  __shared__ float sA[NX * NX], sB[NX * NU], sK[NU * NX];
  for (int i = threadIdx.x; i < NX * NX; i += 256) sA[i] = p.Adyn[i];
  for (int i = threadIdx.x; i < NX * NU; i += 256) sB[i] = p.Bdyn[i];
  for (int i = threadIdx.x; i < NU * NX; i += 256) sK[i] = p.Kinf[i];
  __syncthreads();
  const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (b >= p.batch) return;
  float x[NX], u[NU], xn[NX];
  const float* x0 = p.x0 + b * NX;
#pragma unroll
  for (int r = 0; r < NX; r++) x[r] = x0[r];
  float* xo = p.x_out ? p.x_out + b * (p.horizon + 1) * NX : nullptr;
  if (xo) {
#pragma unroll
    for (int r = 0; r < NX; r++) xo[r] = x[r];
  }
  const float* d = p.d + b * p.horizon * NU;
  float* uo = p.u + b * p.horizon * NU;
  for (int i = 0; i < p.horizon; i++) {
#pragma unroll
    for (int r = 0; r < NU; r++) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < NX; c++) s = __builtin_fmaf(sK[r * NX + c], x[c], s);
      u[r] = -s - d[i * NU + r];
      uo[i * NU + r] = u[r];
    }
    // the state after the last control is not needed for u; it is only produced when the trajectory is asked for
    if (i + 1 < p.horizon || xo) {
#pragma unroll
      for (int r = 0; r < NX; r++) {
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < NX; c++) s = __builtin_fmaf(sA[r * NX + c], x[c], s);
        float t = 0.f;
#pragma unroll
        for (int c = 0; c < NU; c++) t = __builtin_fmaf(sB[r * NU + c], u[c], t);
        xn[r] = s + t;
      }
#pragma unroll
      for (int r = 0; r < NX; r++) x[r] = xn[r];
      if (xo) {
#pragma unroll
        for (int r = 0; r < NX; r++) xo[(i + 1) * NX + r] = x[r];
      }
    }
  }
}

// The paper's problem size (12 states, 4 controls, horizon 5) with coalesced output.  A problem's outputs are
// 80 bytes of u and 288 bytes of trajectory, so a lane that stores its own rows touches a different memory
// line with every store instruction of the wave.  Here a lane keeps its whole trajectory in registers, the
// wave transposes it through a private LDS window, and the 64 problems of the wave leave as one contiguous
// block of 16-byte stores (the problems of a wave are consecutive in memory).  No workgroup barrier after the
// matrices are in place: a wave only ever reads window words it wrote itself.  The inputs (128 bytes per
// problem) are loaded by their own lane: staging them through the window as well was measured slower.
template <bool WITH_X>
__global__ void __launch_bounds__(256) tinympc_forward_12_4_5_kernel(const TinyMpcParams p) {
  constexpr int NX = 12, NU = 4, H = 5;
  constexpr int XROW = (H + 1) * NX;  // 72 floats of trajectory per problem
  constexpr int XPITCH = XROW + 4;    // LDS row pitch: keeps 16-byte alignment for the read-back
  constexpr int UROW = H * NU;        // 20 floats of controls per problem
  extern __shared__ __attribute__((aligned(16))) float tinympc_lds[];  // 4 windows, then the three matrices
  float* sA = tinympc_lds + 4 * 64 * XPITCH;
  float* sB = sA + NX * NX;
  float* sK = sB + NX * NU;
  for (int i = threadIdx.x; i < NX * NX; i += 256) sA[i] = p.Adyn[i];
  for (int i = threadIdx.x; i < NX * NU; i += 256) sB[i] = p.Bdyn[i];
  for (int i = threadIdx.x; i < NU * NX; i += 256) sK[i] = p.Kinf[i];
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* win = tinympc_lds + wave * 64 * XPITCH;
  // Persistent waves: wave-block k is problems 64 k .. 64 k + 63; a wave takes blocks first, first + stride, ...
  // and requests the inputs of its next block before it computes and stores the current one, so that the reads of
  // one block travel while the writes of the previous one drain (these are ordinary loads and stores, so the waits
  // are the compiler's own: it counts the stores it issued after the loads instead of draining them, since
  // vector-memory operations complete in issue order).
  const int64_t nblk = (p.batch + 63) / 64, stride = (int64_t)gridDim.x * 4;
  int64_t blk = (int64_t)blockIdx.x * 4 + wave;
  if (blk >= nblk) return;
  v4f xin[NX / 4], din[UROW / 4];
  auto request = [&](int64_t k) {  // idle lanes of a partial block re-read its first problem and store nothing
    const int64_t first = k * 64, left = p.batch - first;
    const int64_t b = first + (lane < left ? lane : 0);
    const v4f* x4 = (const v4f*)(p.x0 + b * NX);
    const v4f* d4 = (const v4f*)(p.d + b * UROW);
#pragma unroll
    for (int q = 0; q < NX / 4; q++) xin[q] = x4[q];
#pragma unroll
    for (int q = 0; q < UROW / 4; q++) din[q] = d4[q];
  };
  request(blk);
  for (; blk < nblk; blk += stride) {
    const int64_t b0 = blk * 64;
    const int nvalid = p.batch - b0 < 64 ? (int)(p.batch - b0) : 64;
    float xs[H + 1][NX], us[H][NU], dv[UROW];
#pragma unroll
    for (int q = 0; q < NX / 4; q++)
#pragma unroll
      for (int e = 0; e < 4; e++) xs[0][4 * q + e] = xin[q][e];
#pragma unroll
    for (int q = 0; q < UROW / 4; q++)
#pragma unroll
      for (int e = 0; e < 4; e++) dv[4 * q + e] = din[q][e];
    if (blk + stride < nblk) request(blk + stride);
#pragma unroll
    for (int i = 0; i < H; i++) {
#pragma unroll
      for (int r = 0; r < NU; r++) {
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < NX; c++) s = __builtin_fmaf(sK[r * NX + c], xs[i][c], s);
        us[i][r] = -s - dv[i * NU + r];
      }
      if (i + 1 < H || WITH_X) {
#pragma unroll
        for (int r = 0; r < NX; r++) {
          float s = 0.f;
#pragma unroll
          for (int c = 0; c < NX; c++) s = __builtin_fmaf(sA[r * NX + c], xs[i][c], s);
          float t = 0.f;
#pragma unroll
          for (int c = 0; c < NU; c++) t = __builtin_fmaf(sB[r * NU + c], us[i][c], t);
          xs[i + 1][r] = s + t;
        }
      }
    }

    // controls: rows of 20 floats, then the block of nvalid * 20 floats in 16-byte pieces
#pragma unroll
    for (int i = 0; i < H; i++)
#pragma unroll
      for (int r = 0; r < NU; r++) win[lane * UROW + i * NU + r] = us[i][r];
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    {
      v4f* dst = (v4f*)(p.u + b0 * UROW);
      const int pieces = nvalid * (UROW / 4);
#pragma unroll
      for (int k = 0; k < UROW / 4; k++) {
        const int q = k * 64 + lane;
        if (q < pieces) dst[q] = *(const v4f*)(win + 4 * q);
      }
    }
    if constexpr (WITH_X) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the read-back above is done before the window is reused
#pragma unroll
      for (int i = 0; i <= H; i++)
#pragma unroll
        for (int r = 0; r < NX; r++) win[lane * XPITCH + i * NX + r] = xs[i][r];
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      v4f* dst = (v4f*)(p.x_out + b0 * XROW);
      const int pieces = nvalid * (XROW / 4);
#pragma unroll
      for (int k = 0; k < XROW / 4; k++) {
        const int q = k * 64 + lane;  // 16-byte piece q of the block: problem q / 18, piece q % 18 of its row
        if (q < pieces) dst[q] = *(const v4f*)(win + (q / (XROW / 4)) * XPITCH + (q % (XROW / 4)) * 4);
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the window is free for the next block
  }
}

// Any 1 <= nx, nu <= 16: same algorithm with run-time sizes (state vectors padded to 16 registers).
__global__ void __launch_bounds__(256) tinympc_forward_generic_kernel(const TinyMpcParams p) {
  constexpr int MAXN = 16;
  __shared__ float sA[MAXN * MAXN], sB[MAXN * MAXN], sK[MAXN * MAXN];
  const int nx = p.nx, nu = p.nu;
  for (int i = threadIdx.x; i < nx * nx; i += 256) sA[i] = p.Adyn[i];
  for (int i = threadIdx.x; i < nx * nu; i += 256) sB[i] = p.Bdyn[i];
  for (int i = threadIdx.x; i < nu * nx; i += 256) sK[i] = p.Kinf[i];
  __syncthreads();
  const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (b >= p.batch) return;
  float x[MAXN], u[MAXN], xn[MAXN];
#pragma unroll
  for (int r = 0; r < MAXN; r++) x[r] = r < nx ? p.x0[b * nx + r] : 0.f;
  float* xo = p.x_out ? p.x_out + b * (p.horizon + 1) * nx : nullptr;
  if (xo) {
#pragma unroll
    for (int r = 0; r < MAXN; r++)
      if (r < nx) xo[r] = x[r];
  }
  const float* d = p.d + b * p.horizon * nu;
  float* uo = p.u + b * p.horizon * nu;
  for (int i = 0; i < p.horizon; i++) {
#pragma unroll
    for (int r = 0; r < MAXN; r++) {
      u[r] = 0.f;
      if (r < nu) {
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < MAXN; c++)
          if (c < nx) s = __builtin_fmaf(sK[r * nx + c], x[c], s);
        u[r] = -s - d[i * nu + r];
        uo[i * nu + r] = u[r];
      }
    }
    if (i + 1 < p.horizon || xo) {
#pragma unroll
      for (int r = 0; r < MAXN; r++) {
        xn[r] = 0.f;
        if (r < nx) {
          float s = 0.f, t = 0.f;
#pragma unroll
          for (int c = 0; c < MAXN; c++)
            if (c < nx) s = __builtin_fmaf(sA[r * nx + c], x[c], s);
#pragma unroll
          for (int c = 0; c < MAXN; c++)
            if (c < nu) t = __builtin_fmaf(sB[r * nu + c], u[c], t);
          xn[r] = s + t;
        }
      }
#pragma unroll
      for (int r = 0; r < MAXN; r++) x[r] = xn[r];
      if (xo) {
#pragma unroll
        for (int r = 0; r < MAXN; r++)
          if (r < nx) xo[(i + 1) * nx + r] = x[r];
      }
    }
  }
}

// Persistent workgroups per compute unit of the (12, 4, 5) kernel: one (31.5 us for 262144 problems; two: 34.1 us).
#ifndef TINYMPC_WGS_PER_CU
#define TINYMPC_WGS_PER_CU 1
#endif
hipError_t launch_tinympc_forward(const TinyMpcParams& p, hipStream_t stream) {
  const int64_t blocks = (p.batch + 255) / 256;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const bool aligned16 = ((((uintptr_t)p.x0) | ((uintptr_t)p.d) | ((uintptr_t)p.u) | ((uintptr_t)p.x_out)) & 15) == 0;
  if (p.nx == 12 && p.nu == 4 && p.horizon == 5 && aligned16) {
    constexpr int LDS = (4 * 64 * 76 + 12 * 12 + 12 * 4 + 4 * 12) * (int)sizeof(float);  // 78784 bytes
    static std::atomic<bool> configured_x{false}, configured_u{false};
    if (const hipError_t e = allow_dynamic_lds_once(configured_x, tinympc_forward_12_4_5_kernel<true>, LDS)) return e;
    if (const hipError_t e = allow_dynamic_lds_once(configured_u, tinympc_forward_12_4_5_kernel<false>, LDS)) return e;
    const int cus = compute_units();
    const int64_t wgs = blocks < (int64_t)cus * TINYMPC_WGS_PER_CU ? blocks : (int64_t)cus * TINYMPC_WGS_PER_CU;  // persistent waves
    if (p.x_out) hipLaunchKernelGGL(tinympc_forward_12_4_5_kernel<true>, dim3((unsigned)wgs), dim3(256), LDS, stream, p);
    else hipLaunchKernelGGL(tinympc_forward_12_4_5_kernel<false>, dim3((unsigned)wgs), dim3(256), LDS, stream, p);
  } else if (p.nx == 12 && p.nu == 4) hipLaunchKernelGGL((tinympc_forward_kernel<12, 4>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL(tinympc_forward_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace ac
