// Forward pass of the TinyMPC primal update, batched over independent problems:
//   u[i]   = -Kinf . x[i] - d[i]
//   x[i+1] =  Adyn . x[i] + Bdyn . u[i]        i = 0 .. horizon-1
// Per problem the operation moves nx + horizon * nu floats in and horizon * nu out (plus the optional state
// trajectory): with the paper's sizes (12, 4, 5) that is 208 bytes (496 with the trajectory) for 2400 flop, so HBM
// bounds it.  Two families: the paper's sizes run on the matrix units, sixteen problems to a 16 x 16 product
// (tinympc_forward_mfma_kernel); any other size, and unaligned arrays, on the vector ALU with one lane per problem,
// its state vector in registers and the three shared matrices read from LDS with wave-uniform addresses.
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

// The paper's state and control sizes (12, 4) on the matrix units.  With u[i] substituted into the state update a
// step is one 16 x 16 product on the stacked vector z = [x[i] (12); d[i] (4)] of each problem:
//   [x[i + 1]; u[i]] = M . z,     M = [Adyn - Bdyn Kinf, -Bdyn; -Kinf, -I]
// v_mfma_f32_16x16x4_f32 takes a 16 x 4 and a 4 x 16 operand, one value per lane: lane l holds A[l % 16][l / 16] and
// B[l / 16][l % 16], and returns D[4 (l / 16) + v][l % 16] in register v = 0..3.  Sixteen problems are the columns.
// The sum over the 16 rows of z is order-free, so instruction c of a product takes rows 4 g + c (g = l / 16): the
// four registers a lane RECEIVES from one product (rows 4 g + 0..3 of its problem) are exactly the four values it
// FEEDS to the next, with no data movement in between; only the matrix operands are laid out to match (lane
// (m, g) holds column 4 g + c of row m for instruction c: four registers per matrix for the whole kernel).
// A wave owns 64 consecutive problems as four such column blocks; lanes g < 3 carry x, lanes g == 3 carry d and u.
// Some 500 instructions per 64 problems, 80 of them MFMAs, against 2100 on the vector ALU with one problem per
// lane.  Sums are fp32 throughout, in the matrix unit's order and with the closed-loop matrix formed first: equal to
// the recurrence in exact arithmetic, a few ulp from the ascending chains of the other kernels in fp32.
//
// Memory: the inputs and outputs of a wave's 64 problems are four contiguous runs (x0 3 KB, d and u 5 KB each, the
// trajectory 18 KB), but a lane's share of them is 16 bytes per step: stored as produced, a memory line is completed
// by instructions a whole step apart and leaves the L2 half written in between (58 us for 262144 problems; 39 us
// with the results held in registers and stored back to back at the end).  With HC > 0 (horizon HC) d is
// therefore loaded, and u and the trajectory are stored, as whole runs of 16 bytes per lane through a wave-private
// LDS window (u overwrites d in place, step by step; the trajectory goes block by block through a second window).
// HC == 0: any horizon, per-lane loads and stores as the results are produced.
constexpr int TMPC_XPITCH = 304;                         // LDS bytes per problem of a trajectory block (288 + padding)
constexpr int TMPC_WAVE_LDS = 64 * 80 + 16 * TMPC_XPITCH;  // d / u window of 64 problems + trajectory window of 16

template <bool WITH_X, int HC>
__global__ void __launch_bounds__(256) tinympc_forward_mfma_kernel(const TinyMpcParams p) {
  constexpr int NX = 12, NU = 4;
  __shared__ __attribute__((aligned(16))) unsigned char tmpc_lds[HC > 0 ? 4 * TMPC_WAVE_LDS : 16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, g = lane >> 4;
  // Wave-block k is problems 64 k .. 64 k + 63; a wave takes blocks first, first + stride, ... (HC > 0: persistent
  // waves that request their next block's inputs before they compute and store the current one, so that loads,
  // products and stores of different blocks overlap; with one block per wave the whole chip loads, then
  // multiplies, then stores: 38 us for 262144 problems).
  const int64_t nblk = (p.batch + 63) / 64, stride = (int64_t)gridDim.x * 4;
  int64_t blk = (int64_t)blockIdx.x * 4 + wave;
  if (blk >= nblk) return;  // whole waves leave; no wave waits for another
  const int H = HC > 0 ? HC : p.horizon;
  unsigned char* dwin = tmpc_lds + wave * TMPC_WAVE_LDS;  // [64 problems][HC][4] floats: d, then u
  unsigned char* xwin = dwin + 64 * 80;                   // [16 problems][TMPC_XPITCH]

  // matrix operand of instruction c: row m = n, column k = 4 g + c of
  //   M = [ Adyn - Bdyn Kinf   -Bdyn ]     so that   M . [x[i]; d[i]] = [x[i + 1]; u[i]]
  //       [      -Kinf           -I  ]
  // (x[i + 1] = Adyn x[i] + Bdyn u[i] with u[i] = -Kinf x[i] - d[i] substituted; Adyn - Bdyn Kinf is formed here in
  // fp32, four fused multiply-adds per entry in ascending order)
  float mat[4];
#pragma unroll
  for (int c = 0; c < 4; c++) {
    const int k = 4 * g + c;
    float v;
    if (n < NX && k < NX) {
      v = p.Adyn[n * NX + k];
#pragma unroll
      for (int j = 0; j < NU; j++) v = __builtin_fmaf(-p.Bdyn[n * NU + j], p.Kinf[j * NX + k], v);
    } else if (n < NX) {
      v = -p.Bdyn[n * NU + (k - NX)];
    } else if (k < NX) {
      v = -p.Kinf[(n - NX) * NX + k];
    } else {
      v = (k - NX == n - NX) ? -1.f : 0.f;
    }
    mat[c] = v;
  }

  // inputs of a block: d as one contiguous run, 16 bytes per lane and instruction (HC > 0), and per column block the
  // lane's 16 bytes of x0 (lanes past the end re-read the last problem and store nothing).  Every byte is read once
  // and every result written once, so loads and stores carry the non-temporal hint (262144 problems: 27.0 -> 26.3 us
  // with the trajectory, 18.7 -> 16.0 us without)
  v4f din[HC > 0 ? HC : 1], xin[4];
  auto request = [&](int64_t k) {
    const int left = p.batch - k * 64 < 64 ? (int)(p.batch - k * 64) : 64;
    if constexpr (HC > 0) {
      const v4f* src = (const v4f*)(p.d + k * 64 * HC * NU);
#pragma unroll
      for (int j = 0; j < HC; j++) {
        const int q = j * 64 + lane;
        din[j] = q < left * HC ? __builtin_nontemporal_load(src + q) : (v4f){0.f, 0.f, 0.f, 0.f};
      }
    }
#pragma unroll
    for (int b = 0; b < 4; b++) {
      const int64_t q = k * 64 + 16 * b + n;
      xin[b] = g < 3 ? __builtin_nontemporal_load((const v4f*)(p.x0 + (q < p.batch ? q : p.batch - 1) * NX + 4 * g)) : (v4f){0.f, 0.f, 0.f, 0.f};
    }
  };
  request(blk);
  for (; blk < nblk; blk += HC > 0 ? stride : nblk) {
  const int nvalid = p.batch - blk * 64 < 64 ? (int)(p.batch - blk * 64) : 64;
  if constexpr (HC > 0) {
#pragma unroll
    for (int j = 0; j < HC; j++) *(v4f*)(dwin + 16 * (j * 64 + lane)) = din[j];
  }
  v4f z[4];  // lanes g < 3: x0 rows 4 g .. 4 g + 3; lanes g == 3 take d[0] below
  int64_t prob[4];
  bool live[4];
#pragma unroll
  for (int b = 0; b < 4; b++) {
    const int64_t q = blk * 64 + 16 * b + n;
    live[b] = q < p.batch;
    prob[b] = live[b] ? q : p.batch - 1;
    z[b] = xin[b];
  }
  if (HC > 0 && blk + stride < nblk) request(blk + stride);
  v4f hist[HC > 0 ? HC + 1 : 1][4];  // HC > 0, lanes g < 3: the lane's rows of x[0 .. HC]
  if constexpr (HC > 0) {
#pragma unroll
    for (int b = 0; b < 4; b++) hist[0][b] = z[b];
  } else if constexpr (WITH_X) {
#pragma unroll
    for (int b = 0; b < 4; b++)
      if (g < 3 && live[b]) *(v4f*)(p.x_out + prob[b] * (int64_t)(H + 1) * NX + 4 * g) = z[b];  // x[0] = x0
  }

  // z = [x[i]; d[i]]: lanes g == 3 take d[i] (from the window, or from memory)
  auto d_of = [&](int b, int i) {
    if constexpr (HC > 0) return *(const v4f*)(dwin + (16 * b + n) * (HC * 16) + i * 16);
    else return *(const v4f*)(p.d + (prob[b] * H + i) * NU);
  };
#pragma unroll
  for (int b = 0; b < 4; b++)
    if (g == 3) z[b] = d_of(b, 0);
#pragma unroll
  for (int i = 0; i < H; i++) {
    v4f acc[4];
#pragma unroll
    for (int b = 0; b < 4; b++) acc[b] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; c++)  // the four column blocks are independent: their instructions alternate
#pragma unroll
      for (int b = 0; b < 4; b++) acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(mat[c], z[b][c], acc[b], 0, 0, 0);
#pragma unroll
    for (int b = 0; b < 4; b++) {
      if (g == 3) {  // rows 12..15: u[i], into the place of d[i]; then d[i + 1]
        if constexpr (HC > 0) *(v4f*)(dwin + (16 * b + n) * (HC * 16) + i * 16) = acc[b];
        else if (live[b]) *(v4f*)(p.u + (prob[b] * H + i) * NU) = acc[b];
        if (i + 1 < H) z[b] = d_of(b, i + 1);
      } else {       // rows 0..11: x[i + 1]
        z[b] = acc[b];
        if constexpr (HC > 0) hist[i + 1 <= HC ? i + 1 : 0][b] = acc[b];
        else if (WITH_X && live[b]) *(v4f*)(p.x_out + (prob[b] * (int64_t)(H + 1) + i + 1) * NX + 4 * g) = acc[b];
      }
    }
  }

  if constexpr (HC > 0) {
    // u: the window, in memory order, 16 bytes per lane (LDS serves a wave's operations in order: the reads below
    // see the writes above without a wait of their own beyond the compiler's)
    {
      v4f* dst = (v4f*)(p.u + blk * 64 * HC * NU);
      const int pieces = nvalid * HC;
#pragma unroll
      for (int k = 0; k < HC; k++) {
        const int q = k * 64 + lane;
        if (q < pieces) __builtin_nontemporal_store(*(const v4f*)(dwin + 16 * q), dst + q);
      }
    }
    if constexpr (WITH_X) {
      constexpr int XROW = (HC + 1) * NX * 4;  // bytes of trajectory per problem
      constexpr int PPB = XROW / 16;           // 16-byte pieces per problem
#pragma unroll
      for (int b = 0; b < 4; b++) {
        if (g < 3) {
#pragma unroll
          for (int i = 0; i <= HC; i++) *(v4f*)(xwin + n * TMPC_XPITCH + i * (NX * 4) + g * 16) = hist[i][b];
        }
        v4f* dst = (v4f*)(p.x_out + (blk * 64 + 16 * b) * (int64_t)(HC + 1) * NX);
        const int left = nvalid - 16 * b;  // problems of this block that exist
        const int pieces = (left < 0 ? 0 : left > 16 ? 16 : left) * PPB;
#pragma unroll
        for (int k = 0; k < (16 * PPB + 63) / 64; k++) {
          const int q = k * 64 + lane;  // piece q of the block: problem q / PPB, piece q % PPB of its rows
          if (q < pieces) __builtin_nontemporal_store(*(const v4f*)(xwin + (q / PPB) * TMPC_XPITCH + (q % PPB) * 16), dst + q);
        }
      }
    }
  }
  }  // blocks of this wave
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

// Persistent workgroups per compute unit of the (12, 4, 5) kernel: one (27.3 us for 262144 problems; two, three,
// four: 31.1, 33.0, 34.9 us).
#ifndef TINYMPC_WGS_PER_CU
#define TINYMPC_WGS_PER_CU 1
#endif
hipError_t launch_tinympc_forward(const TinyMpcParams& p, hipStream_t stream) {
  const int64_t blocks = (p.batch + 255) / 256;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const bool aligned16 = ((((uintptr_t)p.x0) | ((uintptr_t)p.d) | ((uintptr_t)p.u) | ((uintptr_t)p.x_out)) & 15) == 0;
  if (p.nx == 12 && p.nu == 4 && aligned16) {
    const int64_t waves = (p.batch + 63) / 64;
    const dim3 grid((unsigned)((waves + 3) / 4));
    if (p.horizon == 5) {
      const int64_t slots = (int64_t)compute_units() * TINYMPC_WGS_PER_CU;  // persistent waves
      const dim3 pgrid((unsigned)(grid.x < slots ? grid.x : slots));
      if (p.x_out) hipLaunchKernelGGL((tinympc_forward_mfma_kernel<true, 5>), pgrid, dim3(256), 0, stream, p);
      else hipLaunchKernelGGL((tinympc_forward_mfma_kernel<false, 5>), pgrid, dim3(256), 0, stream, p);
    } else {
      if (p.x_out) hipLaunchKernelGGL((tinympc_forward_mfma_kernel<true, 0>), grid, dim3(256), 0, stream, p);
      else hipLaunchKernelGGL((tinympc_forward_mfma_kernel<false, 0>), grid, dim3(256), 0, stream, p);
    }
  } else if (p.nx == 12 && p.nu == 4) hipLaunchKernelGGL((tinympc_forward_kernel<12, 4>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL(tinympc_forward_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace ac
