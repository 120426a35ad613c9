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

hipError_t launch_tinympc_forward(const TinyMpcParams& p, hipStream_t stream) {
  const int64_t blocks = (p.batch + 255) / 256;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (p.nx == 12 && p.nu == 4) hipLaunchKernelGGL((tinympc_forward_kernel<12, 4>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL(tinympc_forward_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace ac
