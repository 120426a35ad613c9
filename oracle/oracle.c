/*
 * CPU oracle for the dense tensor operations of arxiv 2505.18574 (Autocomp).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the GPU library must compute.  It shares no code, header, table or helper
 * with the HIP path and must never be called from it; only the tests, the
 * smoke check and the CPU-baseline leg of the benchmark may load it.
 *
 * Every function is the textbook definition written out: no tiling, no
 * fusion, no reordering of a sum (each output element adds its terms in
 * ascending k).  The only concession to run time is that independent output
 * rows / batch items are split over OpenMP threads, which changes no result.
 *
 * Precision: integer paths accumulate in int64 (and report any sum that does
 * not fit int32, the accumulator type of the paper's int8 accelerator,
 * Section 4.4); floating-point paths compute in fp64 from the exact values
 * of their bf16 / fp32 inputs.
 *
 * Pins (tests/test_oracle_*.py): exact-rational rounding, brute force on tiny
 * shapes, numpy int64/fp64 library matmuls, identity/zero/linearity/
 * permutation invariants, closed-form padding counts, conv == im2col GEMM,
 * the printed TinyMPC recurrence unrolled by hand.  No function here is
 * "parity unpinned".
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_ACT_NONE 0
#define ORACLE_ACT_RELU 1

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * v / 2^s rounded to the nearest integer, ties to the even integer.
 * The paper only says the accumulator is read back as "scaled-down" input-type
 * data (Appendix C, Fig. 15, bit 29); the power-of-two, round-half-even reading
 * is the one the int8 workloads here are specified with.
 */
int64_t oracle_rne_rshift(int64_t v, int32_t s) {
  if (s <= 0) return v;
  int64_t one = 1;
  int64_t fl = v >> s;               /* floor(v / 2^s): arithmetic shift        */
  int64_t rem = v - (fl << s);       /* 0 <= rem < 2^s                         */
  int64_t half = one << (s - 1);
  if (rem > half) return fl + 1;
  if (rem == half && (fl & 1)) return fl + 1;
  return fl;
}

/* Output stage of the int8 accelerator (Fig. 14: activation set by config_ex;
 * Fig. 15: scaled-down read of the accumulator): shift, saturate, ReLU. */
static int8_t requantise(int64_t acc, int32_t shift, int32_t act) {
  int64_t q = oracle_rne_rshift(acc, shift);
  if (q > 127) q = 127;
  if (q < -128) q = -128;
  if (act == ORACLE_ACT_RELU && q < 0) q = 0;
  return (int8_t)q;
}

int8_t oracle_requantise(int64_t acc, int32_t shift, int32_t act) { return requantise(acc, shift, act); }

/* Element-wise forms of the two functions above, for testing them on arrays. */
void oracle_rne_rshift_vec(const int64_t* v, int32_t s, int64_t* out, int64_t count) {
  for (int64_t i = 0; i < count; i++) out[i] = oracle_rne_rshift(v[i], s);
}

void oracle_requantise_vec(const int64_t* acc, int32_t shift, int32_t act, int8_t* out, int64_t count) {
  for (int64_t i = 0; i < count; i++) out[i] = requantise(acc[i], shift, act);
}

/*
 * int8 GEMM, Section 2 Fig. 2 (C[i][j] += A[i][k]*B[k][j]) with the bias of
 * Fig. 14 ("C = A * B + bias") and the output stage above.
 * A: M x K row-major (lda), B: K x N row-major (ldb), C: M x N row-major (ldc).
 * bias == NULL: none; bias_ld == 0: one row of N values broadcast to every row;
 * otherwise an M x N matrix with row stride bias_ld.
 * acc_out, if non-NULL, receives the raw M x N int64 sums (row stride N).
 * Returns the number of outputs whose exact sum does not fit in int32.
 */
int64_t oracle_gemm_i8(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                       const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                       int64_t M, int64_t N, int64_t K, int32_t shift, int32_t act,
                       int64_t* acc_out) {
  int64_t overflow = 0;
#pragma omp parallel for schedule(static) reduction(+ : overflow)
  for (int64_t i = 0; i < M; i++) {
    int64_t* row = (int64_t*)malloc((size_t)(N > 0 ? N : 1) * sizeof(int64_t));
    for (int64_t j = 0; j < N; j++) row[j] = 0;
    for (int64_t k = 0; k < K; k++) {
      int64_t a = A[i * lda + k];
      for (int64_t j = 0; j < N; j++) row[j] += a * (int64_t)B[k * ldb + j];
    }
    for (int64_t j = 0; j < N; j++) {
      int64_t s = row[j];
      if (bias) s += (bias_ld == 0) ? (int64_t)bias[j] : (int64_t)bias[i * bias_ld + j];
      if (s > INT32_MAX || s < INT32_MIN) overflow++;
      if (acc_out) acc_out[i * N + j] = s;
      if (C) C[i * ldc + j] = requantise(s, shift, act);
    }
    free(row);
  }
  return overflow;
}

/*
 * int8 convolution, direct definition (Section 4.4.2 names the workload; the
 * layouts are NHWC activations, [KH][KW][Cin][Cout] weights, NHWC output):
 *   out[n,oh,ow,co] = stage( bias[co] + sum_{kh,kw,ci} in[n, oh*stride-pad+kh,
 *                            ow*stride-pad+kw, ci] * w[kh,kw,ci,co] )
 * with taps outside the image contributing zero.  OH = (H+2*pad-KH)/stride+1.
 * Returns the count of sums outside int32.
 */
int64_t oracle_conv2d_i8(const int8_t* in, const int8_t* w, const int32_t* bias, int8_t* out,
                         int64_t Nb, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                         int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                         int32_t shift, int32_t act) {
  int64_t OH = (H + 2 * pad - KH) / stride + 1;
  int64_t OW = (W + 2 * pad - KW) / stride + 1;
  int64_t overflow = 0;
  if (OH <= 0 || OW <= 0) return 0;
#pragma omp parallel for schedule(static) collapse(2) reduction(+ : overflow)
  for (int64_t n = 0; n < Nb; n++) {
    for (int64_t oh = 0; oh < OH; oh++) {
      for (int64_t ow = 0; ow < OW; ow++) {
        for (int64_t co = 0; co < Cout; co++) {
          int64_t s = bias ? (int64_t)bias[co] : 0;
          for (int64_t kh = 0; kh < KH; kh++) {
            int64_t ih = oh * stride - pad + kh;
            if (ih < 0 || ih >= H) continue;
            for (int64_t kw = 0; kw < KW; kw++) {
              int64_t iw = ow * stride - pad + kw;
              if (iw < 0 || iw >= W) continue;
              const int8_t* px = in + ((n * H + ih) * W + iw) * Cin;
              const int8_t* wt = w + ((kh * KW + kw) * Cin) * Cout + co;
              for (int64_t ci = 0; ci < Cin; ci++) s += (int64_t)px[ci] * (int64_t)wt[ci * Cout];
            }
          }
          if (s > INT32_MAX || s < INT32_MIN) overflow++;
          out[((n * OH + oh) * OW + ow) * Cout + co] = requantise(s, shift, act);
        }
      }
    }
  }
  return overflow;
}

/*
 * Explicit im2col: row m = (n*OH+oh)*OW+ow, column k = (kh*KW+kw)*Cin+ci,
 * zero where the tap falls in the padding.  Used only to state the invariant
 * "convolution == GEMM on the im2col matrix" with two separately written codes.
 * col: (Nb*OH*OW) x (KH*KW*Cin), row-major, dense.
 */
void oracle_im2col_i8(const int8_t* in, int8_t* col, int64_t Nb, int64_t H, int64_t W, int64_t Cin,
                      int64_t KH, int64_t KW, int64_t stride, int64_t pad) {
  int64_t OH = (H + 2 * pad - KH) / stride + 1;
  int64_t OW = (W + 2 * pad - KW) / stride + 1;
  int64_t Kc = KH * KW * Cin;
  for (int64_t n = 0; n < Nb; n++)
    for (int64_t oh = 0; oh < OH; oh++)
      for (int64_t ow = 0; ow < OW; ow++) {
        int64_t m = (n * OH + oh) * OW + ow;
        for (int64_t kh = 0; kh < KH; kh++)
          for (int64_t kw = 0; kw < KW; kw++) {
            int64_t ih = oh * stride - pad + kh, iw = ow * stride - pad + kw;
            for (int64_t ci = 0; ci < Cin; ci++) {
              int8_t v = 0;
              if (ih >= 0 && ih < H && iw >= 0 && iw < W) v = in[((n * H + ih) * W + iw) * Cin + ci];
              col[m * Kc + (kh * KW + kw) * Cin + ci] = v;
            }
          }
      }
}

/* A bf16 value is the upper half of an fp32 bit pattern; widening is exact. */
static double bf16_to_double(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

double oracle_bf16_to_double(uint16_t b) { return bf16_to_double(b); }

/*
 * bf16 GEMM with wide output (the GEMM of Fig. 2 at the 4096^3 shape of
 * Appendix A Table 5): C = alpha * (A.B) + beta * C_in, all in fp64.
 * A: M x K bf16 bits (lda), B: K x N bf16 bits (ldb); C_in: fp32 M x N (ldc_in)
 * read only when beta != 0; C_out: fp64 M x N dense.
 */
void oracle_gemm_bf16(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb,
                      const float* C_in, int64_t ldc_in, double* C_out,
                      int64_t M, int64_t N, int64_t K, double alpha, double beta) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; i++) {
    double* row = C_out + i * N;
    for (int64_t j = 0; j < N; j++) row[j] = 0.0;
    for (int64_t k = 0; k < K; k++) {
      double a = bf16_to_double(A[i * lda + k]);
      for (int64_t j = 0; j < N; j++) row[j] += a * bf16_to_double(B[k * ldb + j]);
    }
    for (int64_t j = 0; j < N; j++) {
      double v = alpha * row[j];
      if (beta != 0.0) v += beta * (double)C_in[i * ldc_in + j];
      row[j] = v;
    }
  }
}

/*
 * The same definition evaluated only at listed (row, col) positions, so that
 * full-size results can be spot-checked; also returns sum_k |a*b| per sample,
 * the scale of the rounding-error bound.
 */
void oracle_gemm_bf16_at(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb,
                         const float* C_in, int64_t ldc_in, int64_t K, double alpha, double beta,
                         const int64_t* rows, const int64_t* cols, int64_t nsamples,
                         double* out, double* abs_sum) {
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < nsamples; s++) {
    int64_t i = rows[s], j = cols[s];
    double acc = 0.0, mag = 0.0;
    for (int64_t k = 0; k < K; k++) {
      double p = bf16_to_double(A[i * lda + k]) * bf16_to_double(B[k * ldb + j]);
      acc += p;
      mag += p < 0 ? -p : p;
    }
    double v = alpha * acc;
    if (beta != 0.0) v += beta * (double)C_in[i * ldc_in + j];
    out[s] = v;
    if (abs_sum) abs_sum[s] = mag;
  }
}

/* int8 GEMM at listed positions (same definition as oracle_gemm_i8). */
void oracle_gemm_i8_at(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                       const int32_t* bias, int64_t bias_ld, int64_t K, int32_t shift, int32_t act,
                       const int64_t* rows, const int64_t* cols, int64_t nsamples, int8_t* out) {
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < nsamples; s++) {
    int64_t i = rows[s], j = cols[s];
    int64_t acc = 0;
    for (int64_t k = 0; k < K; k++) acc += (int64_t)A[i * lda + k] * (int64_t)B[k * ldb + j];
    if (bias) acc += (bias_ld == 0) ? (int64_t)bias[j] : (int64_t)bias[i * bias_ld + j];
    out[s] = requantise(acc, shift, act);
  }
}

/*
 * Batched small dense algebra (the fine-grained workload of Section 4.4.3 /
 * Appendix D.2: n x n products followed by a matrix-vector product and an
 * element-wise add), per item b, in fp64 from the fp32 inputs:
 *   C_b = A_b . B_b            (n x n)
 *   y_b = C_b . x_b + d_b      (C_b not rounded in between)
 * A, B: [batch][n][n]; x, d: [batch][n].  C_out: [batch][n][n] fp64 or NULL;
 * y_out: [batch][n] fp64 or NULL (then x, d are not read); d NULL = no add.
 */
void oracle_batched_gemm_f32(const float* A, const float* B, double* C_out,
                             const float* x, const float* d, double* y_out,
                             int64_t n, int64_t batch) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < batch; b++) {
    double Cb[32 * 32];
    const float* Ab = A + b * n * n;
    const float* Bb = B + b * n * n;
    for (int64_t i = 0; i < n; i++)
      for (int64_t j = 0; j < n; j++) {
        double s = 0.0;
        for (int64_t k = 0; k < n; k++) s += (double)Ab[i * n + k] * (double)Bb[k * n + j];
        Cb[i * n + j] = s;
      }
    if (C_out)
      for (int64_t e = 0; e < n * n; e++) C_out[b * n * n + e] = Cb[e];
    if (y_out) {
      for (int64_t i = 0; i < n; i++) {
        double s = 0.0;
        for (int64_t j = 0; j < n; j++) s += Cb[i * n + j] * (double)x[b * n + j];
        if (d) s += (double)d[b * n + i];
        y_out[b * n + i] = s;
      }
    }
  }
}

/*
 * Forward pass of the TinyMPC primal update (Appendix D.2), batched over
 * independent problems, in fp64 from fp32 inputs:
 *   u[i]   = -Kinf . x[i] - d[i]
 *   x[i+1] =  Adyn . x[i] + Bdyn . u[i]          i = 0 .. horizon-1
 * Adyn: [nx][nx], Bdyn: [nx][nu], Kinf: [nu][nx] shared by all problems;
 * x0: [batch][nx]; d: [batch][horizon][nu]; u_out: [batch][horizon][nu];
 * x_out: [batch][horizon+1][nx] or NULL (row 0 is x0; the last row is the
 * state the paper notes is computed but never used).
 */
void oracle_tinympc_forward(const float* Adyn, const float* Bdyn, const float* Kinf,
                            const float* x0, const float* d, double* u_out, double* x_out,
                            int64_t nx, int64_t nu, int64_t horizon, int64_t batch) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < batch; b++) {
    double x[64], xn[64], u[64];
    for (int64_t r = 0; r < nx; r++) x[r] = (double)x0[b * nx + r];
    if (x_out)
      for (int64_t r = 0; r < nx; r++) x_out[(b * (horizon + 1)) * nx + r] = x[r];
    for (int64_t i = 0; i < horizon; i++) {
      for (int64_t r = 0; r < nu; r++) {
        double s = 0.0;
        for (int64_t c = 0; c < nx; c++) s += (double)Kinf[r * nx + c] * x[c];
        u[r] = -s - (double)d[(b * horizon + i) * nu + r];
        u_out[(b * horizon + i) * nu + r] = u[r];
      }
      for (int64_t r = 0; r < nx; r++) {
        double s = 0.0;
        for (int64_t c = 0; c < nx; c++) s += (double)Adyn[r * nx + c] * x[c];
        double t = 0.0;
        for (int64_t c = 0; c < nu; c++) t += (double)Bdyn[r * nu + c] * u[c];
        xn[r] = s + t;
      }
      for (int64_t r = 0; r < nx; r++) x[r] = xn[r];
      if (x_out)
        for (int64_t r = 0; r < nx; r++) x_out[(b * (horizon + 1) + i + 1) * nx + r] = x[r];
    }
  }
}
