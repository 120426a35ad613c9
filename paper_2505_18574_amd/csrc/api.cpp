// C ABI of the library (include/ac.h): argument validation on the host, then a
// launch on the caller's stream.  Nothing here allocates, frees or synchronises.
#include "../../include/ac.h"
#include "common.hpp"

#include <limits.h>

namespace {

bool fits_i32(int64_t v) { return v >= 0 && v <= INT_MAX; }

// *out = a * b for non-negative factors that each fit int32, false when the product does not fit int32.
bool mul_i32(int64_t a, int64_t b, int64_t* out) {
  if (!fits_i32(a) || !fits_i32(b)) return false;
  *out = a * b;  // below 2^62
  return fits_i32(*out);
}

// Sizes of an (implicit) GEMM the kernels and planners index without overflow: every dimension at most 2^29 (row
// lengths in bytes and rounded-up tile counts are 32-bit) and at most 2^31 - 1 tiles of 64 x 64 (work counters are
// 32-bit; such an output would be 8 TB).
bool gemm_dims_supported(int64_t M, int64_t N, int64_t K) {
  const int64_t lim = 1ll << 29;
  if (M < 0 || N < 0 || K < 0 || M > lim || N > lim || K > lim) return false;
  return ((M + 63) / 64) * ((N + 63) / 64) <= INT_MAX;
}

ac_status check_stage(int32_t shift, int32_t act) {
  if (shift < 0 || shift > 31) return AC_ERR_SHIFT;
  if (act != AC_ACT_NONE && act != AC_ACT_RELU) return AC_ERR_ACT;
  return AC_OK;
}

}  // namespace

extern "C" {

const char* ac_status_string(ac_status status) {
  switch (status) {
    case AC_OK: return "ok";
    case AC_ERR_NULL: return "a required pointer is NULL";
    case AC_ERR_SHAPE: return "a size is negative or outside the supported range";
    case AC_ERR_STRIDE: return "a leading dimension is smaller than the row length";
    case AC_ERR_SHIFT: return "shift must be in 0..31";
    case AC_ERR_ACT: return "unknown activation";
    case AC_ERR_ALIAS: return "an output has the same base address as an input";
    case AC_ERR_WORKSPACE: return "workspace too small or misaligned";
    case AC_ERR_LAUNCH: return "the HIP runtime refused the launch";
    case AC_ERR_PLAN: return "unknown tile, or a K split that this shape or these operands cannot take";
    default: return "unknown status";
  }
}

int32_t ac_version(void) { return 100; }

size_t ac_gemm_i8_workspace_bytes(int32_t M, int32_t N, int32_t K) {
  if (M <= 0 || N <= 0 || K <= 0 || !gemm_dims_supported(M, N, K)) return 0;
  // the plan for operands that the one-wave-per-tile kernel does not take (and for the convolution with this
  // implicit-GEMM shape): the most any launch of the shape asks for
  const ac::GemmPlan plan = ac::plan_gemm_i8(M, N, K, true, 0);
  if (plan.splits <= 1) return 0;
  // int32 partial sums of every K slice
  return (size_t)plan.splits * (size_t)M * (size_t)N * sizeof(int32_t);
}

size_t ac_gemm_i8_planned_workspace_bytes(int32_t M, int32_t N, int32_t K, int32_t tile, int32_t splits) {
  ac::GemmPlan plan;
  if (M <= 0 || N <= 0 || K <= 0 || !gemm_dims_supported(M, N, K) || !ac::make_plan_i8(K, tile, splits, &plan) || plan.splits <= 1) return 0;
  return (size_t)plan.splits * (size_t)M * (size_t)N * sizeof(int32_t);
}

size_t ac_gemm_bf16_workspace_bytes(int32_t M, int32_t N, int32_t K) {
  if (M <= 0 || N <= 0 || K <= 0 || !gemm_dims_supported(M, N, K)) return 0;
  const ac::GemmPlan plan = ac::plan_gemm_bf16(M, N, K);
  if (plan.splits <= 1) return 0;
  // fp32 partial products of every K slice
  return (size_t)plan.splits * (size_t)M * (size_t)N * sizeof(float);
}

size_t ac_gemm_bf16_planned_workspace_bytes(int32_t M, int32_t N, int32_t K, int32_t tile, int32_t splits) {
  ac::GemmPlan plan;
  if (M <= 0 || N <= 0 || K <= 0 || !gemm_dims_supported(M, N, K) || !ac::make_plan_bf16(K, tile, splits, &plan) || plan.splits <= 1) return 0;
  return (size_t)plan.splits * (size_t)M * (size_t)N * sizeof(float);
}

void ac_gemm_i8_auto_plan(int32_t M, int32_t N, int32_t K, int32_t have_workspace, int32_t* tile, int32_t* splits) {
  if (!gemm_dims_supported(M, N, K)) M = N = K = 0;  // sizes the calls refuse: the plan of the empty problem
  const ac::GemmPlan plan = ac::plan_gemm_i8(M, N, K, have_workspace != 0, 1);
  if (tile) *tile = plan.tile;
  if (splits) *splits = plan.splits;
}

void ac_gemm_bf16_auto_plan(int32_t M, int32_t N, int32_t K, int32_t* tile, int32_t* splits) {
  if (!gemm_dims_supported(M, N, K)) M = N = K = 0;
  const ac::GemmPlan plan = ac::plan_gemm_bf16(M, N, K);
  if (tile) *tile = plan.tile;
  if (splits) *splits = plan.splits;
}

}  // extern "C"

namespace {

// ac_gemm_i8 and ac_gemm_i8_planned: `planned` selects the caller's (tile, splits) over the library's choice.
ac_status gemm_i8_entry(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                        const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                        int32_t M, int32_t N, int32_t K, int32_t shift, int32_t act,
                        void* workspace, size_t workspace_bytes, bool planned, int32_t tile, int32_t splits, void* stream,
                        bool static_workspace = false) {
  if (!gemm_dims_supported(M, N, K)) return AC_ERR_SHAPE;
  if (ac_status s = check_stage(shift, act)) return s;
  if (lda < K || ldb < N || ldc < N) return AC_ERR_STRIDE;
  if (bias && bias_ld != 0 && bias_ld < N) return AC_ERR_STRIDE;
  if (bias_ld < 0) return AC_ERR_STRIDE;
  ac::GemmPlan plan;
  if (planned && !ac::make_plan_i8(K, tile, splits, &plan)) return AC_ERR_PLAN;
  if ((workspace == nullptr) != (workspace_bytes == 0)) return AC_ERR_WORKSPACE;
  const size_t need = planned ? ac_gemm_i8_planned_workspace_bytes(M, N, K, tile, splits) : ac_gemm_i8_workspace_bytes(M, N, K);
  if (workspace && (((uintptr_t)workspace & 15) != 0 || workspace_bytes < need)) return AC_ERR_WORKSPACE;
  if (planned && need > 0 && !workspace) return AC_ERR_WORKSPACE;
  if (static_workspace && need > AC_STATIC_SCRATCH_BYTES) return AC_ERR_WORKSPACE;  // partial sums beyond the library's own buffer

  ac::GemmParams p = {};
  p.A = A; p.B = B; p.C = C; p.bias = bias;
  p.lda = lda; p.ldb = ldb; p.ldc = ldc; p.bias_ld = bias_ld;
  p.M = M; p.N = N; p.K = K; p.shift = shift; p.act = act;
  p.splits = 1;
  // what a named plan asks of the operands is checked for every call, empty problems included
  if (planned && plan.splits > 1 && !ac::gemm_i8_fast_path(p)) return AC_ERR_PLAN;
  if (planned && (tile == 320 || tile == 160) && !(ac::gemm_i8_fast_path(p) && ac::wstat_eligible(p, tile))) return AC_ERR_PLAN;
  if (planned && (tile == 321 || tile == 161)) return AC_ERR_PLAN;  // the patch kernel is a convolution kernel
  if (planned && tile == 32 && !ac::gemm_i8_fast_path(p)) return AC_ERR_PLAN;
  if (M == 0 || N == 0) return AC_OK;
  if (!C || (K > 0 && (!A || !B))) return AC_ERR_NULL;
  if ((const void*)C == (const void*)A || (const void*)C == (const void*)B || (const void*)C == (const void*)bias)
    return AC_ERR_ALIAS;
  if (static_workspace && need > 0) {
    // the call is valid and its plan cuts K: the partial sums go through the current GPU's copy of the library's buffer
    if (ac::static_scratch(&workspace) != hipSuccess) return AC_ERR_LAUNCH;
    workspace_bytes = AC_STATIC_SCRATCH_BYTES;
  }
  p.partial = (int32_t*)workspace;
  return ac::launch_gemm_i8(p, (hipStream_t)stream, planned ? &plan : nullptr) == hipSuccess ? AC_OK : AC_ERR_LAUNCH;
}

ac_status gemm_bf16_entry(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb,
                          float* C, int64_t ldc, int32_t M, int32_t N, int32_t K,
                          float alpha, float beta, void* workspace, size_t workspace_bytes,
                          bool planned, int32_t tile, int32_t splits, void* stream) {
  if (!gemm_dims_supported(M, N, K)) return AC_ERR_SHAPE;
  if (lda < K || ldb < N || ldc < N) return AC_ERR_STRIDE;
  ac::GemmPlan plan;
  if (planned && !ac::make_plan_bf16(K, tile, splits, &plan)) return AC_ERR_PLAN;
  if ((workspace == nullptr) != (workspace_bytes == 0)) return AC_ERR_WORKSPACE;
  const size_t need = planned ? ac_gemm_bf16_planned_workspace_bytes(M, N, K, tile, splits) : ac_gemm_bf16_workspace_bytes(M, N, K);
  if (workspace && (((uintptr_t)workspace & 15) != 0 || workspace_bytes < need)) return AC_ERR_WORKSPACE;
  ac::GemmParams p = {};
  p.A = A; p.B = B; p.C = C;
  p.lda = lda; p.ldb = ldb; p.ldc = ldc;
  p.M = M; p.N = N; p.K = K; p.alpha = alpha; p.beta = beta;
  p.splits = 1;
  p.partial = (int32_t*)workspace;
  if (planned && plan.splits > 1 && !ac::gemm_bf16_fast_path(p)) return AC_ERR_PLAN;
  if (M == 0 || N == 0) return AC_OK;
  if (!C || (K > 0 && (!A || !B))) return AC_ERR_NULL;
  if ((const void*)C == (const void*)A || (const void*)C == (const void*)B) return AC_ERR_ALIAS;

  return ac::launch_gemm_bf16(p, (hipStream_t)stream, planned ? &plan : nullptr) == hipSuccess ? AC_OK : AC_ERR_LAUNCH;
}

}  // namespace

extern "C" {

ac_status ac_gemm_i8(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                     const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                     int32_t M, int32_t N, int32_t K, int32_t shift, int32_t act,
                     void* workspace, size_t workspace_bytes, void* stream) {
  return gemm_i8_entry(A, lda, B, ldb, bias, bias_ld, C, ldc, M, N, K, shift, act, workspace, workspace_bytes, false, 0, 0, stream);
}

ac_status ac_gemm_i8_static(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                            const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                            int32_t M, int32_t N, int32_t K, int32_t shift, int32_t act, void* stream) {
  static_assert(AC_STATIC_SCRATCH_BYTES == ac::STATIC_SCRATCH_BYTES, "header and library disagree on the scratch size");
  return gemm_i8_entry(A, lda, B, ldb, bias, bias_ld, C, ldc, M, N, K, shift, act, nullptr, 0, false, 0, 0, stream, true);
}

ac_status ac_gemm_i8_t(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                       const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                       int32_t M, int32_t N, int32_t K, int32_t shift, int32_t act,
                       int32_t trans_a, int32_t trans_b, void* stream) {
  if (!gemm_dims_supported(M, N, K)) return AC_ERR_SHAPE;
  if (ac_status s = check_stage(shift, act)) return s;
  if (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N) || ldc < N) return AC_ERR_STRIDE;
  if (bias_ld < 0 || (bias && bias_ld != 0 && bias_ld < N)) return AC_ERR_STRIDE;
  if (M == 0 || N == 0) return AC_OK;
  if (!C || (K > 0 && (!A || !B))) return AC_ERR_NULL;
  if ((const void*)C == (const void*)A || (const void*)C == (const void*)B || (const void*)C == (const void*)bias)
    return AC_ERR_ALIAS;
  ac::GemmParams p = {};
  p.A = A; p.B = B; p.C = C; p.bias = bias;
  p.lda = lda; p.ldb = ldb; p.ldc = ldc; p.bias_ld = bias_ld;
  p.M = M; p.N = N; p.K = K; p.shift = shift; p.act = act;
  p.splits = 1;
  return ac::launch_gemm_i8_trans(p, trans_a != 0, trans_b != 0, (hipStream_t)stream) == hipSuccess ? AC_OK : AC_ERR_LAUNCH;
}

ac_status ac_gemm_i8_planned(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                             const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                             int32_t M, int32_t N, int32_t K, int32_t shift, int32_t act,
                             void* workspace, size_t workspace_bytes, int32_t tile, int32_t splits, void* stream) {
  return gemm_i8_entry(A, lda, B, ldb, bias, bias_ld, C, ldc, M, N, K, shift, act, workspace, workspace_bytes, true, tile, splits, stream);
}

ac_status ac_gemm_i8_acc32(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                           const int32_t* bias, int64_t bias_ld, int32_t* C, int64_t ldc,
                           int32_t M, int32_t N, int32_t K, void* stream) {
  if (!gemm_dims_supported(M, N, K)) return AC_ERR_SHAPE;
  if (lda < K || ldb < N || ldc < N) return AC_ERR_STRIDE;
  if (bias_ld < 0 || (bias && bias_ld != 0 && bias_ld < N)) return AC_ERR_STRIDE;
  if (M == 0 || N == 0) return AC_OK;
  if (!C || (K > 0 && (!A || !B))) return AC_ERR_NULL;
  if ((const void*)C == (const void*)A || (const void*)C == (const void*)B || (const void*)C == (const void*)bias) return AC_ERR_ALIAS;
  ac::GemmParams p = {};
  p.A = A; p.B = B; p.C = C; p.bias = bias;
  p.lda = lda; p.ldb = ldb; p.ldc = ldc; p.bias_ld = bias_ld;
  p.M = M; p.N = N; p.K = K;
  p.splits = 1;
  return ac::launch_gemm_i8_acc32(p, (hipStream_t)stream) == hipSuccess ? AC_OK : AC_ERR_LAUNCH;
}

static ac_status conv2d_i8_entry(const int8_t* in, const int8_t* w, const int32_t* bias, int8_t* out,
                                 int32_t Nb, int32_t H, int32_t W, int32_t Cin, int32_t Cout,
                                 int32_t KH, int32_t KW, int32_t stride, int32_t pad,
                                 int32_t shift, int32_t act,
                                 void* workspace, size_t workspace_bytes, bool planned, int32_t tile, int32_t splits, void* stream) {
  if (Nb < 0 || H < 0 || W < 0 || Cin < 0 || Cout < 0 || KH < 1 || KW < 1 || stride < 1 || pad < 0) return AC_ERR_SHAPE;
  if (ac_status s = check_stage(shift, act)) return s;
  if ((int64_t)KH > (int64_t)H + 2 * (int64_t)pad || (int64_t)KW > (int64_t)W + 2 * (int64_t)pad) return AC_ERR_SHAPE;
  if (H > 32767 - pad || W > 32767 - pad) return AC_ERR_SHAPE;  // image coordinates are kept in 16 bits
  const int64_t OH = ((int64_t)H + 2 * pad - KH) / stride + 1, OW = ((int64_t)W + 2 * pad - KW) / stride + 1;
  // The kernel indexes the image and the implicit GEMM with 32-bit offsets.  Every product below is formed one
  // factor at a time and refused as soon as it leaves int32, so that none of them can overflow int64 first
  // (a large stride keeps OH * OW tiny while Nb, H * W and Cin are all near 2^31).
  int64_t M = 0, K = 0, in_elems = 0, window = 0;
  if (!mul_i32(Nb, OH, &M) || !mul_i32(M, OW, &M)) return AC_ERR_SHAPE;
  if (!mul_i32(KH, KW, &K) || !mul_i32(K, Cin, &K)) return AC_ERR_SHAPE;
  if (!mul_i32(Nb, H, &in_elems) || !mul_i32(in_elems, W, &in_elems) || !mul_i32(in_elems, Cin, &in_elems)) return AC_ERR_SHAPE;
  if (!mul_i32(KH, W, &window) || !mul_i32(window, Cin, &window)) return AC_ERR_SHAPE;
  if (!gemm_dims_supported(M, Cout, K) || !fits_i32(in_elems + window)) return AC_ERR_SHAPE;
  ac::GemmPlan plan;
  if (planned && !ac::make_plan_i8((int32_t)K, tile, splits, &plan)) return AC_ERR_PLAN;
  if ((workspace == nullptr) != (workspace_bytes == 0)) return AC_ERR_WORKSPACE;
  const size_t need = planned ? ac_gemm_i8_planned_workspace_bytes((int32_t)M, Cout, (int32_t)K, tile, splits)
                              : ac_gemm_i8_workspace_bytes((int32_t)M, Cout, (int32_t)K);
  if (workspace && (((uintptr_t)workspace & 15) != 0 || workspace_bytes < need)) return AC_ERR_WORKSPACE;
  if (planned && need > 0 && !workspace) return AC_ERR_WORKSPACE;
  if (M == 0 || Cout == 0) return AC_OK;
  if (!out || (K > 0 && (!in || !w))) return AC_ERR_NULL;
  if ((const void*)out == (const void*)in || (const void*)out == (const void*)w || (const void*)out == (const void*)bias)
    return AC_ERR_ALIAS;

  ac::GemmParams p = {};
  p.A = in; p.B = w; p.C = out; p.bias = bias;
  p.lda = 0; p.ldb = Cout; p.ldc = Cout; p.bias_ld = 0;
  p.M = (int32_t)M; p.N = Cout; p.K = (int32_t)K; p.shift = shift; p.act = act;
  p.H = H; p.W = W; p.Cin = Cin; p.KW = KW; p.OH = (int32_t)OH; p.OW = (int32_t)OW; p.stride = stride; p.pad = pad;
  p.KH = KH; p.a_bytes = (int32_t)in_elems;
  p.dCin = ac::FastDiv::make((unsigned)(Cin > 0 ? Cin : 1)); p.dKW = ac::FastDiv::make((unsigned)KW);
  p.dOW = ac::FastDiv::make((unsigned)(OW > 0 ? OW : 1)); p.dOH = ac::FastDiv::make((unsigned)(OH > 0 ? OH : 1));
  p.splits = 1;
  p.partial = (int32_t*)workspace;
  if (planned) {
    // a K split, the weight-stationary, patch and one-wave-per-tile kernels need the direct-to-LDS path: 16-byte aligned
    // operands, channel counts in multiples of 16, at most 32 kernel taps
    const bool fast = ac::conv_i8_fast_path(p);
    const bool ws = tile == 320 || tile == 160, patch = tile == 321 || tile == 161;
    if ((plan.splits > 1 || ws || patch || tile == 32) && !fast) return AC_ERR_PLAN;
    if (ws && !ac::wstat_eligible(p, tile)) return AC_ERR_PLAN;
    if (patch && !ac::conv_halo_eligible(p, tile)) return AC_ERR_PLAN;
  }
  return ac::launch_conv2d_i8(p, (hipStream_t)stream, planned ? &plan : nullptr) == hipSuccess ? AC_OK : AC_ERR_LAUNCH;
}

ac_status ac_conv2d_i8(const int8_t* in, const int8_t* w, const int32_t* bias, int8_t* out,
                       int32_t Nb, int32_t H, int32_t W, int32_t Cin, int32_t Cout,
                       int32_t KH, int32_t KW, int32_t stride, int32_t pad,
                       int32_t shift, int32_t act,
                       void* workspace, size_t workspace_bytes, void* stream) {
  return conv2d_i8_entry(in, w, bias, out, Nb, H, W, Cin, Cout, KH, KW, stride, pad, shift, act, workspace, workspace_bytes, false, 0, 0, stream);
}

ac_status ac_conv2d_i8_planned(const int8_t* in, const int8_t* w, const int32_t* bias, int8_t* out,
                               int32_t Nb, int32_t H, int32_t W, int32_t Cin, int32_t Cout,
                               int32_t KH, int32_t KW, int32_t stride, int32_t pad,
                               int32_t shift, int32_t act,
                               void* workspace, size_t workspace_bytes, int32_t tile, int32_t splits, void* stream) {
  return conv2d_i8_entry(in, w, bias, out, Nb, H, W, Cin, Cout, KH, KW, stride, pad, shift, act, workspace, workspace_bytes, true, tile, splits, stream);
}

ac_status ac_gemm_bf16(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb,
                       float* C, int64_t ldc, int32_t M, int32_t N, int32_t K,
                       float alpha, float beta, void* stream) {
  return gemm_bf16_entry(A, lda, B, ldb, C, ldc, M, N, K, alpha, beta, nullptr, 0, false, 0, 0, stream);
}

ac_status ac_gemm_bf16_ws(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb,
                          float* C, int64_t ldc, int32_t M, int32_t N, int32_t K,
                          float alpha, float beta, void* workspace, size_t workspace_bytes, void* stream) {
  return gemm_bf16_entry(A, lda, B, ldb, C, ldc, M, N, K, alpha, beta, workspace, workspace_bytes, false, 0, 0, stream);
}

ac_status ac_gemm_bf16_planned(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb,
                               float* C, int64_t ldc, int32_t M, int32_t N, int32_t K,
                               float alpha, float beta, void* workspace, size_t workspace_bytes,
                               int32_t tile, int32_t splits, void* stream) {
  return gemm_bf16_entry(A, lda, B, ldb, C, ldc, M, N, K, alpha, beta, workspace, workspace_bytes, true, tile, splits, stream);
}

ac_status ac_batched_gemm_f32(const float* A, const float* B, float* C,
                              const float* x, const float* d, float* y,
                              int32_t n, int64_t batch, void* stream) {
  if (n < 1 || n > 16 || batch < 0) return AC_ERR_SHAPE;
  if (batch == 0) return AC_OK;
  if (!A || !B) return AC_ERR_NULL;
  if (!C && !x) return AC_ERR_NULL;       // nothing requested
  if ((x != nullptr) != (y != nullptr)) return AC_ERR_NULL;
  if (d && !x) return AC_ERR_NULL;
  const void* ins[4] = {A, B, x, d};
  for (const void* q : ins)
    if (q && ((const void*)C == q || (const void*)y == q)) return AC_ERR_ALIAS;
  if (C && (const void*)C == (const void*)y) return AC_ERR_ALIAS;

  ac::BatchedParams p = {A, B, C, x, d, y, n, batch};
  return ac::launch_batched_f32(p, (hipStream_t)stream) == hipSuccess ? AC_OK : AC_ERR_LAUNCH;
}

ac_status ac_tinympc_forward_f32(const float* Adyn, const float* Bdyn, const float* Kinf,
                                 const float* x0, const float* d, float* u, float* x_out,
                                 int32_t nx, int32_t nu, int32_t horizon, int64_t batch, void* stream) {
  if (nx < 1 || nx > 16 || nu < 1 || nu > 16 || horizon < 0 || batch < 0) return AC_ERR_SHAPE;
  if (batch == 0 || horizon == 0) return AC_OK;  // no control to compute
  if (!Adyn || !Bdyn || !Kinf || !x0 || !d || !u) return AC_ERR_NULL;
  const void* ins[5] = {Adyn, Bdyn, Kinf, x0, d};
  for (const void* q : ins)
    if ((const void*)u == q || (x_out && (const void*)x_out == q)) return AC_ERR_ALIAS;
  if (x_out && (const void*)x_out == (const void*)u) return AC_ERR_ALIAS;
  ac::TinyMpcParams p = {Adyn, Bdyn, Kinf, x0, d, u, x_out, nx, nu, horizon, batch};
  return ac::launch_tinympc_forward(p, (hipStream_t)stream) == hipSuccess ? AC_OK : AC_ERR_LAUNCH;
}

}  // extern "C"
