/*
 * ac.h - C ABI of the MI355X (gfx950) dense tensor library.
 *
 * The operations are the ones arxiv 2505.18574 (Autocomp) optimises on its
 * accelerators: int8 GEMM and convolution with the int8 accelerator's bias /
 * scale-down / saturate / ReLU output stage (Section 4.4, Appendix C), the
 * large GEMM of the GPU study (Appendix A, Table 5) in bf16 with fp32
 * accumulation, and the batched fine-grained fp32 linear algebra of the
 * TinyMPC study (Section 4.4.3, Appendix D.2).
 *
 * Conventions shared by every entry point
 *  - Every data pointer is a DEVICE pointer into ordinary (coarse-grained)
 *    device memory owned by the caller.  The library allocates nothing, frees
 *    nothing and never synchronises: work is enqueued on `stream` (a
 *    hipStream_t passed as void*; NULL = the default stream) and the call
 *    returns once the kernels are launched.
 *  - No result depends on an earlier call.  What the library does keep for the
 *    life of the process is set-up, not results: it serves ONE GPU per process
 *    (the compute-unit count of the device that is current at the first call
 *    sizes every launch), each kernel is configured for its LDS size the first
 *    time it is launched, and ac_gemm_i8_static owns a partial-sum buffer.  The
 *    kernel / tile choices are calibrated on the 256 compute units in 8 XCDs of
 *    an MI355X; on another count they stay correct and are merely untuned.
 *  - All matrices are row-major.  Leading dimensions (lda, ...) are in
 *    ELEMENTS and may exceed the row length.
 *  - An output must not share its base address with an input
 *    (AC_ERR_ALIAS); partially overlapping buffers are undefined.
 *  - Arguments are validated on the host before anything is launched; on any
 *    error a negative ac_status is returned and no work is enqueued.
 *    No C++ exception crosses this boundary.
 *  - Zero-sized problems (M, N or batch == 0) return AC_OK without a launch.
 *  - GEMM sizes (for a convolution: those of its implicit GEMM) are supported up to 2^29 per dimension and
 *    2^31 - 1 blocks of 64 x 64 outputs; larger ones return AC_ERR_SHAPE.
 */
#ifndef AC_H_
#define AC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t ac_status;

enum {
  AC_OK = 0,
  AC_ERR_NULL = -1,      /* a required pointer is NULL                              */
  AC_ERR_SHAPE = -2,     /* a negative size, or a size outside the supported range  */
  AC_ERR_STRIDE = -3,    /* a leading dimension smaller than the row length         */
  AC_ERR_SHIFT = -4,     /* shift outside 0..31                                     */
  AC_ERR_ACT = -5,       /* unknown activation                                      */
  AC_ERR_ALIAS = -6,     /* an output has the same base address as an input         */
  AC_ERR_WORKSPACE = -7, /* workspace pointer/size inconsistent                     */
  AC_ERR_LAUNCH = -8,    /* the HIP runtime refused the launch                      */
  AC_ERR_PLAN = -9       /* unknown tile, or a K split the shape/operands cannot take */
};

/* Activations of the output stage (Appendix C, Fig. 14: the `act` field of
 * config_ex).  The normalisation-type activations listed there are not part
 * of this library. */
enum { AC_ACT_NONE = 0, AC_ACT_RELU = 1 };

/*
 * int8 GEMM with the int8 accelerator's output stage.
 *
 *   acc[i][j] = sum_k A[i][k] * B[k][j] + bias(i, j)           exact, int32
 *   C[i][j]   = act( sat8( rne_rshift(acc[i][j], shift) ) )    int8
 *
 * The contraction is the matrix product of Section 2 (Fig. 2) on the
 * A[M][K], B[K][N], C[M][N] operands of the paper's GEMM kernels
 * (Appendix D.1).  The bias enters through the accumulator ("C = A * B +
 * bias", Appendix C Fig. 14); the int8 result is the scaled-down read of the
 * accumulator with the configured activation (Appendix C Fig. 15, bit 29).
 * rne_rshift(v, s) is v / 2^s rounded to the nearest integer with halves to
 * the even neighbour; sat8 clamps to [-128, 127]; act is AC_ACT_NONE or
 * AC_ACT_RELU.  The result is defined when every exact sum fits in int32.
 *
 *   A     device, int8,  M x K, row stride lda >= K
 *   B     device, int8,  K x N, row stride ldb >= N
 *   bias  device, int32; NULL = no bias; bias_ld == 0: a row of N values added
 *         to every row of the product; bias_ld >= N: an M x N matrix with that
 *         row stride
 *   C     device, int8,  M x N, row stride ldc >= N (written, never read)
 *   K == 0 gives C = stage(bias).
 *   workspace / workspace_bytes: optional device scratch of at least
 *         ac_gemm_i8_workspace_bytes(M, N, K) bytes, 16-byte aligned, which
 *         lets the library split the K range of shapes with few output tiles
 *         over more compute units; its contents on entry and exit are
 *         unspecified and concurrent calls must not share it.  NULL / 0 is
 *         always accepted (no split).  A non-NULL workspace that is too small
 *         or misaligned gives AC_ERR_WORKSPACE.
 */
ac_status ac_gemm_i8(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                     const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                     int32_t M, int32_t N, int32_t K, int32_t shift, int32_t act,
                     void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace with which ac_gemm_i8 (or ac_conv2d_i8 with this implicit-GEMM
 * shape) may split K (0 when no launch of the shape would split; operands that
 * run on the one-wave-per-tile kernel, tile code 32 below, leave it untouched).
 * Pure host arithmetic. */
size_t ac_gemm_i8_workspace_bytes(int32_t M, int32_t N, int32_t K);

/*
 * ac_gemm_i8 for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same operands, same plan and same result
 * (bit for bit) as ac_gemm_i8 with a workspace of ac_gemm_i8_workspace_bytes(M, N, K) bytes; the int32 partial
 * sums of a cut K range go through a buffer of AC_STATIC_SCRATCH_BYTES bytes that is part of the library's
 * device code (every GPU that runs the library holds its own copy until the process ends).  The call allocates
 * and frees nothing and calls no allocating routine; the first call on a GPU whose plan cuts K resolves that
 * GPU's copy of the buffer (one symbol lookup, no stream work), so make one such call before a capture.
 *   - A shape whose partial sums need more than AC_STATIC_SCRATCH_BYTES returns AC_ERR_WORKSPACE and nothing is
 *     launched (ac_gemm_i8_workspace_bytes tells in advance); shapes the library does not cut never touch the buffer.
 *   - Nothing in the buffer has to start at zero: every partial sum that is read was written by the same call.
 *   - All calls on one GPU share that GPU's buffer: calls that may overlap in time on one GPU (different streams,
 *     or graphs replayed concurrently) race on it and must be serialised by the caller.
 *   - The GPU that is current at the call must be the one `stream` belongs to.
 * Validation, error codes and operand rules otherwise as for ac_gemm_i8.
 */
#define AC_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
ac_status ac_gemm_i8_static(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                            const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                            int32_t M, int32_t N, int32_t K, int32_t shift, int32_t act, void* stream);

/*
 * int8 GEMM with the raw accumulator as output: C32[i][j] = sum_k A[i][k] * B[k][j] + bias(i, j) in int32,
 * with no scaling and no activation.  This is the accumulator-type read of the paper's accelerator
 * (Appendix C, Fig. 15: bit 29 of an accumulator read address selects the full accumulator value and skips
 * activation and scaling).  Operands and bias as for ac_gemm_i8; C is int32, M x N, row stride ldc >= N.
 */
ac_status ac_gemm_i8_acc32(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                           const int32_t* bias, int64_t bias_ld, int32_t* C, int64_t ldc,
                           int32_t M, int32_t N, int32_t K, void* stream);

/*
 * ac_gemm_i8 with transposed operands (the A_transpose / B_transpose fields of config_ex, Appendix C Fig. 14).
 *   trans_a != 0: A points to A^T, a K x M row-major array with row stride lda >= M
 *   trans_b != 0: B points to B^T, an N x K row-major array with row stride ldb >= K
 * Everything else (bias, output stage, C, error behaviour) as for ac_gemm_i8; with both flags zero the call
 * is ac_gemm_i8 without a workspace.  An operand is staged in LDS in its memory order and the transposition
 * happens in the LDS read.  Operands that qualify for the direct-to-LDS kernels (16-byte aligned base pointers
 * and row pitches; M (when trans_a), N and K multiples of 16) run on those, at the rate of the untransposed
 * product and never with a cut K range; anything else, any alignment included, on a register-staged kernel.
 */
ac_status ac_gemm_i8_t(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                       const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                       int32_t M, int32_t N, int32_t K, int32_t shift, int32_t act,
                       int32_t trans_a, int32_t trans_b, void* stream);

/*
 * int8 2-D convolution (the convolution workload of Section 4.4.2) computed
 * as an implicit GEMM with M = Nb*OH*OW, N = Cout, K = KH*KW*Cin, followed by
 * the same output stage as ac_gemm_i8:
 *
 *   out[n][oh][ow][co] = stage( bias[co] + sum_{kh,kw,ci}
 *        in[n][oh*stride - pad + kh][ow*stride - pad + kw][ci] * w[kh][kw][ci][co] )
 *
 * Taps outside the image read as zero.  OH = (H + 2*pad - KH) / stride + 1
 * (integer division), OW likewise.
 *
 *   in    device, int8, [Nb][H][W][Cin]      (dense NHWC)
 *   w     device, int8, [KH][KW][Cin][Cout]  (dense; the K x N matrix of the GEMM)
 *   bias  device, int32, [Cout], or NULL
 *   out   device, int8, [Nb][OH][OW][Cout]   (dense NHWC; written, never read)
 *   stride >= 1, pad >= 0, KH <= H + 2*pad, KW <= W + 2*pad, else AC_ERR_SHAPE.
 *   workspace: as for ac_gemm_i8 with the implicit-GEMM shape.
 */
ac_status ac_conv2d_i8(const int8_t* in, const int8_t* w, const int32_t* bias, int8_t* out,
                       int32_t Nb, int32_t H, int32_t W, int32_t Cin, int32_t Cout,
                       int32_t KH, int32_t KW, int32_t stride, int32_t pad,
                       int32_t shift, int32_t act,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * bf16 GEMM with fp32 accumulation and fp32 output (the square GEMM of
 * Appendix A Table 5, at the reduced input precision Section 4.6 reports as
 * the route to the matrix units):
 *
 *   C = alpha * (A . B) + beta * C
 *
 *   A  device, bf16 bit patterns (uint16), M x K, row stride lda >= K
 *   B  device, bf16 bit patterns,          K x N, row stride ldb >= N
 *   C  device, fp32, M x N, row stride ldc >= N; read only when beta != 0
 *      (with beta == 0 it may hold anything, NaN included)
 *   K == 0 gives C = beta * C.
 * Products are exact in fp32; sums are accumulated in fp32 in an unspecified
 * order.  Shapes with few output tiles and a deep K are cut along K (see the
 * planned launches below) where the library's estimate, the cost of the
 * combining atomic adds included, is at least a fifth below that of the best
 * uncut plan: the slices then add into C with fp32 atomic adds, and the sums
 * may differ in the last bits from run to run (ac_gemm_bf16_ws with a
 * workspace gives the same bits every run).  C must be ordinary device memory
 * as the conventions above say: the atomic adds are the hardware's own.
 */
ac_status ac_gemm_bf16(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb,
                       float* C, int64_t ldc, int32_t M, int32_t N, int32_t K,
                       float alpha, float beta, void* stream);

/*
 * ac_gemm_bf16 with an optional device workspace (same operands and result).  Where ac_gemm_bf16 cuts K, its
 * slices add into C with atomic adds in no fixed order; with a workspace of at least
 * ac_gemm_bf16_workspace_bytes(M, N, K) bytes (16-byte aligned) the slices leave fp32 partial products there and
 * a second kernel sums them in slice order, so the result is the same on every run.  The workspace rules are
 * those of ac_gemm_i8: contents unspecified on entry and exit, not shared by concurrent calls, NULL / 0 always
 * accepted (then the call is ac_gemm_bf16), too small or misaligned gives AC_ERR_WORKSPACE.  Operands that do
 * not qualify for the direct-to-LDS kernels (see the planned launches) are not cut and leave the workspace unused.
 */
ac_status ac_gemm_bf16_ws(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb,
                          float* C, int64_t ldc, int32_t M, int32_t N, int32_t K,
                          float alpha, float beta, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace with which ac_gemm_bf16_ws sums its K slices in a fixed order for this shape (0 when the
 * shape is not cut).  Pure host arithmetic. */
size_t ac_gemm_bf16_workspace_bytes(int32_t M, int32_t N, int32_t K);

/*
 * Batched small fp32 linear algebra (the fine-grained workload of Section
 * 4.4.3: small dense products chained with matrix-vector products and
 * element-wise adds), for each item b independently:
 *
 *   C_b = A_b . B_b                 (n x n)
 *   y_b = C_b . x_b + d_b           (uses the unrounded-in-between fp32 C_b)
 *
 *   A, B  device, fp32, [batch][n][n] dense
 *   C     device, fp32, [batch][n][n], or NULL to skip storing the product
 *   x     device, fp32, [batch][n], or NULL to skip the matrix-vector stage
 *   d     device, fp32, [batch][n], or NULL for no add
 *   y     device, fp32, [batch][n]; required iff x != NULL
 *   1 <= n <= 16; at least one of C, y must be requested.
 */
ac_status ac_batched_gemm_f32(const float* A, const float* B, float* C,
                              const float* x, const float* d, float* y,
                              int32_t n, int64_t batch, void* stream);

/*
 * Forward pass of the TinyMPC primal update (Appendix D.2), batched over independent problems that
 * share the three model matrices:
 *
 *   u[i]   = -Kinf . x[i] - d[i]
 *   x[i+1] =  Adyn . x[i] + Bdyn . u[i]          i = 0 .. horizon-1,  x[0] = x0
 *
 *   Adyn   device, fp32, [nx][nx]     Bdyn  device, fp32, [nx][nu]     Kinf  device, fp32, [nu][nx]
 *   x0     device, fp32, [batch][nx]
 *   d      device, fp32, [batch][horizon][nu]
 *   u      device, fp32, [batch][horizon][nu]   (written)
 *   x_out  device, fp32, [batch][horizon + 1][nx], or NULL: the state trajectory x[0..horizon]; when NULL the
 *          state after the last control, which the paper notes is never used, is not computed
 *   1 <= nx, nu <= 16 (the paper's problem has nx = 12, nu = 4, horizon = 5); horizon == 0 or batch == 0
 *   return AC_OK without a launch.  Arithmetic is fp32 throughout.  With nx = 12, nu = 4 and x0, d, u, x_out
 *   16-byte aligned the call runs on the matrix units: u[i] is substituted into the state update,
 *   [x[i+1]; u[i]] = [Adyn - Bdyn Kinf, -Bdyn; -Kinf, -I] . [x[i]; d[i]], with Adyn - Bdyn Kinf formed first (four
 *   fused multiply-adds per entry) and the sums of a product in the matrix unit's order; this equals the
 *   recurrence in exact arithmetic (and bit for bit on small-integer data) and differs from it by rounding, a few
 *   units in the last place per step.  Every other case evaluates the recurrence as written, each sum a fused
 *   multiply-add chain in ascending index order.
 */
ac_status ac_tinympc_forward_f32(const float* Adyn, const float* Bdyn, const float* Kinf,
                                 const float* x0, const float* d, float* u, float* x_out,
                                 int32_t nx, int32_t nu, int32_t horizon, int64_t batch, void* stream);

/*
 * Planned launches: the caller, not the library, names the block tile and the K split.
 *
 * The paper's search keeps a candidate only if it is still correct and ranks the survivors by
 * measured latency (Section 3.3); on this chip the candidates of a GEMM are its block tile and K split.  These
 * entry points run one named candidate so that a tuner can time each of them on the caller's own shape; the
 * results are those of ac_gemm_i8 / ac_gemm_bf16 (bit for bit for int8; for bf16 up to the summation order).
 *
 *   tile    block tile code: 64, 128, 256 = square tile of that edge; 192 = the tile of 256 rows x 128 columns;
 *           int8 only: 320 / 160 = the weight-stationary kernel with 256- / 128-row tiles (a 64-column block of
 *           B stays in LDS for all of K while tiles of A stream past it, the arrangement of the paper's best
 *           accelerator schedule, Appendix D.1).  It takes splits == 1, operands that qualify for the
 *           direct-to-LDS kernels (below), no bias or a bias row (bias_ld == 0), and K <= 1536 (320) / 2048 (160).
 *           int8 only: 32 = one wave per 32 x 32 output tile, one to four independent waves per workgroup and
 *           no barrier anywhere, for the accelerator-sized layers of Sections 4.4.1 and 4.4.2 whose whole
 *           launch lasts a few microseconds.  It takes operands that qualify for the direct-to-LDS kernels and
 *           K a multiple of 64, at least 64 (K slices, splits > 1, are whole 64-byte K tiles; every (tile,
 *           slice) is then a wave of its own).  ac_gemm_i8 and ac_conv2d_i8 pick it, uncut, for such operands
 *           where it measured ahead of every tiled plan: the fewer the tiles of 32 x 32, the deeper the K (up
 *           to 512 tiles K <= 1024, up to 1024 K <= 384, up to 2048 K <= 192, for a convolution K <= 640).
 *           ac_conv2d_i8_planned only: 321 / 161 = the convolution patch kernel with units of 256 / 128 output
 *           pixels: the weights of a 64-channel block AND the image patch a unit needs are both held in LDS, so
 *           every input pixel is fetched once per unit instead of once per kernel tap.  It takes splits == 1,
 *           Cin a multiple of 32, K <= 2048, out 16-byte aligned with Cout a multiple of 16, and a patch that
 *           fits: 2 x (patch rows x patch width x (Cin + 16)) + 64 K bytes <= 160 KB.
 *   splits  1 = no split; n > 1 cuts the K range into at most n slices of equal whole K tiles (64 bytes of K
 *           per tile for tiles 256 and 32, 128 bytes otherwise), each slice a workgroup (tile 32: a wave) of its own.  Needs operands
 *           that qualify for the direct-to-LDS kernels: base pointers and row pitches of A and B multiples of
 *           16 bytes, K and N multiples of 16 (int8) or 8 (bf16) elements, C 4-byte (int8) or 16-byte (bf16)
 *           aligned with ldc a multiple of 4, and row pitches below 13 MB (A) and 33 MB (B): a tile's rows are
 *           addressed with 32-bit byte offsets from the tile's first row.
 *           int8: slices leave int32 partial sums in `workspace`, which must hold
 *           ac_gemm_i8_planned_workspace_bytes() bytes; a second kernel sums them and applies the output stage.
 *           bf16, with a workspace of ac_gemm_bf16_planned_workspace_bytes() bytes: slices leave fp32 partial
 *           products there and a second kernel sums them in slice order and applies alpha / beta (the result
 *           is the same on every run).  bf16, workspace NULL / 0: a first kernel sets C = beta * C, then every
 *           slice adds alpha * (its product) with fp32 atomic adds, in no fixed order (slow for large M * N).
 *           Workspace rules as for ac_gemm_i8: 16-byte aligned, large enough, else AC_ERR_WORKSPACE.
 *   AC_ERR_PLAN: unknown tile code, splits < 1 or larger than the number of K tiles, or splits > 1 / a
 *           weight-stationary tile / tile 32 with operands that do not qualify.  Everything else as for the unplanned call.
 * ac_conv2d_i8_planned is ac_conv2d_i8 with the tile and K split of its implicit GEMM (M = Nb OH OW, N = Cout,
 *           K = KH KW Cin) named by the caller; "qualify" there means 16-byte aligned in / w, Cin and Cout
 *           multiples of 16, out 4-byte aligned; workspace size from ac_gemm_i8_planned_workspace_bytes(M, N, K, ...).
 * ac_gemm_*_auto_plan report what the unplanned call would choose for a shape (pure host arithmetic).
 * Operands that do not qualify for the direct-to-LDS kernels run on a generic kernel with square tiles, which
 * takes code 192 as 128.
 */
ac_status ac_gemm_i8_planned(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb,
                             const int32_t* bias, int64_t bias_ld, int8_t* C, int64_t ldc,
                             int32_t M, int32_t N, int32_t K, int32_t shift, int32_t act,
                             void* workspace, size_t workspace_bytes, int32_t tile, int32_t splits, void* stream);
size_t ac_gemm_i8_planned_workspace_bytes(int32_t M, int32_t N, int32_t K, int32_t tile, int32_t splits);
ac_status ac_conv2d_i8_planned(const int8_t* in, const int8_t* w, const int32_t* bias, int8_t* out,
                               int32_t Nb, int32_t H, int32_t W, int32_t Cin, int32_t Cout,
                               int32_t KH, int32_t KW, int32_t stride, int32_t pad,
                               int32_t shift, int32_t act,
                               void* workspace, size_t workspace_bytes, int32_t tile, int32_t splits, void* stream);
ac_status ac_gemm_bf16_planned(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb,
                               float* C, int64_t ldc, int32_t M, int32_t N, int32_t K,
                               float alpha, float beta, void* workspace, size_t workspace_bytes,
                               int32_t tile, int32_t splits, void* stream);
size_t ac_gemm_bf16_planned_workspace_bytes(int32_t M, int32_t N, int32_t K, int32_t tile, int32_t splits);
void ac_gemm_i8_auto_plan(int32_t M, int32_t N, int32_t K, int32_t have_workspace, int32_t* tile, int32_t* splits);
void ac_gemm_bf16_auto_plan(int32_t M, int32_t N, int32_t K, int32_t* tile, int32_t* splits);

/* Static, NUL-terminated description of a status code. */
const char* ac_status_string(ac_status status);

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t ac_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AC_H_ */
