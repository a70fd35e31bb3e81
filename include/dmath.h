/*
 * dmath.h - C ABI of the MI355X-native per-GPU dense kernels of a distributed
 * math library (dMath, arXiv 1604.01416).
 *
 * The paper's distributed matrix multiplication (section "Matrix Multiplication")
 * has every worker issue, per stage, one asynchronous dense multiply on blocks
 * it holds, accumulating into its block of C; its DNN pipeline adds forward
 * convolutions that run data-parallel with no communication (abstract, section
 * "Introduction").  This library is that per-GPU work and nothing else, on one
 * gfx950 device, in the three storage precisions of section "Precisions": FP32
 * (dmath_gemm, dmath_gemm_panels, the convolutions: FP32 in, FP32 MFMA accumulate,
 * FP32 out), IEEE half storage with FP32 arithmetic (dmath_hgemm) and FP64
 * (dmath_dgemm).
 *
 * General rules for every entry point
 *   - All matrix / tensor pointers are DEVICE pointers owned by the caller, to
 *     FP32 data unless the entry point says otherwise (binary16 bit patterns for
 *     dmath_hgemm, FP64 for dmath_dgemm); scalars are passed by value from the host.
 *   - `stream` is a hipStream_t passed as void*; NULL means the default stream.
 *     Calls enqueue work on that stream and return without synchronising.
 *   - The library allocates no device memory.  Kernels that need scratch use the
 *     workspace handed over with dmath_set_workspace(), or fall back to a path
 *     that needs none.
 *   - Arguments are validated before anything is launched; a call that returns
 *     an error has not touched its outputs.  dmath_last_error_arg() gives the
 *     1-based position of the offending argument of the last failed call made
 *     by the calling thread.
 *   - Outputs must not overlap inputs.
 *   - Results are deterministic: the same call on the same data gives the same
 *     bits (no atomics in any reduction).
 */
#ifndef DMATH_H
#define DMATH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DMATH_OK = 0,
    DMATH_ERR_INVALID_ARG = 1, /* negative size, bad leading dimension, bad enum */
    DMATH_ERR_NULL_PTR = 2,    /* NULL operand that the call would have to touch */
    DMATH_ERR_UNSUPPORTED = 3, /* valid request outside what is implemented */
    DMATH_ERR_LAUNCH = 4,      /* the HIP runtime refused the launch */
    DMATH_ERR_WORKSPACE = 5    /* workspace pointer / size inconsistent */
} dmath_status;

typedef enum { DMATH_OP_N = 0, DMATH_OP_T = 1 } dmath_op;

/*
 * Local block multiply, the GEMM each worker runs per stage (section "Matrix
 * Multiplication"; one-GPU column of table "Matrix Multiplication Performance";
 * the transposed forms are the variants that section mentions and the fully
 * connected layer products Y = W^T X, grad X = W grad Y of figure
 * "cyclic_gemm_cache_fwd"):
 *
 *     C[M x N] = alpha * op(A)[M x K] * op(B)[K x N] + beta * C
 *
 * ROW-MAJOR storage.  transA == N: A is stored M x K, element (i,k) at
 * A[i*lda + k], lda >= max(1,K).  transA == T: A is stored K x M, element (i,k)
 * of op(A) at A[k*lda + i], lda >= max(1,M).  transB == N: B stored K x N,
 * ldb >= max(1,N); transB == T: B stored N x K, ldb >= max(1,K).  C is M x N
 * with ldc >= max(1,N).  Leading dimensions let a block be a window of a larger
 * row panel.  Any 4-byte aligned pointer and any legal leading dimension work;
 * 16-byte aligned pointers with leading dimensions that are multiples of 4 take
 * the fast path.  lda or ldb above 2^22 elements (a window of a row panel more than
 * 4 Mi elements wide) is served by kernels with 64-bit offsets on one tile
 * configuration (128 x 128; a configuration forced with dmath_set_override is
 * ignored for such a call), not by the shape-tuned ones.
 *
 * M == 0 or N == 0: nothing happens.  K == 0 or alpha == 0: C = beta*C and A, B
 * are not read (they may be NULL).  beta == 0: C is write-only, its old contents
 * (NaN, Inf) never reach the result.
 *
 * Errors: INVALID_ARG for a bad enum, negative size or short leading dimension;
 * NULL_PTR for a NULL operand that would be read or written; LAUNCH if the
 * runtime rejects the kernel launch.
 */
dmath_status dmath_gemm(dmath_op transA, dmath_op transB,
                        int64_t M, int64_t N, int64_t K,
                        float alpha, const float *A, int64_t lda,
                        const float *B, int64_t ldb,
                        float beta, float *C, int64_t ldc,
                        void *stream);

/*
 * dmath_gemm for callers that cannot allocate device memory or register a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, conventions,
 * kernels and results as dmath_gemm, but the scratch of split plans (K slices of a product with few
 * tiles, partial sums and counters of tail tiles) is an array of DMATH_NOALLOC_SCRATCH_BYTES that is
 * part of the library's device image: every GPU the library runs on holds one copy until the process
 * ends.  The call allocates nothing and frees nothing (no hipMalloc, no hipFree, no allocating library
 * routine), ignores the workspace registered with dmath_set_workspace, and only enqueues kernels; the
 * counters it needs at zero are cleared by a kernel on `stream`, not by a memset.
 *
 * A shape whose plan wants more scratch than that (dmath_gemm_workspace_bytes(...) >
 * DMATH_NOALLOC_SCRATCH_BYTES, e.g. 6144^3) is refused with WORKSPACE (dmath_last_error_arg() == 0)
 * before anything is launched, C untouched; it is not silently run on a slower plan.  All calls on one
 * GPU share that GPU's array, which keeps the last call's contents: calls that overlap in time on one
 * GPU (different streams, or different host threads) race and must be serialised by the caller.  The
 * first call on a device looks the array's address up (hipGetSymbolAddress) and should be made outside
 * stream capture; LAUNCH if that lookup fails.  Other errors as for dmath_gemm.
 */
#define DMATH_NOALLOC_SCRATCH_BYTES (32u << 20)
dmath_status dmath_gemm_noalloc(dmath_op transA, dmath_op transB,
                                int64_t M, int64_t N, int64_t K,
                                float alpha, const float *A, int64_t lda,
                                const float *B, int64_t ldb,
                                float beta, float *C, int64_t ldc,
                                void *stream);

/*
 * The same multiply for matrices kept in half-precision storage (section "Precisions": IEEE 16-bit
 * half floats halve the bytes stored and moved, while the arithmetic stays single precision):
 *
 *     C = half( alpha * op(A) * op(B) + beta * float(C) )
 *
 * A, B and C hold IEEE 754 binary16 bit patterns (uint16_t); every element is converted exactly to
 * FP32, products and sums are FP32 (MFMA) exactly as in dmath_gemm, and the result is rounded to half
 * once (to nearest even) when it is stored.  alpha and beta are FP32.  Leading dimensions count
 * elements.  The fast path needs 8-byte aligned pointers and leading dimensions that are multiples of
 * 4; anything 2-byte aligned works.  Conventions, errors and split-K workspace as for dmath_gemm (the
 * split-K slices are FP32); UNSUPPORTED if the rotated-image comparison configuration is forced.
 *
 * Two kernels implement it.  When A and B are 16-byte aligned, lda and ldb are multiples of 8, K is a
 * multiple of 32 and an operand stored along its own index (A for transA == T, B for transB == N) has a
 * multiple of 8 rows / columns, the FP16-input matrix instruction is used: products of two halves are
 * exact in FP32 and it accumulates in FP32, so it computes the same sums (in another order) at 16 times
 * the FP32 matrix rate.  Every other case runs the FP32 matrix instruction on operands widened on the
 * fly.  dmath_set_hgemm_path forces one of them for this thread's later calls: -1 automatic, 0 the
 * FP32 instruction; 1, 2 the FP16-input instruction with the 256 x 256 tile of 8 waves or the 128 x 128
 * tile of 4 waves (automatic: 1 for large outputs, 2 for small ones; forced: UNSUPPORTED when the
 * conditions do not hold).  With K a multiple of 64 the FP16-input kernel loads whole 128-byte lines
 * global -> LDS and runs on the 16x16x32 form of the instruction, otherwise it stages a K tile of 32
 * through registers on the 32x32x16 form.  A tile configuration forced with dmath_set_override also
 * selects the FP32 instruction.
 */
dmath_status dmath_hgemm(dmath_op transA, dmath_op transB,
                         int64_t M, int64_t N, int64_t K,
                         float alpha, const uint16_t *A, int64_t lda,
                         const uint16_t *B, int64_t ldb,
                         float beta, uint16_t *C, int64_t ldc,
                         void *stream);
dmath_status dmath_set_hgemm_path(int path);
/* Workspace dmath_hgemm would like for this shape (either kernel; 0 if it would not split). */
size_t dmath_hgemm_workspace_bytes(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K);

/*
 * The same multiply in double precision (section "Precisions": single and double precision are the
 * library's two nominal precisions): A, B, C, alpha and beta are FP64, products and sums are FP64 on
 * the double-precision matrix instruction.  Layout conventions, quick returns and error codes as for
 * dmath_gemm; any 8-byte aligned pointers and any legal leading dimensions are accepted.  A product
 * with few output tiles is cut into K slices when the registered workspace holds them (FP64 arrays of
 * M x N, added in slice order by a second kernel: results do not depend on timing); without a workspace
 * it runs unsplit on few compute units.  dmath_dgemm_workspace_bytes returns what the automatic plan
 * would like (0 if it would not split); a split factor forced with dmath_set_override applies here too.
 * dmath_set_dgemm_config forces one of the two tile configurations (0: 256 x 128, 1: 128 x 128;
 * -1 automatic) for this thread.
 */
dmath_status dmath_dgemm(dmath_op transA, dmath_op transB,
                         int64_t M, int64_t N, int64_t K,
                         double alpha, const double *A, int64_t lda,
                         const double *B, int64_t ldb,
                         double beta, double *C, int64_t ldc,
                         void *stream);
dmath_status dmath_set_dgemm_config(int tile_config);
size_t dmath_dgemm_workspace_bytes(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K);

/*
 * Accumulating sequence of block multiplies in one call (section "Matrix Multiplication": a worker's
 * block of C is the sum, over the stages, of products of the A and B blocks it holds at that stage;
 * section "Memory Management" and figure "cyclic_gemm_cache_fwd": with the blocks cached on the
 * device the whole sum runs without communication):
 *
 *     C[M x N] = alpha * sum_{p < npanels} op(A[p])[M x K] * op(B[p])[K x N] + beta * C
 *
 * A and B are HOST arrays of npanels DEVICE pointers, read before the call returns; every panel has
 * the same shape, orientation and leading dimension (conventions of dmath_gemm).  beta applies once.
 * When K is a multiple of 16 and the operands qualify for dmath_gemm's fast path (16-byte aligned
 * panels, leading dimensions multiples of 4) the whole sum is one kernel launch per 32 panels that
 * keeps the C tile in registers, so C is read and written once per launch instead of once per panel;
 * otherwise the call is the same as npanels accumulating dmath_gemm calls.  Rounding differs from
 * that sequence only in summation order.
 *
 * npanels == 0, K == 0 or alpha == 0: C = beta*C and no panel pointer is read.
 * Errors as for dmath_gemm; NULL_PTR also for a NULL entry of A (argument 8) or B (argument 10).
 */
dmath_status dmath_gemm_panels(dmath_op transA, dmath_op transB,
                               int64_t M, int64_t N, int64_t K, int64_t npanels,
                               float alpha, const float *const *A, int64_t lda,
                               const float *const *B, int64_t ldb,
                               float beta, float *C, int64_t ldc,
                               void *stream);

/*
 * Forward convolution (the DNN primitive of the abstract and of section
 * "Introduction"; the paper delegates its formula to the DNN library it calls,
 * so the usual DNN definition is used: cross-correlation, zero padding):
 *
 *     y[n][j][p][q] = alpha * sum_{c,r,s} x[n][c][p*stride_h + r - pad_h][q*stride_w + s - pad_w]
 *                                         * w[j][c][r][s]   +   beta * y[n][j][p][q]
 *
 * x is N x C x H x W, w is Kout x C x R x S, y is N x Kout x P x Q, all dense
 * and packed in that order, with P = (H + 2*pad_h - R)/stride_h + 1 and
 * Q = (W + 2*pad_w - S)/stride_w + 1 (integer division; the filter must fit:
 * H + 2*pad_h >= R, W + 2*pad_w >= S).  Taps that fall outside x count as zero.
 * Dilation 1, one group, no bias.  The product is evaluated as a matrix
 * multiply one of whose operands is generated on the fly from x; the unfolded
 * matrix is never stored.  When a workspace of at least Kout*C*R*S*4 bytes is
 * registered (dmath_set_workspace), C is a multiple of 16 and R*S <= 32, the
 * filters are first copied into it in tap-major order, which makes the
 * generated operand cheaper to address.  When the output tiles do not fill whole
 * rounds over the compute units, the tiles of the last, partial round are cut into
 * K slices whose partial sums and counters also live in the workspace (after the
 * filter copy); with no workspace, or one too small, the call runs without either.
 * A split-K factor forced with dmath_set_override does not apply to the forward
 * and backward-data convolutions (only such tail tiles are ever split there).
 *
 * Empty outputs (N, Kout, P or Q zero) are a no-op; C == 0 or alpha == 0 gives
 * y = beta*y without reading x or w; beta == 0 makes y write-only.
 *
 * Errors: INVALID_ARG for negative sizes, R or S < 1, strides < 1, negative
 * padding or a filter larger than the padded input; NULL_PTR as for dmath_gemm;
 * UNSUPPORTED if a tensor has 2^31 or more elements per image-channel plane set
 * that 32-bit in-kernel offsets cannot address.
 */
dmath_status dmath_conv2d_fwd(int64_t N, int64_t C, int64_t H, int64_t W,
                              int64_t Kout, int64_t R, int64_t S,
                              int64_t pad_h, int64_t pad_w,
                              int64_t stride_h, int64_t stride_w,
                              float alpha, const float *x, const float *w,
                              float beta, float *y, void *stream);

/*
 * Gradient of dmath_conv2d_fwd with respect to x (the backward pass of the same DNN primitive; the
 * paper's pipeline is forward and backward):
 *
 *     dx[n][c][h][w] = alpha * sum over (j, r, s) and the (p, q) with p*stride_h + r - pad_h == h and
 *                              q*stride_w + s - pad_w == w of  dy[n][j][p][q] * w[j][c][r][s]
 *                      + beta * dx[n][c][h][w]
 *
 * N, C, H, W, Kout, R, S, pads and strides describe the FORWARD convolution; dy is N x Kout x P x Q
 * with P, Q as defined there, w is Kout x C x R x S, dx is N x C x H x W.  It runs on the same kernels
 * as the forward pass with the roles of the channel dimensions exchanged, and always needs a registered
 * workspace of at least C*Kout*R*S*4 bytes (rounded up to 256) for the transposed filters: without one
 * it returns WORKSPACE.  Stride 1 with pads smaller than the filter takes the fast forward-style path;
 * other strides and pads use a general gather.  Conventions for empty tensors, alpha == 0 and beta == 0,
 * and the error codes are those of dmath_conv2d_fwd (argument positions likewise, dy in place of x and
 * dx in place of y).
 */
dmath_status dmath_conv2d_bwd_data(int64_t N, int64_t C, int64_t H, int64_t W,
                                   int64_t Kout, int64_t R, int64_t S,
                                   int64_t pad_h, int64_t pad_w,
                                   int64_t stride_h, int64_t stride_w,
                                   float alpha, const float *dy, const float *w,
                                   float beta, float *dx, void *stream);

/*
 * Gradient of dmath_conv2d_fwd with respect to the filters:
 *
 *     dw[j][c][r][s] = alpha * sum over (n, p, q) with the tap inside x of
 *                              dy[n][j][p][q] * x[n][c][p*stride_h + r - pad_h][q*stride_w + s - pad_w]
 *                      + beta * dw[j][c][r][s]
 *
 * Arguments describe the FORWARD convolution; x is N x C x H x W, dy is N x Kout x P x Q, dw is
 * Kout x C x R x S.  The reduction over all output pixels is long and the result small, so with a
 * registered workspace the sum is cut into K slices (dmath_gemm's plain split-K, sized like a GEMM with
 * M = Kout, N = C*R*S, K = N*P*Q: see dmath_gemm_workspace_bytes); without one it runs unsplit.
 * Conventions and error codes as for dmath_conv2d_fwd (argument 13 is x, 14 is dy, 16 is dw);
 * UNSUPPORTED if the rotated-image comparison configuration is forced.
 */
dmath_status dmath_conv2d_bwd_filter(int64_t N, int64_t C, int64_t H, int64_t W,
                                     int64_t Kout, int64_t R, int64_t S,
                                     int64_t pad_h, int64_t pad_w,
                                     int64_t stride_h, int64_t stride_w,
                                     float alpha, const float *x, const float *dy,
                                     float beta, float *dw, void *stream);

/*
 * Scratch for the split-K path of dmath_gemm (used when the output alone has
 * too few tiles to fill the device, as for the skinny products of a fully
 * connected layer).  dmath_gemm_workspace_bytes() returns how many bytes the
 * call with these arguments would like (0 if it would not split).
 * dmath_set_workspace() registers a caller-owned device buffer for the current
 * host thread's later calls; NULL / 0 removes it.  With no workspace, or one
 * that is too small, dmath_gemm silently uses a path that needs none.  The
 * buffer must stay valid, and must not be shared by calls running concurrently
 * on different streams.  WORKSPACE is returned for a NULL pointer with a
 * non-zero size or a pointer that is not 16-byte aligned.
 */
size_t dmath_gemm_workspace_bytes(dmath_op transA, dmath_op transB,
                                  int64_t M, int64_t N, int64_t K);
dmath_status dmath_set_workspace(void *device_ptr, size_t bytes);

/*
 * Tuning hook for benchmarks: force the tile configuration (index into the
 * library's table, see dmath_config_name) and the split-K factor used by later
 * dmath_gemm / dmath_conv2d_fwd calls of this thread.  -1 restores the automatic
 * choice.  A forced split-K larger than 1 still needs a workspace.  Returns
 * INVALID_ARG for an index outside the table.
 */
dmath_status dmath_set_override(int tile_config, int split_k);

/*
 * Which tile configuration and split-K factor dmath_gemm would use for this shape right now (given
 * this thread's workspace and override).  Host-side only, launches nothing.  tile_config receives -1
 * when the call would not run a tile kernel (empty output or K == 0).  Either pointer may be NULL.
 */
dmath_status dmath_gemm_plan(dmath_op transA, dmath_op transB, int64_t M, int64_t N, int64_t K,
                             int *tile_config, int *split_k);
int dmath_num_configs(void);
const char *dmath_config_name(int tile_config); /* NULL outside the table */

/*
 * Measurement hook: when device_ptr is not NULL it must point to 32 uint64 values (256 bytes) of
 * device memory; workgroups 0..7 of every later dmath_gemm tile kernel launched by this thread (the
 * first workgroup placed on each of the 8 dies, which clock independently) each write four of them:
 * the shader-clock counter and the fixed 100 MHz counter when the workgroup starts, and both again
 * when it ends.  (shader clocks elapsed) / (100 MHz ticks elapsed) * 100 MHz is the clock that die
 * ran at while the workgroup lived; the benchmark reports it next to the nominal 2.4 GHz.  Entries of
 * workgroups the launch does not have stay untouched.  NULL switches the hook off.  INVALID_ARG
 * unless 8-byte aligned.
 */
dmath_status dmath_set_clock_probe(void *device_ptr);

/* 1-based index of the argument rejected by this thread's last failed call, 0 if none. */
int dmath_last_error_arg(void);
const char *dmath_status_string(dmath_status status);
const char *dmath_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DMATH_H */
