/*
 * CPU oracle for the per-GPU dense kernels of a distributed math library
 * (dMath, arXiv 1604.01416).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path links, loads or calls
 * this file; it shares no code, header, table or helper with the HIP library.
 * It exists so that the GPU results can be checked against the plain
 * definitions of the operations, evaluated in FP64.
 *
 * What it computes
 *   - GEMM, the local block update every worker issues per stage of the cyclic
 *     matrix multiplication (section "Matrix Multiplication"; timed for one GPU
 *     in table "Matrix Multiplication Performance"), with the transposed
 *     variants the same section asks for and the fully-connected-layer forms of
 *     figure "cyclic_gemm_cache_fwd" (Y = W^T X, grad X = W grad Y):
 *         ref[i][j] = alpha * sum_{k<K} opA(i,k) * opB(k,j)  +  beta * C0[i][j]
 *     row-major storage, opA(i,k) = A[i*lda+k] (N) or A[k*lda+i] (T), same for B.
 *   - Forward convolution, the DNN primitive named in the abstract and in
 *     section "Introduction" (data-parallel, needs no communication); the paper
 *     leaves the formula to the DNN library it calls, so the reading used is the
 *     usual DNN one: cross-correlation (no kernel flip), zero padding, dilation
 *     1, one group, no bias, NCHW input, KCRS filters, NKPQ output:
 *         ref[n][j][p][q] = alpha * sum_{c,r,s} x[n][c][p*sh+r-ph][q*sw+s-pw] * w[j][c][r][s]
 *                           + beta * y0[n][j][p][q]
 *   - The two gradients of that convolution (its adjoints), the accumulating
 *     sum of several block products, and the GEMM on IEEE half-precision storage
 *     with wide accumulation (section "Precisions"): see the comment at each.
 *   - For all of them, the companion magnitude sum (same expression with every factor
 *     replaced by its absolute value) that the acceptance bound
 *         |gpu - ref| <= 4*K*2^-24 * mag + 1e-6
 *     needs.
 *
 * Conventions where the paper is silent (reference-BLAS ones): beta == 0 means
 * C0 / y0 is never read (NaN there does not propagate); alpha == 0 means A and B
 * (x and w) are never read.
 *
 * Arithmetic: inputs are FP32 and are promoted exactly to FP64; every product
 * and sum is FP64, terms added in ascending k (GEMM) or ascending (c, r, s)
 * (convolution).  No blocking, no reordering.  OpenMP only splits the
 * independent output rows / output planes across threads.
 *
 * Parity status: every function here is pinned by tests that do not use this
 * file to produce the expected value (integer-exact cases against int64
 * arithmetic, identity / permutation / rank-1 / all-ones closed forms,
 * transposition identities, delta filters, tap-count closed forms, brute force
 * in Python, and library float64 matmul / conv2d; for the gradients the adjoint
 * identity and torch.nn.grad; for the panel sum the product of concatenations;
 * for half storage numpy's own binary16 conversion on all 65536 patterns; for
 * double precision exact rational arithmetic and cancellation cases that FP64
 * accumulation gets wrong).  Each has a hand-worked fixture under
 * tests/golden/ where the paper prints no example of its own.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline double a_elem(const float *A, int64_t lda, int tA, int64_t i, int64_t k)
{
    return (double)(tA ? A[k * lda + i] : A[i * lda + k]);
}

static inline double b_elem(const float *B, int64_t ldb, int tB, int64_t k, int64_t j)
{
    return (double)(tB ? B[j * ldb + k] : B[k * ldb + j]);
}

/*
 * Full GEMM.  ref and mag are dense M x N (row stride N) FP64 outputs; mag may
 * be NULL.  C0 may be NULL when beta == 0.  Returns 0, or 1 on a bad argument.
 */
int oracle_gemm(int transA, int transB, int64_t M, int64_t N, int64_t K,
                double alpha, const float *A, int64_t lda,
                const float *B, int64_t ldb,
                double beta, const float *C0, int64_t ldc,
                double *ref, double *mag)
{
    if (M < 0 || N < 0 || K < 0 || !ref) return 1;
    if (beta != 0.0 && !C0 && M > 0 && N > 0) return 1;
    if (alpha != 0.0 && K > 0 && M > 0 && N > 0 && (!A || !B)) return 1;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        double *s = (double *)calloc((size_t)(N > 0 ? N : 1), sizeof(double));
        double *t = (double *)calloc((size_t)(N > 0 ? N : 1), sizeof(double));
        if (!s || !t) {
#pragma omp atomic write
            fail = 1;
            free(s);
            free(t);
            continue;
        }
        if (alpha != 0.0) {
            for (int64_t k = 0; k < K; ++k) {
                const double a = a_elem(A, lda, transA, i, k);
                const double fa = fabs(a);
                for (int64_t j = 0; j < N; ++j) {
                    const double b = b_elem(B, ldb, transB, k, j);
                    s[j] += a * b;
                    t[j] += fa * fabs(b);
                }
            }
        }
        for (int64_t j = 0; j < N; ++j) {
            double r = (alpha != 0.0) ? alpha * s[j] : 0.0;
            double m = (alpha != 0.0) ? fabs(alpha) * t[j] : 0.0;
            if (beta != 0.0) {
                const double c0 = (double)C0[i * ldc + j];
                r += beta * c0;
                m += fabs(beta) * fabs(c0);
            }
            ref[i * N + j] = r;
            if (mag) mag[i * N + j] = m;
        }
        free(s);
        free(t);
    }
    return fail;
}

/*
 * GEMM at chosen output positions (pi[p], pj[p]), p < npts: the same sums, one
 * output element at a time, so that problems too large for the full routine can
 * still be checked on a sample.
 */
int oracle_gemm_points(int transA, int transB, int64_t M, int64_t N, int64_t K,
                       double alpha, const float *A, int64_t lda,
                       const float *B, int64_t ldb,
                       double beta, const float *C0, int64_t ldc,
                       int64_t npts, const int64_t *pi, const int64_t *pj,
                       double *ref, double *mag)
{
    if (M < 0 || N < 0 || K < 0 || npts < 0 || !ref) return 1;
    for (int64_t p = 0; p < npts; ++p)
        if (pi[p] < 0 || pi[p] >= M || pj[p] < 0 || pj[p] >= N) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < npts; ++p) {
        const int64_t i = pi[p], j = pj[p];
        double s = 0.0, t = 0.0;
        if (alpha != 0.0) {
            for (int64_t k = 0; k < K; ++k) {
                const double a = a_elem(A, lda, transA, i, k);
                const double b = b_elem(B, ldb, transB, k, j);
                s += a * b;
                t += fabs(a) * fabs(b);
            }
        }
        double r = (alpha != 0.0) ? alpha * s : 0.0;
        double m = (alpha != 0.0) ? fabs(alpha) * t : 0.0;
        if (beta != 0.0) {
            const double c0 = (double)C0[i * ldc + j];
            r += beta * c0;
            m += fabs(beta) * fabs(c0);
        }
        ref[p] = r;
        if (mag) mag[p] = m;
    }
    return 0;
}

/*
 * Accumulating sequence of block products into one C block (section "Matrix
 * Multiplication": a worker's C block is the sum, over the stages, of the
 * products of the A and B blocks it holds at each stage; section "Memory
 * Management" / figure "cyclic_gemm_cache_fwd": with the blocks cached, the
 * whole sum runs locally):
 *
 *     C = alpha * sum_{p < npanels} op(A_p)[M x K] * op(B_p)[K x N] + beta * C0
 *
 * A and B are arrays of npanels pointers; every panel has the same K and
 * leading dimension.  With pi == NULL all M x N elements are produced (ref, mag
 * dense, row stride N); otherwise only the npts positions (pi[t], pj[t]).
 * beta is applied once to C0, not once per panel.
 */
int oracle_gemm_panels(int transA, int transB, int64_t M, int64_t N, int64_t K, int64_t npanels,
                       double alpha, const float *const *A, int64_t lda,
                       const float *const *B, int64_t ldb,
                       double beta, const float *C0, int64_t ldc,
                       int64_t npts, const int64_t *pi, const int64_t *pj,
                       double *ref, double *mag)
{
    if (M < 0 || N < 0 || K < 0 || npanels < 0 || npts < 0 || !ref) return 1;
    if (beta != 0.0 && !C0 && M > 0 && N > 0) return 1;
    const int product = alpha != 0.0 && K > 0 && npanels > 0 && M > 0 && N > 0;
    if (product) {
        if (!A || !B) return 1;
        for (int64_t p = 0; p < npanels; ++p)
            if (!A[p] || !B[p]) return 1;
    }
    const int64_t total = pi ? npts : M * N;
    if (pi)
        for (int64_t t = 0; t < npts; ++t)
            if (pi[t] < 0 || pi[t] >= M || pj[t] < 0 || pj[t] >= N) return 1;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < total; ++t) {
        const int64_t i = pi ? pi[t] : t / N, j = pi ? pj[t] : t % N;
        double s = 0.0, m = 0.0;
        if (product) {
            for (int64_t p = 0; p < npanels; ++p)
                for (int64_t k = 0; k < K; ++k) {
                    const double a = a_elem(A[p], lda, transA, i, k);
                    const double b = b_elem(B[p], ldb, transB, k, j);
                    s += a * b;
                    m += fabs(a) * fabs(b);
                }
        }
        double r = product ? alpha * s : 0.0;
        double g = product ? fabs(alpha) * m : 0.0;
        if (beta != 0.0) {
            const double c0 = (double)C0[i * ldc + j];
            r += beta * c0;
            g += fabs(beta) * fabs(c0);
        }
        ref[t] = r;
        if (mag) mag[t] = g;
    }
    return 0;
}

/*
 * IEEE 754 binary16 -> double, from the format: 1 sign bit, 5 exponent bits
 * (bias 15), 10 fraction bits; exponent 0 is zero / subnormal (fraction * 2^-24),
 * exponent 31 is infinity (fraction 0) or NaN.
 */
double oracle_half_to_double(uint16_t h)
{
    const int sign = (h >> 15) & 1, e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);
    return sign ? -v : v;
}

static inline double ha_elem(const uint16_t *A, int64_t lda, int tA, int64_t i, int64_t k)
{
    return oracle_half_to_double(tA ? A[k * lda + i] : A[i * lda + k]);
}

static inline double hb_elem(const uint16_t *B, int64_t ldb, int tB, int64_t k, int64_t j)
{
    return oracle_half_to_double(tB ? B[j * ldb + k] : B[k * ldb + j]);
}

/*
 * GEMM on half-precision storage (section "Precisions": matrices stored as IEEE
 * half floats, the arithmetic done in a wider precision):
 *
 *     ref[i][j] = alpha * sum_k opA(i,k) * opB(k,j) + beta * C0[i][j]
 *
 * with A, B, C0 arrays of binary16 bit patterns, each converted exactly to FP64;
 * ref and mag are the unrounded FP64 values (the rounding of the stored result
 * to half is the caller's tolerance, not applied here).  pi == NULL: all M x N
 * elements (row stride N); else only the npts positions (pi[t], pj[t]).
 */
int oracle_hgemm(int transA, int transB, int64_t M, int64_t N, int64_t K,
                 double alpha, const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb,
                 double beta, const uint16_t *C0, int64_t ldc,
                 int64_t npts, const int64_t *pi, const int64_t *pj,
                 double *ref, double *mag)
{
    if (M < 0 || N < 0 || K < 0 || npts < 0 || !ref) return 1;
    if (beta != 0.0 && !C0 && M > 0 && N > 0) return 1;
    const int product = alpha != 0.0 && K > 0 && M > 0 && N > 0;
    if (product && (!A || !B)) return 1;
    const int64_t total = pi ? npts : M * N;
    if (pi)
        for (int64_t t = 0; t < npts; ++t)
            if (pi[t] < 0 || pi[t] >= M || pj[t] < 0 || pj[t] >= N) return 1;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < total; ++t) {
        const int64_t i = pi ? pi[t] : t / N, j = pi ? pj[t] : t % N;
        double s = 0.0, m = 0.0;
        if (product) {
            for (int64_t k = 0; k < K; ++k) {
                const double a = ha_elem(A, lda, transA, i, k);
                const double b = hb_elem(B, ldb, transB, k, j);
                s += a * b;
                m += fabs(a) * fabs(b);
            }
        }
        double r = product ? alpha * s : 0.0;
        double g = product ? fabs(alpha) * m : 0.0;
        if (beta != 0.0) {
            const double c0 = oracle_half_to_double(C0[i * ldc + j]);
            r += beta * c0;
            g += fabs(beta) * fabs(c0);
        }
        ref[t] = r;
        if (mag) mag[t] = g;
    }
    return 0;
}

/*
 * Double-precision GEMM (section "Precisions": single and double precision are
 * the library's nominal precisions).  Inputs are FP64; to stand above the
 * arithmetic it checks, every product and sum is carried in long double (the
 * x87 80-bit format here: 64-bit significand, so the accumulated rounding error
 * is 2^-11 of what FP64 accumulation of the same terms may commit), and rounded
 * to double once at the end.  mag is the same sum over absolute values.
 *
 *     ref[i][j] = alpha * sum_k opA(i,k) * opB(k,j) + beta * C0[i][j]
 *
 * pi == NULL: all M x N elements (row stride N); else the npts positions.
 */
int oracle_dgemm(int transA, int transB, int64_t M, int64_t N, int64_t K,
                 double alpha, const double *A, int64_t lda,
                 const double *B, int64_t ldb,
                 double beta, const double *C0, int64_t ldc,
                 int64_t npts, const int64_t *pi, const int64_t *pj,
                 double *ref, double *mag)
{
    if (M < 0 || N < 0 || K < 0 || npts < 0 || !ref) return 1;
    if (beta != 0.0 && !C0 && M > 0 && N > 0) return 1;
    const int product = alpha != 0.0 && K > 0 && M > 0 && N > 0;
    if (product && (!A || !B)) return 1;
    const int64_t total = pi ? npts : M * N;
    if (pi)
        for (int64_t t = 0; t < npts; ++t)
            if (pi[t] < 0 || pi[t] >= M || pj[t] < 0 || pj[t] >= N) return 1;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < total; ++t) {
        const int64_t i = pi ? pi[t] : t / N, j = pi ? pj[t] : t % N;
        long double s = 0.0L, m = 0.0L;
        if (product) {
            for (int64_t k = 0; k < K; ++k) {
                const long double a = transA ? A[k * lda + i] : A[i * lda + k];
                const long double b = transB ? B[j * ldb + k] : B[k * ldb + j];
                s += a * b;
                m += fabsl(a) * fabsl(b);
            }
        }
        long double r = product ? (long double)alpha * s : 0.0L;
        long double g = product ? fabsl((long double)alpha) * m : 0.0L;
        if (beta != 0.0) {
            const long double c0 = C0[i * ldc + j];
            r += (long double)beta * c0;
            g += fabsl((long double)beta) * fabsl(c0);
        }
        ref[t] = (double)r;
        if (mag) mag[t] = (double)g;
    }
    return 0;
}

int oracle_long_double_digits(void) { return __LDBL_MANT_DIG__; }

static inline int64_t conv_out_dim(int64_t in, int64_t pad, int64_t filt, int64_t stride)
{
    const int64_t span = in + 2 * pad - filt;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* One output element of the direct convolution: loops over (c, r, s) only. */
static inline void conv_point(int64_t C, int64_t H, int64_t W, int64_t R, int64_t S,
                              int64_t ph, int64_t pw, int64_t sh, int64_t sw,
                              const float *x_img, const float *w_filt,
                              int64_t p, int64_t q, double *sum, double *msum)
{
    double s_acc = 0.0, t_acc = 0.0;
    for (int64_t c = 0; c < C; ++c)
        for (int64_t r = 0; r < R; ++r)
            for (int64_t s = 0; s < S; ++s) {
                const int64_t ih = p * sh + r - ph;
                const int64_t iw = q * sw + s - pw;
                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                const double xv = (double)x_img[(c * H + ih) * W + iw];
                const double wv = (double)w_filt[(c * R + r) * S + s];
                s_acc += xv * wv;
                t_acc += fabs(xv) * fabs(wv);
            }
    *sum = s_acc;
    *msum = t_acc;
}

/*
 * Full direct convolution (loops n, j, p, q, c, r, s).  ref / mag are dense
 * N x Kout x P x Q FP64; mag may be NULL; y0 may be NULL when beta == 0.
 */
int oracle_conv2d_fwd(int64_t N, int64_t C, int64_t H, int64_t W,
                      int64_t Kout, int64_t R, int64_t S,
                      int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w,
                      double alpha, const float *x, const float *w,
                      double beta, const float *y0, double *ref, double *mag)
{
    if (N < 0 || C < 0 || H < 0 || W < 0 || Kout < 0 || R < 1 || S < 1) return 1;
    if (pad_h < 0 || pad_w < 0 || stride_h < 1 || stride_w < 1 || !ref) return 1;
    const int64_t P = conv_out_dim(H, pad_h, R, stride_h);
    const int64_t Q = conv_out_dim(W, pad_w, S, stride_w);
    if (beta != 0.0 && !y0 && N * Kout * P * Q > 0) return 1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < Kout; ++j) {
            const float *x_img = x + n * C * H * W;
            const float *w_filt = w + j * C * R * S;
            for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q) {
                    const int64_t o = ((n * Kout + j) * P + p) * Q + q;
                    double s = 0.0, t = 0.0;
                    if (alpha != 0.0)
                        conv_point(C, H, W, R, S, pad_h, pad_w, stride_h, stride_w,
                                   x_img, w_filt, p, q, &s, &t);
                    double r = (alpha != 0.0) ? alpha * s : 0.0;
                    double m = (alpha != 0.0) ? fabs(alpha) * t : 0.0;
                    if (beta != 0.0) {
                        const double c0 = (double)y0[o];
                        r += beta * c0;
                        m += fabs(beta) * fabs(c0);
                    }
                    ref[o] = r;
                    if (mag) mag[o] = m;
                }
        }
    return 0;
}

/* Convolution at chosen flat output offsets idx[p] into the N x Kout x P x Q array. */
int oracle_conv2d_fwd_points(int64_t N, int64_t C, int64_t H, int64_t W,
                             int64_t Kout, int64_t R, int64_t S,
                             int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w,
                             double alpha, const float *x, const float *w,
                             double beta, const float *y0,
                             int64_t npts, const int64_t *idx, double *ref, double *mag)
{
    if (N < 0 || C < 0 || H < 0 || W < 0 || Kout < 0 || R < 1 || S < 1) return 1;
    if (pad_h < 0 || pad_w < 0 || stride_h < 1 || stride_w < 1 || !ref || npts < 0) return 1;
    const int64_t P = conv_out_dim(H, pad_h, R, stride_h);
    const int64_t Q = conv_out_dim(W, pad_w, S, stride_w);
    const int64_t total = N * Kout * P * Q;
    for (int64_t t = 0; t < npts; ++t)
        if (idx[t] < 0 || idx[t] >= total) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < npts; ++t) {
        int64_t o = idx[t];
        const int64_t q = o % Q;
        o /= Q;
        const int64_t p = o % P;
        o /= P;
        const int64_t j = o % Kout;
        const int64_t n = o / Kout;
        double s = 0.0, m = 0.0;
        if (alpha != 0.0)
            conv_point(C, H, W, R, S, pad_h, pad_w, stride_h, stride_w,
                       x + n * C * H * W, w + j * C * R * S, p, q, &s, &m);
        double r = (alpha != 0.0) ? alpha * s : 0.0;
        double mm = (alpha != 0.0) ? fabs(alpha) * m : 0.0;
        if (beta != 0.0) {
            const double c0 = (double)y0[idx[t]];
            r += beta * c0;
            mm += fabs(beta) * fabs(c0);
        }
        ref[t] = r;
        if (mag) mag[t] = mm;
    }
    return 0;
}

/*
 * Backward passes of the same convolution (the paper's DNN pipeline is forward and backward; it names
 * separate data- and filter-gradient work in its discussion of streams).  Both are the adjoints of the
 * forward definition above with respect to x and to w, written out directly:
 *
 *   dx[n][c][h][w]  = alpha * sum_{j,r,s : p*sh + r - ph == h, q*sw + s - pw == w, 0 <= p < P, 0 <= q < Q}
 *                             dy[n][j][p][q] * w[j][c][r][s]                      + beta * dx0[n][c][h][w]
 *   dw[j][c][r][s]  = alpha * sum_{n,p,q : 0 <= p*sh + r - ph < H, 0 <= q*sw + s - pw < W}
 *                             dy[n][j][p][q] * x[n][c][p*sh + r - ph][q*sw + s - pw] + beta * dw0[j][c][r][s]
 *
 * FP64 sums in the loop order written (j, r, s for dx; n, p, q for dw), magnitude sums alongside.
 */
static inline void bwd_data_point(int64_t Kout, int64_t C, int64_t P, int64_t Q, int64_t R, int64_t S,
                                  int64_t ph, int64_t pw, int64_t sh, int64_t sw,
                                  const float *dy_img, const float *w, int64_t c, int64_t h, int64_t wcol,
                                  double *sum, double *msum)
{
    double s_acc = 0.0, t_acc = 0.0;
    for (int64_t j = 0; j < Kout; ++j)
        for (int64_t r = 0; r < R; ++r)
            for (int64_t s = 0; s < S; ++s) {
                const int64_t th = h + ph - r, tw = wcol + pw - s;
                if (th < 0 || tw < 0 || th % sh != 0 || tw % sw != 0) continue;
                const int64_t p = th / sh, q = tw / sw;
                if (p >= P || q >= Q) continue;
                const double g = (double)dy_img[(j * P + p) * Q + q];
                const double wv = (double)w[((j * C + c) * R + r) * S + s];
                s_acc += g * wv;
                t_acc += fabs(g) * fabs(wv);
            }
    *sum = s_acc;
    *msum = t_acc;
}

/* idx == NULL: every element of dx (npts ignored, ref / mag are N*C*H*W); else the flat offsets idx[0..npts). */
int oracle_conv2d_bwd_data(int64_t N, int64_t C, int64_t H, int64_t W,
                           int64_t Kout, int64_t R, int64_t S,
                           int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w,
                           double alpha, const float *dy, const float *w,
                           double beta, const float *dx0,
                           int64_t npts, const int64_t *idx, double *ref, double *mag)
{
    if (N < 0 || C < 0 || H < 0 || W < 0 || Kout < 0 || R < 1 || S < 1) return 1;
    if (pad_h < 0 || pad_w < 0 || stride_h < 1 || stride_w < 1 || !ref) return 1;
    const int64_t P = conv_out_dim(H, pad_h, R, stride_h);
    const int64_t Q = conv_out_dim(W, pad_w, S, stride_w);
    const int64_t total = N * C * H * W;
    const int64_t count = idx ? npts : total;
    if (idx)
        for (int64_t t = 0; t < npts; ++t)
            if (idx[t] < 0 || idx[t] >= total) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t) {
        int64_t o = idx ? idx[t] : t;
        const int64_t flat = o;
        const int64_t wc = o % W;
        o /= W;
        const int64_t h = o % H;
        o /= H;
        const int64_t c = o % C;
        const int64_t n = o / C;
        double s = 0.0, m = 0.0;
        if (alpha != 0.0)
            bwd_data_point(Kout, C, P, Q, R, S, pad_h, pad_w, stride_h, stride_w, dy + n * Kout * P * Q, w, c, h, wc,
                           &s, &m);
        double r = (alpha != 0.0) ? alpha * s : 0.0;
        double mm = (alpha != 0.0) ? fabs(alpha) * m : 0.0;
        if (beta != 0.0) {
            const double c0 = (double)dx0[flat];
            r += beta * c0;
            mm += fabs(beta) * fabs(c0);
        }
        ref[t] = r;
        if (mag) mag[t] = mm;
    }
    return 0;
}

/* idx == NULL: every element of dw (ref / mag are Kout*C*R*S); else the flat offsets idx[0..npts). */
int oracle_conv2d_bwd_filter(int64_t N, int64_t C, int64_t H, int64_t W,
                             int64_t Kout, int64_t R, int64_t S,
                             int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w,
                             double alpha, const float *x, const float *dy,
                             double beta, const float *dw0,
                             int64_t npts, const int64_t *idx, double *ref, double *mag)
{
    if (N < 0 || C < 0 || H < 0 || W < 0 || Kout < 0 || R < 1 || S < 1) return 1;
    if (pad_h < 0 || pad_w < 0 || stride_h < 1 || stride_w < 1 || !ref) return 1;
    const int64_t P = conv_out_dim(H, pad_h, R, stride_h);
    const int64_t Q = conv_out_dim(W, pad_w, S, stride_w);
    const int64_t total = Kout * C * R * S;
    const int64_t count = idx ? npts : total;
    if (idx)
        for (int64_t t = 0; t < npts; ++t)
            if (idx[t] < 0 || idx[t] >= total) return 1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < count; ++t) {
        int64_t o = idx ? idx[t] : t;
        const int64_t flat = o;
        const int64_t s = o % S;
        o /= S;
        const int64_t r = o % R;
        o /= R;
        const int64_t c = o % C;
        const int64_t j = o / C;
        double s_acc = 0.0, t_acc = 0.0;
        if (alpha != 0.0) {
            for (int64_t n = 0; n < N; ++n)
                for (int64_t p = 0; p < P; ++p) {
                    const int64_t ih = p * stride_h + r - pad_h;
                    if (ih < 0 || ih >= H) continue;
                    for (int64_t q = 0; q < Q; ++q) {
                        const int64_t iw = q * stride_w + s - pad_w;
                        if (iw < 0 || iw >= W) continue;
                        const double g = (double)dy[((n * Kout + j) * P + p) * Q + q];
                        const double xv = (double)x[((n * C + c) * H + ih) * W + iw];
                        s_acc += g * xv;
                        t_acc += fabs(g) * fabs(xv);
                    }
                }
        }
        double rr = (alpha != 0.0) ? alpha * s_acc : 0.0;
        double mm = (alpha != 0.0) ? fabs(alpha) * t_acc : 0.0;
        if (beta != 0.0) {
            const double c0 = (double)dw0[flat];
            rr += beta * c0;
            mm += fabs(beta) * fabs(c0);
        }
        ref[t] = rr;
        if (mag) mag[t] = mm;
    }
    return 0;
}
