/*
 * CPU oracle for the Walsh-Hadamard output layer  y = alpha (.) (H x) + beta  and its backward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain fp64 statement of what the layer
 * computes.  Nothing in the product path (the HIP library and its Python binding) may include,
 * link or call it; only the tests, the smoke check and the benchmark's CPU-baseline leg do.
 * It shares no code, header, table or helper with the HIP kernels.
 *
 * What is computed (paper, Sec. 4.1, Eq. 1; Fig. 1 for the sign pattern; Fig. 2 for the
 * butterfly network):
 *
 *   H_raw[j][k] = (-1)^popcount(j AND k)            Sylvester ("natural") order: the 4x4 block
 *                                                   drawn in Fig. 1 has rows ++++ / +-+- / ++-- / +--+
 *   H           = H_raw / sqrt(d)                   the normalised matrix, H^T H = I (Sec. 4.1)
 *   z[n][j]     = sum_k H[j][k] x[n][k]             Y H per token; H is symmetric so Y H = (H y^T)^T
 *   y[n][j]     = alpha[j] * z[n][j] + beta[j]      Eq. 1
 *
 * Backward (the paper states only its O(d log d) complexity, Table 1; the formulas follow from
 * Eq. 1 by the chain rule, with H^T = H):
 *
 *   dbeta[j]  = sum_n dy[n][j]
 *   dalpha[j] = sum_n dy[n][j] * z[n][j]
 *   dx[n][k]  = sum_j H[j][k] * alpha[j] * dy[n][j]
 *
 * Widths d = 12 * 2^m (the paper trains d = 768 and d = 1536, Table 2, and does not say which
 * matrix it uses there; this is this library's reading):
 *
 *   H_raw = P12 (x) S_{2^m}                         Kronecker product: S is the Sylvester matrix above,
 *                                                   P12 acts across the 12 contiguous blocks of 2^m
 *                                                   features, H_raw[j][k] = P12[j / 2^m][k / 2^m] *
 *                                                   (-1)^popcount((j mod 2^m) AND (k mod 2^m))
 *   P12                                             the symmetric order-12 Hadamard matrix of Paley's
 *                                                   second construction over GF(5), with rows and
 *                                                   columns negated so that row 0 and column 0 are all +1
 *
 * P12 is symmetric with +-1 entries and P12 P12 = 12 I, so everything Sec. 4.1 uses still holds:
 * H = H_raw / sqrt(d) is symmetric, orthogonal, has entries +-1/sqrt(d) and a constant first row.
 *
 * Two independent ways to apply H are provided and cross-checked by the tests:
 *   method 0  "matrix": the definition, an explicit O(d^2) sum per token;
 *   method 1  "fast"  : the in-place butterfly network of Fig. 2 -- stages with stride
 *                       1, 2, 4, ..., d/2; each stage replaces the pair (a_i, a_{i+stride}) by
 *                       (a_i + a_{i+stride}, a_i - a_{i+stride}) -- followed by one 1/sqrt(d) scale.
 *                       For d = 12 * 2^m the strides stop at 2^(m-1) (each block of 2^m on its own)
 *                       and the 12 blocks are then combined entry by entry with P12.
 *
 * All arithmetic is IEEE double.  Inputs may be stored as double, float or bfloat16 bit patterns;
 * they are widened exactly, so input rounding is never part of an error budget.
 * Tokens are independent and are spread over OpenMP threads; nothing else is blocked, fused or
 * reordered.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { WHT_ORACLE_F64 = 0, WHT_ORACLE_F32 = 1, WHT_ORACLE_BF16 = 2 };
enum { WHT_ORACLE_MATRIX = 0, WHT_ORACLE_FAST = 1 };

/* ---- exact widening of a stored element to double ------------------------------------------ */

/* bfloat16 is the upper 16 bits of an IEEE binary32 value. */
double wht_oracle_bf16_bits_to_double(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double widen(const void *base, int64_t idx, int dtype)
{
    switch (dtype) {
    case WHT_ORACLE_F64:  return ((const double *)base)[idx];
    case WHT_ORACLE_F32:  return (double)((const float *)base)[idx];
    default:              return wht_oracle_bf16_bits_to_double(((const uint16_t *)base)[idx]);
    }
}

static int is_pow2(int64_t d) { return d >= 1 && (d & (d - 1)) == 0; }

/* Widths with a definition here: 2^n, and 12 * 2^m. */
static int is_twelve_width(int64_t d) { return d >= 12 && d % 12 == 0 && is_pow2(d / 12); }
static int is_width(int64_t d) { return is_pow2(d) || is_twelve_width(d); }

/* Length of the Sylvester factor: d itself, or 2^m for d = 12 * 2^m. */
static int64_t sylvester_len(int64_t d) { return is_pow2(d) ? d : d / 12; }

/* ---- the sign pattern (Fig. 1) -------------------------------------------------------------- */

/* +1 or -1: entry (j,k) of the unnormalised Sylvester Hadamard matrix. */
int wht_oracle_sign(uint32_t j, uint32_t k)
{
    uint32_t common = j & k;
    int ones = 0;
    while (common) { ones += (int)(common & 1u); common >>= 1; }
    return (ones % 2 == 0) ? 1 : -1;
}

/* ---- the order-12 factor ---------------------------------------------------------------------- */

/* Quadratic character of GF(5): 0 for 0, +1 for the squares {1, 4}, -1 for {2, 3}. */
static int chi5(int a)
{
    a %= 5;
    if (a < 0) a += 5;
    if (a == 0) return 0;
    return (a == 1 || a == 4) ? 1 : -1;
}

/* Symmetric conference matrix of order 6: zero diagonal, first row and column +1, Jacobsthal core. */
static int conference6(int i, int j)
{
    if (i == j) return 0;
    if (i == 0 || j == 0) return 1;
    return chi5(i - j);
}

/* Paley's second construction: every entry c of the conference matrix becomes c * [[1,1],[1,-1]],
 * every zero (the diagonal) becomes [[1,-1],[-1,-1]]. */
static int paley12_raw(int a, int b)
{
    static const int plus_block[2][2]  = { { 1, 1 }, { 1, -1 } };
    static const int diag_block[2][2]  = { { 1, -1 }, { -1, -1 } };
    int i = a / 2, u = a % 2, j = b / 2, v = b % 2;
    return (i == j) ? diag_block[u][v] : conference6(i, j) * plus_block[u][v];
}

/* Entry (a,b), 0 <= a,b < 12, of P12: row a and column b of the raw matrix are negated when the raw
 * matrix has -1 in row 0 at that index, which makes row 0 and column 0 all +1 and keeps symmetry. */
int wht_oracle_h12(int a, int b)
{
    return paley12_raw(0, a) * paley12_raw(a, b) * paley12_raw(0, b);
}

/* +1 or -1: entry (j,k) of the unnormalised matrix of width d (d = 2^n or 12 * 2^m; 0 otherwise). */
int wht_oracle_sign_d(int64_t d, uint32_t j, uint32_t k)
{
    if (!is_width(d) || j >= d || k >= d) return 0;
    if (is_pow2(d)) return wht_oracle_sign(j, k);
    uint32_t len = (uint32_t)sylvester_len(d);
    return wht_oracle_h12((int)(j / len), (int)(k / len)) * wht_oracle_sign(j % len, k % len);
}

/* ---- method 0: the definition --------------------------------------------------------------- */

/* out[j] = (1/sqrt d) sum_k sign(j,k) in[k] */
static void apply_H_matrix(const double *in, double *out, int64_t d)
{
    const double scale = 1.0 / sqrt((double)d);
    for (int64_t j = 0; j < d; ++j) {
        double acc = 0.0;
        for (int64_t k = 0; k < d; ++k)
            acc += (double)wht_oracle_sign_d(d, (uint32_t)j, (uint32_t)k) * in[k];
        out[j] = scale * acc;
    }
}

/* ---- method 1: the butterfly network (Fig. 2) ----------------------------------------------- */

/* One stage, in place: every pair (i, i+stride) whose lower index has the stride bit clear. */
void wht_oracle_butterfly_stage(double *a, int64_t d, int64_t stride)
{
    for (int64_t block = 0; block < d; block += 2 * stride) {
        for (int64_t i = block; i < block + stride; ++i) {
            double top = a[i];
            double bot = a[i + stride];
            a[i]          = top + bot;
            a[i + stride] = top - bot;
        }
    }
}

static void apply_H_fast(const double *in, double *out, int64_t d)
{
    const double scale = 1.0 / sqrt((double)d);
    const int64_t len = sylvester_len(d);
    for (int64_t k = 0; k < d; ++k) out[k] = in[k];
    for (int64_t stride = 1; stride < len; stride *= 2)
        wht_oracle_butterfly_stage(out, d, stride);
    if (len != d) {                              /* d = 12 * len: combine the 12 blocks with P12 */
        for (int64_t r = 0; r < len; ++r) {
            double blk[12];
            for (int b = 0; b < 12; ++b) blk[b] = out[b * len + r];
            for (int a = 0; a < 12; ++a) {
                double acc = 0.0;
                for (int b = 0; b < 12; ++b) acc += (double)wht_oracle_h12(a, b) * blk[b];
                out[a * len + r] = acc;
            }
        }
    }
    for (int64_t k = 0; k < d; ++k) out[k] *= scale;
}

static void apply_H(const double *in, double *out, int64_t d, int method)
{
    if (method == WHT_ORACLE_MATRIX) apply_H_matrix(in, out, d);
    else                             apply_H_fast(in, out, d);
}

/* ---- public entry points -------------------------------------------------------------------- */

/* z = H x for N tokens. x: [N,d] of `dtype`; z: [N,d] double.  Returns 0, or -1 on bad arguments. */
int wht_oracle_transform(const void *x, double *z, int64_t N, int64_t d, int dtype, int method)
{
    if (!x || !z || N < 0 || !is_width(d)) return -1;
    int failed = 0;
#pragma omp parallel
    {
        double *row = (double *)malloc((size_t)d * sizeof(double));
        if (!row) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (int64_t n = 0; n < N; ++n) {
                for (int64_t k = 0; k < d; ++k) row[k] = widen(x, n * d + k, dtype);
                apply_H(row, z + n * d, d, method);
            }
        }
        free(row);
    }
    return failed ? -2 : 0;
}

/* Eq. 1: y = alpha (.) (H x) + beta.  alpha, beta: [d] double; y: [N,d] double. */
int wht_oracle_forward(const void *x, const double *alpha, const double *beta, double *y,
                       int64_t N, int64_t d, int dtype, int method)
{
    if (!alpha || !beta) return -1;
    int rc = wht_oracle_transform(x, y, N, d, dtype, method);
    if (rc) return rc;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < d; ++j)
            y[n * d + j] = alpha[j] * y[n * d + j] + beta[j];
    return 0;
}

/*
 * Eq. 1 followed by the residual connection of the attention block (the paper's motivation for
 * the output projection notes that its result feeds the residual add after the block; Sec. 6 names
 * missing operator fusion as the reason the measured speed-ups lag the operation count):
 *     y = resid + alpha (.) (H x) + beta.     resid: [N,d] of `dtype`.
 */
int wht_oracle_forward_residual(const void *x, const double *alpha, const double *beta,
                                const void *resid, double *y,
                                int64_t N, int64_t d, int dtype, int method)
{
    if (!resid) return -1;
    int rc = wht_oracle_forward(x, alpha, beta, y, N, d, dtype, method);
    if (rc) return rc;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < d; ++j)
            y[n * d + j] = widen(resid, n * d + j, dtype) + y[n * d + j];
    return 0;
}

/*
 * The statistic a following RMS normalisation needs from the residual stream (Sec. 6 names the
 * interplay with RMSNorm as open; fusing the statistic into the layer's epilogue saves the
 * normalisation its reduction pass):   sumsq[n] = sum_j y[n][j]^2,   y as returned by
 * wht_oracle_forward_residual (unrounded).
 */
int wht_oracle_row_sumsq(const double *y, double *sumsq, int64_t N, int64_t d)
{
    if (!y || !sumsq || N < 0 || d < 1) return -1;
    for (int64_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int64_t j = 0; j < d; ++j) acc += y[n * d + j] * y[n * d + j];
        sumsq[n] = acc;
    }
    return 0;
}

/*
 * Backward.  dy, x: [N,d] of `dtype`; alpha: [d] double.
 * dx: [N,d] double or NULL (skip);  dalpha, dbeta: [d] double or NULL (skip both).
 * The sums over tokens are taken per thread over its contiguous share of tokens, in token order,
 * and the per-thread sums are then added in thread order.
 */
int wht_oracle_backward(const void *dy, const void *x, const double *alpha,
                        double *dx, double *dalpha, double *dbeta,
                        int64_t N, int64_t d, int dtype, int method)
{
    if (!dy || !x || !alpha || N < 0 || !is_width(d)) return -1;
    if ((dalpha == NULL) != (dbeta == NULL)) return -1;
    const int want_param_grads = dalpha != NULL;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    double *partial = NULL;                 /* [nthreads][2][d] */
    if (want_param_grads) {
        partial = (double *)calloc((size_t)nthreads * 2 * (size_t)d, sizeof(double));
        if (!partial) return -2;
    }
    int failed = 0;
#pragma omp parallel num_threads(nthreads)
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        double *xr = (double *)malloc((size_t)d * sizeof(double));
        double *zr = (double *)malloc((size_t)d * sizeof(double));
        double *gr = (double *)malloc((size_t)d * sizeof(double));
        double *hr = (double *)malloc((size_t)d * sizeof(double));
        if (!xr || !zr || !gr || !hr) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
            double *my_dalpha = want_param_grads ? partial + (size_t)tid * 2 * d : NULL;
            double *my_dbeta  = want_param_grads ? my_dalpha + d : NULL;
#pragma omp for schedule(static)
            for (int64_t n = 0; n < N; ++n) {
                if (want_param_grads) {
                    for (int64_t k = 0; k < d; ++k) xr[k] = widen(x, n * d + k, dtype);
                    apply_H(xr, zr, d, method);                       /* z = H x */
                    for (int64_t j = 0; j < d; ++j) {
                        double g = widen(dy, n * d + j, dtype);
                        my_dbeta[j]  += g;
                        my_dalpha[j] += g * zr[j];
                    }
                }
                if (dx) {
                    for (int64_t j = 0; j < d; ++j)
                        gr[j] = alpha[j] * widen(dy, n * d + j, dtype);
                    apply_H(gr, hr, d, method);                       /* dx = H (alpha (.) dy) */
                    for (int64_t k = 0; k < d; ++k) dx[n * d + k] = hr[k];
                }
            }
        }
        free(xr); free(zr); free(gr); free(hr);
    }
    if (want_param_grads && !failed) {
        for (int64_t j = 0; j < d; ++j) { dalpha[j] = 0.0; dbeta[j] = 0.0; }
        for (int t = 0; t < nthreads; ++t)
            for (int64_t j = 0; j < d; ++j) {
                dalpha[j] += partial[(size_t)t * 2 * d + j];
                dbeta[j]  += partial[(size_t)t * 2 * d + d + j];
            }
    }
    free(partial);
    return failed ? -2 : 0;
}

int wht_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void wht_oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
