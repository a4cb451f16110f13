/* Drives every entry point of oracle/wht_oracle.c on exact-size heap buffers, so that a run under
 * AddressSanitizer / UndefinedBehaviorSanitizer exposes any out-of-bounds access, misaligned use or
 * undefined arithmetic in the oracle; also cross-checks its two methods.  Host only. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

double wht_oracle_bf16_bits_to_double(uint16_t bits);
int wht_oracle_sign(uint32_t j, uint32_t k);
int wht_oracle_h12(int a, int b);
int wht_oracle_sign_d(int64_t d, uint32_t j, uint32_t k);
void wht_oracle_butterfly_stage(double *a, int64_t d, int64_t stride);
int wht_oracle_transform(const void *x, double *z, int64_t N, int64_t d, int dtype, int method);
int wht_oracle_forward(const void *x, const double *alpha, const double *beta, double *y,
                       int64_t N, int64_t d, int dtype, int method);
int wht_oracle_forward_residual(const void *x, const double *alpha, const double *beta, const void *resid,
                                double *y, int64_t N, int64_t d, int dtype, int method);
int wht_oracle_row_sumsq(const double *y, double *sumsq, int64_t N, int64_t d);
int wht_oracle_backward(const void *dy, const void *x, const double *alpha, double *dx, double *dalpha,
                        double *dbeta, int64_t N, int64_t d, int dtype, int method);
int wht_oracle_num_threads(void);
void wht_oracle_set_num_threads(int n);

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static uint32_t rng_state = 12345u;
static double uniform(void) { rng_state = rng_state * 1664525u + 1013904223u; return (rng_state >> 8) / 16777216.0 - 0.5; }

static void one_shape(int64_t N, int64_t d, int dtype)
{
    const size_t n = (size_t)(N * d);
    const size_t esz = dtype == 0 ? 8 : (dtype == 1 ? 4 : 2);      /* the oracle's codes: 0 f64, 1 f32, 2 bf16 */
    void *x = malloc(n * esz + (n == 0)), *dy = malloc(n * esz + (n == 0));
    double *alpha = malloc((size_t)d * 8), *beta = malloc((size_t)d * 8);
    double *y0 = malloc(n * 8 + 8), *y1 = malloc(n * 8 + 8), *dx0 = malloc(n * 8 + 8), *dx1 = malloc(n * 8 + 8);
    double *da0 = malloc((size_t)d * 8), *db0 = malloc((size_t)d * 8), *da1 = malloc((size_t)d * 8), *db1 = malloc((size_t)d * 8);
    double *ss = malloc((size_t)N * 8 + 8);
    for (size_t i = 0; i < n; ++i) {
        if (dtype == 0) { ((double *)x)[i] = uniform(); ((double *)dy)[i] = uniform(); }
        else if (dtype == 1) { ((float *)x)[i] = (float)uniform(); ((float *)dy)[i] = (float)uniform(); }
        else {
            union { float f; uint32_t u; } a = { (float)uniform() }, b = { (float)uniform() };
            ((uint16_t *)x)[i] = (uint16_t)(a.u >> 16); ((uint16_t *)dy)[i] = (uint16_t)(b.u >> 16);
        }
    }
    for (int64_t j = 0; j < d; ++j) { alpha[j] = 1.0 + uniform(); beta[j] = 0.1 * uniform(); }
    EXPECT(wht_oracle_forward(x, alpha, beta, y0, N, d, dtype, 0) == 0);
    EXPECT(wht_oracle_forward(x, alpha, beta, y1, N, d, dtype, 1) == 0);
    EXPECT(wht_oracle_backward(dy, x, alpha, dx0, da0, db0, N, d, dtype, 0) == 0);
    EXPECT(wht_oracle_backward(dy, x, alpha, dx1, da1, db1, N, d, dtype, 1) == 0);
    double worst = 0.0;
    for (size_t i = 0; i < n; ++i) { worst = fmax(worst, fabs(y0[i] - y1[i])); worst = fmax(worst, fabs(dx0[i] - dx1[i])); }
    for (int64_t j = 0; j < d; ++j) { worst = fmax(worst, fabs(da0[j] - da1[j])); worst = fmax(worst, fabs(db0[j] - db1[j])); }
    EXPECT(worst < 1e-9);
    EXPECT(wht_oracle_backward(dy, x, alpha, NULL, da1, db1, N, d, dtype, 1) == 0);      /* outputs left out */
    EXPECT(wht_oracle_backward(dy, x, alpha, dx1, NULL, NULL, N, d, dtype, 1) == 0);
    EXPECT(wht_oracle_forward_residual(x, alpha, beta, dy, y1, N, d, dtype, 1) == 0);
    EXPECT(wht_oracle_row_sumsq(y1, ss, N, d) == 0);
    EXPECT(wht_oracle_transform(x, y1, N, d, dtype, 1) == 0);
    free(x); free(dy); free(alpha); free(beta); free(y0); free(y1); free(dx0); free(dx1);
    free(da0); free(db0); free(da1); free(db1); free(ss);
}

int main(void)
{
    const int64_t widths[] = {1, 2, 4, 32, 256, 1024, 12, 24, 768, 1536};
    for (size_t w = 0; w < sizeof widths / sizeof widths[0]; ++w)
        for (int dtype = 0; dtype < 3; ++dtype) {
            one_shape(0, widths[w], dtype);
            one_shape(1, widths[w], dtype);
            one_shape(5, widths[w], dtype);
        }
    wht_oracle_set_num_threads(3);
    one_shape(7, 512, 2);
    EXPECT(wht_oracle_num_threads() == 3);
    /* bad arguments come back as errors, not as accesses */
    double z[4];
    float xf[4] = {1, 2, 3, 4};
    EXPECT(wht_oracle_transform(NULL, z, 1, 4, 1, 1) != 0);
    EXPECT(wht_oracle_transform(xf, z, 1, 3, 1, 1) != 0);
    EXPECT(wht_oracle_transform(xf, z, -1, 4, 1, 1) != 0);
    EXPECT(wht_oracle_backward(xf, xf, NULL, z, NULL, NULL, 1, 4, 1, 1) != 0);
    /* sign tables and a butterfly stage at their index limits */
    EXPECT(wht_oracle_sign(0xffffffffu, 0xffffffffu) == 1 && wht_oracle_sign(1, 1) == -1);
    EXPECT(wht_oracle_h12(0, 11) == 1 && (wht_oracle_h12(11, 11) == 1 || wht_oracle_h12(11, 11) == -1));
    EXPECT(wht_oracle_sign_d(768, 767, 767) * wht_oracle_sign_d(768, 767, 767) == 1);
    double a8[8] = {1, 2, 3, 4, 5, 6, 7, 8};
    wht_oracle_butterfly_stage(a8, 8, 4);
    EXPECT(a8[0] == 6 && a8[4] == -4);
    EXPECT(wht_oracle_bf16_bits_to_double(0x3f80) == 1.0 && wht_oracle_bf16_bits_to_double(0xc000) == -2.0);
    printf(failures ? "oracle_sanitize_driver: %d failure(s)\n" : "oracle_sanitize_driver: ok\n", failures);
    return failures ? 1 : 0;
}
