/*
 * CPU oracle, expert FFN at full size.  TEST INFRASTRUCTURE ONLY: never linked
 * into or called by the HIP library.
 *
 * Computes, in fp64 and by the definition, one expert of a sparse MoE block
 * (arXiv 2312.17238, Sec. 2.1: the MoE replaces the feed-forward block) on
 * group-wise quantized weights (Sec. 4.2: a scale and a zero point per group of
 * consecutive weights):
 *
 *     W^[r][c] = (q[r][c] - zero[r][c/g]) * scale[r][c/g]
 *     u = W1^ h,  v = W3^ h,  a = u / (1 + exp(-u)) * v,  y = W2^ a
 *
 * Matrices are row-major [out][in]; w1, w3: [F][H]; w2: [H][F]; one byte per
 * code; scale and zero are IEEE binary16 bit patterns.  Each output row is one
 * sequential fp64 sum over its columns in increasing order; rows are
 * independent and shared among OpenMP threads, which does not change any sum.
 *
 * The numpy oracle computes the same definition through a dense matrix product;
 * the tests require the two to agree to 1e-12 relative on small shapes, which
 * pins this file to it.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double half_bits_to_double(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int exp = (b >> 10) & 0x1f;
    int man = b & 0x3ff;
    double v;
    if (exp == 0)
        v = ldexp((double)man, -24);              /* zero and subnormals */
    else if (exp == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexp((double)(man + 1024), exp - 25); /* (1 + man/1024) * 2^(exp-15) */
    return sign ? -v : v;
}

/* out[r] = sum_c (q[r][c] - zero[r][c/g]) * scale[r][c/g] * x[c] */
static void dequant_matvec(int rows, int cols, int g, const uint8_t *q, const uint16_t *scale,
                           const uint16_t *zero, const double *x, double *out)
{
    int groups = cols / g;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const uint8_t *qr = q + (size_t)r * cols;
        double acc = 0.0;
        for (int c = 0; c < cols; ++c) {
            size_t m = (size_t)r * groups + c / g;
            double w = ((double)qr[c] - half_bits_to_double(zero[m])) * half_bits_to_double(scale[m]);
            acc += w * x[c];
        }
        out[r] = acc;
    }
}

/* One expert.  h: [H] binary16 bits.  y_out: [H] fp64.  Returns 0, or -1 on bad sizes / no memory. */
int moe_oracle_expert_ffn(int H, int F, int g, const uint16_t *h_f16,
                          const uint8_t *q1, const uint16_t *s1, const uint16_t *z1,
                          const uint8_t *q3, const uint16_t *s3, const uint16_t *z3,
                          const uint8_t *q2, const uint16_t *s2, const uint16_t *z2,
                          double *y_out)
{
    if (H <= 0 || F <= 0 || g <= 0 || H % g || F % g)
        return -1;
    double *h = malloc(sizeof(double) * H);
    double *u = malloc(sizeof(double) * F);
    double *v = malloc(sizeof(double) * F);
    if (!h || !u || !v) {
        free(h); free(u); free(v);
        return -1;
    }
    for (int i = 0; i < H; ++i)
        h[i] = half_bits_to_double(h_f16[i]);
    dequant_matvec(F, H, g, q1, s1, z1, h, u);
    dequant_matvec(F, H, g, q3, s3, z3, h, v);
    for (int i = 0; i < F; ++i)
        u[i] = u[i] / (1.0 + exp(-u[i])) * v[i];
    dequant_matvec(H, F, g, q2, s2, z2, u, y_out);
    free(h); free(u); free(v);
    return 0;
}

/* The same loops for experts whose per-group scale and zero are given as fp64 values (two-level formats:
 * the caller evaluates the second level, a few numbers per row, by its own definition). */
static void dequant_matvec_f64(int rows, int cols, int g, const uint8_t *q, const double *scale,
                               const double *zero, const double *x, double *out)
{
    int groups = cols / g;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const uint8_t *qr = q + (size_t)r * cols;
        double acc = 0.0;
        for (int c = 0; c < cols; ++c) {
            size_t m = (size_t)r * groups + c / g;
            acc += ((double)qr[c] - zero[m]) * scale[m] * x[c];
        }
        out[r] = acc;
    }
}

int moe_oracle_expert_ffn_f64meta(int H, int F, int g, const uint16_t *h_f16,
                                  const uint8_t *q1, const double *s1, const double *z1,
                                  const uint8_t *q3, const double *s3, const double *z3,
                                  const uint8_t *q2, const double *s2, const double *z2,
                                  double *y_out)
{
    if (H <= 0 || F <= 0 || g <= 0 || H % g || F % g)
        return -1;
    double *h = malloc(sizeof(double) * H);
    double *u = malloc(sizeof(double) * F);
    double *v = malloc(sizeof(double) * F);
    if (!h || !u || !v) {
        free(h); free(u); free(v);
        return -1;
    }
    for (int i = 0; i < H; ++i)
        h[i] = half_bits_to_double(h_f16[i]);
    dequant_matvec_f64(F, H, g, q1, s1, z1, h, u);
    dequant_matvec_f64(F, H, g, q3, s3, z3, h, v);
    for (int i = 0; i < F; ++i)
        u[i] = u[i] / (1.0 + exp(-u[i])) * v[i];
    dequant_matvec_f64(H, F, g, q2, s2, z2, u, y_out);
    free(h); free(u); free(v);
    return 0;
}

int moe_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
