/*
 * CPU oracle for fused residual-add + RMSNorm.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  It shares no code with the GPU path and must never be called from
 * it: only the test-suite, the smoke check and the CPU-baseline leg of the
 * benchmark may build or call it.
 *
 * What it defines.  The paper (Section 3.1, "Correctness") only fixes the frame:
 * a tuned kernel S~ must agree with the original S on a finite test set under a
 * metric d and tolerance eps; the tuner may change execution strategy, never
 * the operator.  The operator itself is the serving kernel fused_add_rmsnorm
 * named in Section 4 ("Kernels").  Its arithmetic is written out here, per row:
 *
 *   1. h[j]    = f32(x[j]) + f32(r[j])            one IEEE fp32 add, RNE
 *   2. res[j]  = RNE(h[j] -> residual dtype)       identity for fp32 residual
 *   3. ss      = sum_j h[j]^2                      see "variants" below
 *      rstd    = fp32( 1 / sqrt(ss / N + eps) )
 *   4. y[j]    = RNE( (h[j] * rstd) * f32(w[j]) -> x dtype )
 *                two fp32 multiplies in that order, on the UNROUNDED h
 *
 * Variants of step 3 (argument `variant`):
 *   0  canonical : every h^2 is exact in fp64 (24x24 bits); summed left to right
 *                  in fp64; mean, sqrt and reciprocal in fp64; one rounding to
 *                  fp32.  This is the value every fp32 summation order
 *                  approximates, so it does not depend on a GPU launch shape.
 *   1  seq32     : literal fp32: ss summed left to right in fp32 (separate
 *                  multiply and add), mean = ss / (float)N, rstd = 1/sqrtf(mean+eps)
 *   2  pair32    : as seq32 but the sum is a balanced pairwise tree in fp32
 *
 * Storage formats.  bf16 and fp16 are handled as raw uint16 bit patterns; the
 * encode/decode routines below are written from the IEEE-754 / bfloat16
 * definitions (nearest, ties to even; subnormals kept; overflow to infinity).
 *
 * Pins (tests/test_oracle_*.py): exact rational brute force on tiny inputs,
 * closed forms (unit weight RMS, constant row, one-hot row, zero row), exact
 * invariants (row permutation, negation, power-of-two scaling, column
 * permutation), agreement of the three variants within 1 ulp, and independent
 * library conversions (numpy / torch CPU) for the four format routines.
 *
 * Build:  gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp -fPIC -shared
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_BF16 = 0, ORACLE_FP16 = 1, ORACLE_FP16_RES32 = 2, ORACLE_FP32 = 3 };
enum { ORACLE_CANONICAL = 0, ORACLE_SEQ32 = 1, ORACLE_PAIR32 = 2 };

/* ---- bit casts -------------------------------------------------------- */
static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* ---- bfloat16: the upper 16 bits of an fp32 ---------------------------- */
float oracle_bf16_to_f32(uint16_t b) { return bits_f32((uint32_t)b << 16); }

uint16_t oracle_f32_to_bf16(float f)
{
    uint32_t u = f32_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)          /* NaN: keep sign, force quiet */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep = u >> 16;                       /* truncated candidate        */
    uint32_t rem = u & 0xffffu;                    /* discarded 16 bits          */
    /* nearest; on an exact tie pick the candidate whose last bit is 0.  The
     * increment carries into the exponent field, which is the right next value
     * (and becomes infinity past the largest finite bf16). */
    if (rem > 0x8000u || (rem == 0x8000u && (keep & 1u)))
        keep += 1u;
    return (uint16_t)keep;
}

/* ---- IEEE binary16 ---------------------------------------------------- */
float oracle_f16_to_f32(uint16_t hbits)
{
    int sign = (hbits >> 15) & 1;
    int e = (hbits >> 10) & 0x1f;
    int m = hbits & 0x3ff;
    float v;
    if (e == 0)
        v = ldexpf((float)m, -24);                 /* subnormal or zero          */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexpf((float)(m + 1024), e - 25);     /* (1 + m/1024) * 2^(e-15)    */
    return sign ? -v : v;
}

uint16_t oracle_f32_to_f16(float f)
{
    uint16_t sign = (uint16_t)((f32_bits(f) >> 16) & 0x8000u);
    if (isnan(f))
        return (uint16_t)(sign | 0x7e00u);
    double a = fabs((double)f);
    if (a == 0.0)
        return sign;
    if (isinf(f))
        return (uint16_t)(sign | 0x7c00u);
    int ex;
    (void)frexp(a, &ex);                           /* a = m * 2^ex, m in [0.5,1) */
    int e = ex - 1;                                /* a in [2^e, 2^(e+1))        */
    if (e < -14) {
        /* below the smallest normal: spacing is 2^-24 everywhere.  rint() is
         * round-half-even in the default rounding mode; q == 1024 lands on
         * the smallest normal, whose bit pattern is exactly 0x0400. */
        double q = rint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)q);
    }
    double q = rint(ldexp(a, 10 - e));             /* in [1024, 2048]            */
    if (q == 2048.0) { q = 1024.0; e += 1; }
    if (e > 15)
        return (uint16_t)(sign | 0x7c00u);         /* rounds past 65504: inf     */
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)((int)q - 1024));
}

/* ---- element access by dtype ------------------------------------------ */
static int x_is_f32(int dtype) { return dtype == ORACLE_FP32; }
static int r_is_f32(int dtype) { return dtype == ORACLE_FP32 || dtype == ORACLE_FP16_RES32; }
static int half_is_bf16(int dtype) { return dtype == ORACLE_BF16; }

static float load16(const void *p, int64_t i, int dtype)
{
    uint16_t b = ((const uint16_t *)p)[i];
    return half_is_bf16(dtype) ? oracle_bf16_to_f32(b) : oracle_f16_to_f32(b);
}
static void store16(void *p, int64_t i, int dtype, float v)
{
    ((uint16_t *)p)[i] = half_is_bf16(dtype) ? oracle_f32_to_bf16(v) : oracle_f32_to_f16(v);
}
static float load_x(const void *p, int64_t i, int dtype)
{
    return x_is_f32(dtype) ? ((const float *)p)[i] : load16(p, i, dtype);
}
static float load_r(const void *p, int64_t i, int dtype)
{
    return r_is_f32(dtype) ? ((const float *)p)[i] : load16(p, i, dtype);
}
static void store_y(void *p, int64_t i, int dtype, float v)
{
    if (x_is_f32(dtype)) ((float *)p)[i] = v; else store16(p, i, dtype, v);
}
static void store_r(void *p, int64_t i, int dtype, float v)
{
    if (r_is_f32(dtype)) ((float *)p)[i] = v; else store16(p, i, dtype, v);
}

/* ---- step 3 variants --------------------------------------------------- */
float oracle_rstd_canonical(double ss, int64_t N, float eps)
{
    return (float)(1.0 / sqrt(ss / (double)N + (double)eps));
}

static float pairwise_sum_sq(const float *h, int64_t n)
{
    if (n == 1) return h[0] * h[0];
    int64_t half = n / 2;
    float a = pairwise_sum_sq(h, half);
    float b = pairwise_sum_sq(h + half, n - half);
    return a + b;
}

static float row_rstd(const float *h, int64_t N, float eps, int variant)
{
    if (variant == ORACLE_CANONICAL) {
        double ss = 0.0;
        for (int64_t j = 0; j < N; ++j)
            ss += (double)h[j] * (double)h[j];
        return oracle_rstd_canonical(ss, N, eps);
    }
    float ss;
    if (variant == ORACLE_SEQ32) {
        ss = 0.0f;
        for (int64_t j = 0; j < N; ++j) {
            float sq = h[j] * h[j];
            ss = ss + sq;
        }
    } else {
        ss = pairwise_sum_sq(h, N);
    }
    float mean = ss / (float)N;
    return 1.0f / sqrtf(mean + eps);
}

/*
 * The operator, out of place on host arrays.
 *   x [M,N] x-dtype, r [M,N] residual dtype, w [N] x-dtype (row-major, stride N)
 *   y_out [M,N] x-dtype, res_out [M,N] residual dtype
 *   rstd_out: optional [M] fp32 (may be NULL)
 *   nthreads: rows are split over this many OpenMP threads (rows only).
 * Returns 0, or -1 on a bad argument.
 */
int oracle_addrms(const void *x, const void *r, const void *w, float eps,
                  int64_t M, int64_t N, int dtype, int variant,
                  void *y_out, void *res_out, float *rstd_out, int nthreads)
{
    if (M < 0 || N <= 0 || dtype < 0 || dtype > 3 || variant < 0 || variant > 2)
        return -1;
    if (nthreads < 1) nthreads = 1;
    int failed = 0;
#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        float *h = (float *)malloc((size_t)N * sizeof(float));
        if (!h) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        for (int64_t j = 0; j < N; ++j) {
            float xf = load_x(x, i * N + j, dtype);
            float rf = load_r(r, i * N + j, dtype);
            h[j] = xf + rf;
            store_r(res_out, i * N + j, dtype, h[j]);
        }
        float rstd = row_rstd(h, N, eps, variant);
        if (rstd_out) rstd_out[i] = rstd;
        for (int64_t j = 0; j < N; ++j) {
            float wf = load_x(w, j, dtype);
            float t = h[j] * rstd;
            float v = t * wf;
            store_y(y_out, i * N + j, dtype, v);
        }
        free(h);
    }
    return failed ? -1 : 0;
}

/*
 * Unrounded fp64 path for invariant checks: h = x + r exactly in fp64,
 * ms = mean(h^2), y64 = h * w / sqrt(ms + eps).  No intermediate is rounded to
 * fp32 or to a storage format.
 */
int oracle_addrms_y64(const void *x, const void *r, const void *w, double eps,
                      int64_t M, int64_t N, int dtype, double *y64)
{
    if (M < 0 || N <= 0 || dtype < 0 || dtype > 3)
        return -1;
    for (int64_t i = 0; i < M; ++i) {
        double ss = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            double hj = (double)load_x(x, i * N + j, dtype) + (double)load_r(r, i * N + j, dtype);
            ss += hj * hj;
        }
        double denom = sqrt(ss / (double)N + eps);
        for (int64_t j = 0; j < N; ++j) {
            double hj = (double)load_x(x, i * N + j, dtype) + (double)load_r(r, i * N + j, dtype);
            y64[i * N + j] = hj * (double)load_x(w, j, dtype) / denom;
        }
    }
    return 0;
}

/* Array forms of the four format routines, so the pins can sweep many values. */
void oracle_f32_to_bf16_array(const float *in, uint16_t *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = oracle_f32_to_bf16(in[i]); }
void oracle_f32_to_f16_array(const float *in, uint16_t *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = oracle_f32_to_f16(in[i]); }
void oracle_bf16_to_f32_array(const uint16_t *in, float *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = oracle_bf16_to_f32(in[i]); }
void oracle_f16_to_f32_array(const uint16_t *in, float *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = oracle_f16_to_f32(in[i]); }
