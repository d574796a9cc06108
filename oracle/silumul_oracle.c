/*
 * CPU oracle for silu_and_mul.  TEST INFRASTRUCTURE ONLY (same rules as the
 * add+RMSNorm oracle beside it: no code shared with the GPU path, never called
 * from it).
 *
 * The paper tunes three serving kernels (Section 4, "Kernels"); silu_and_mul is
 * the gated activation of a SwiGLU feed-forward block.  Its plain definition,
 * for an input row of 2d elements (gate half first, then the up half):
 *
 *     out[j] = silu(x[j]) * x[d + j],   silu(g) = g / (1 + exp(-g)),   j < d
 *
 * The oracle evaluates this in fp64 (inputs widen exactly) and rounds the real
 * result once, nearest-even, into the storage format of x.  A GPU version that
 * computes in fp32 with hardware exp/reciprocal differs from the real value by
 * a few fp32 ulps, i.e. it lands on the same 16-bit value except within that
 * distance of a rounding boundary, where it may be one unit off.
 *
 * Storage formats are raw uint16 bit patterns (bf16, fp16) or fp32; the format
 * routines are the ones in addrms_oracle.c (this file is compiled with it).
 *
 * Pins (tests/test_oracle_silumul.py): silu(g) - silu(-g) = g; zeros in either
 * half give zeros; large positive gates pass the up value through; a 50-digit
 * decimal evaluation rounded with exact rationals on random small inputs; the
 * half-row layout on position-coded inputs; torch CPU in fp64.
 */
#include <math.h>
#include <stdint.h>

float oracle_bf16_to_f32(uint16_t b);
uint16_t oracle_f32_to_bf16(float f);
float oracle_f16_to_f32(uint16_t h);
uint16_t oracle_f32_to_f16(float f);

enum { SM_BF16 = 0, SM_FP16 = 1, SM_FP32 = 3 };

static double sm_load(const void *p, int64_t i, int dtype)
{
    if (dtype == SM_FP32) return (double)((const float *)p)[i];
    uint16_t b = ((const uint16_t *)p)[i];
    return (double)(dtype == SM_BF16 ? oracle_bf16_to_f32(b) : oracle_f16_to_f32(b));
}

/* fp64 -> storage with a single rounding.  For the 16-bit formats the value is
 * first checked against the fp32 grid: rounding fp64 -> fp32 -> 16 bits could
 * double-round, so the 16-bit result is decided from the fp64 value directly by
 * picking the nearer of the two 16-bit neighbours of its fp32 truncation. */
static uint16_t round_to_16(double v, int dtype)
{
    /* candidates: the format values just below and just above (in magnitude) */
    float f = (float)v;                                   /* close enough to locate the cell */
    uint16_t a = dtype == SM_BF16 ? oracle_f32_to_bf16(f) : oracle_f32_to_f16(f);
    /* a is within one unit of the answer; test a-1, a, a+1 (same sign) against v exactly */
    uint16_t best = a;
    double best_err = INFINITY;
    for (int delta = -1; delta <= 1; ++delta) {
        int mag = (int)(a & 0x7fff) + delta;
        if (mag < 0) continue;
        uint16_t cand = (uint16_t)((a & 0x8000) | (uint16_t)mag);
        double cv = (double)(dtype == SM_BF16 ? oracle_bf16_to_f32(cand) : oracle_f16_to_f32(cand));
        if (isnan(cv)) continue;
        double err = fabs(cv - v);                        /* exact: both are fp64-representable, close */
        if (err < best_err || (err == best_err && (cand & 1) == 0)) { best_err = err; best = cand; }
    }
    return best;
}

/* x [M, 2d] storage dtype, out [M, d] same dtype; row-major, contiguous. */
int oracle_silumul(const void *x, int64_t M, int64_t d, int dtype, void *out, int nthreads)
{
    if (M < 0 || d <= 0 || !(dtype == SM_BF16 || dtype == SM_FP16 || dtype == SM_FP32)) return -1;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < d; ++j) {
            double g = sm_load(x, i * 2 * d + j, dtype);
            double u = sm_load(x, i * 2 * d + d + j, dtype);
            double s = g / (1.0 + exp(-g));
            double v = s * u;
            if (dtype == SM_FP32) ((float *)out)[i * d + j] = (float)v;
            else ((uint16_t *)out)[i * d + j] = round_to_16(v, dtype);
        }
    }
    return 0;
}

/* The unrounded fp64 value, for pins and for relative-error grading of fp32 output. */
int oracle_silumul_f64(const void *x, int64_t M, int64_t d, int dtype, double *out)
{
    if (M < 0 || d <= 0 || !(dtype == SM_BF16 || dtype == SM_FP16 || dtype == SM_FP32)) return -1;
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < d; ++j) {
            double g = sm_load(x, i * 2 * d + j, dtype);
            double u = sm_load(x, i * 2 * d + d + j, dtype);
            out[i * d + j] = g / (1.0 + exp(-g)) * u;
        }
    return 0;
}
