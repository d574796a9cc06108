/*
 * CPU oracle for merge_attn_states.  TEST INFRASTRUCTURE ONLY (same rules as the
 * other oracles here: no code shared with the GPU path, never called from it).
 *
 * Third of the serving kernels the paper evaluates (Section 4, "Kernels"; its
 * Kernel-1 shape list is (n, h, d) = tokens x heads x head size).  Attention
 * computed over two disjoint parts of the keys gives two partial outputs, each
 * normalised by its own softmax denominator, and the logarithm of that
 * denominator (log-sum-exp, natural log).  Merging them is the textbook
 * log-sum-exp combination, per token and head:
 *
 *     m      = max(s_a, s_b)
 *     e_a    = exp(s_a - m),  e_b = exp(s_b - m)
 *     v_out  = (e_a * v_a + e_b * v_b) / (e_a + e_b)        for each of the d lanes
 *     s_out  = m + log(e_a + e_b)
 *
 * Evaluated in fp64; v_out is rounded once, nearest-even, into the storage format
 * of v (bf16 or fp16, raw uint16 bit patterns), s_out once into fp32.  Inputs are
 * assumed finite.
 *
 * Layout: v_a, v_b, v_out are [rows, d] row-major with rows = n * h; s_a, s_b,
 * s_out are fp32 [rows].
 *
 * Pins (tests/test_oracle_mergestates.py): equal scores give the average; a score
 * gap of 80 returns the dominant part unchanged; swapping the two parts changes
 * nothing; a common shift of the scores shifts s_out and leaves v_out; s_out
 * against numpy's logaddexp; outputs lie between the two inputs; 50-digit decimal
 * evaluation with exact-rational rounding.
 */
#include <math.h>
#include <stdint.h>

float oracle_bf16_to_f32(uint16_t b);
uint16_t oracle_f32_to_bf16(float f);
float oracle_f16_to_f32(uint16_t h);
uint16_t oracle_f32_to_f16(float f);

enum { MS_BF16 = 0, MS_FP16 = 1 };

static double ms_load(const uint16_t *p, int64_t i, int dtype)
{
    return (double)(dtype == MS_BF16 ? oracle_bf16_to_f32(p[i]) : oracle_f16_to_f32(p[i]));
}

/* Nearest format value to the fp64 value v, ties to even, without a detour through fp32:
 * the fp32 conversion only locates the cell, the three candidates around it are compared
 * against v exactly. */
static uint16_t ms_round16(double v, int dtype)
{
    float f = (float)v;
    uint16_t a = dtype == MS_BF16 ? oracle_f32_to_bf16(f) : oracle_f32_to_f16(f);
    uint16_t best = a;
    double best_err = INFINITY;
    for (int delta = -1; delta <= 1; ++delta) {
        int mag = (int)(a & 0x7fff) + delta;
        if (mag < 0) continue;
        uint16_t cand = (uint16_t)((a & 0x8000) | (uint16_t)mag);
        double cv = (double)(dtype == MS_BF16 ? oracle_bf16_to_f32(cand) : oracle_f16_to_f32(cand));
        if (isnan(cv)) continue;
        double err = fabs(cv - v);
        if (err < best_err || (err == best_err && (cand & 1) == 0)) { best_err = err; best = cand; }
    }
    return best;
}

int oracle_mergestates(const uint16_t *va, const float *sa, const uint16_t *vb, const float *sb,
                       int64_t rows, int64_t d, int dtype, uint16_t *vout, float *sout, double *vout64)
{
    if (rows < 0 || d <= 0 || (dtype != MS_BF16 && dtype != MS_FP16)) return -1;
    for (int64_t i = 0; i < rows; ++i) {
        double a = (double)sa[i], b = (double)sb[i];
        double m = a > b ? a : b;
        double ea = exp(a - m), eb = exp(b - m);
        double denom = ea + eb;
        if (sout) sout[i] = (float)(m + log(denom));
        for (int64_t j = 0; j < d; ++j) {
            double v = (ea * ms_load(va, i * d + j, dtype) + eb * ms_load(vb, i * d + j, dtype)) / denom;
            if (vout) vout[i * d + j] = ms_round16(v, dtype);
            if (vout64) vout64[i * d + j] = v;
        }
    }
    return 0;
}
