/*
 * silu_and_mul for AMD MI355X (gfx950) behind the same two-stage tuner as addrms:
 * the second of the serving kernels the paper evaluates (Section 4, "Kernels").
 *
 *     out[i, j] = silu(x[i, j]) * x[i, d + j],   silu(g) = g / (1 + exp(-g)),   0 <= j < d
 *
 * x is [M, 2d] row-major (gate half, then up half); out is [M, d]; both of one
 * storage format (ADDRMS_BF16, ADDRMS_FP16 or ADDRMS_FP32).  Arithmetic is fp32 with
 * the hardware exponential and reciprocal; the result is rounded once, to nearest
 * even, into the storage format.  Against the real value it is exact except within
 * a few fp32 ulps of a rounding boundary, where it may be one unit off.
 *
 * Configurations, budgets, reports, the feasible-region rules, the search and the
 * specialised table are the ones of addrms.h (addrms_cfg.reduce must be 0: there is
 * no reduction).  Pointer kinds, status codes and error text as in addrms.h.
 */
#ifndef SILUMUL_H
#define SILUMUL_H

#include "addrms.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One asynchronous launch.  x: device, [M, 2d]; out: device, [M, d], must not overlap x.
 * M == 0 is a no-op.  cfg: host; NULL = specialised table, else the default cfg.
 * stream: hipStream_t as void*.  Never synchronises, never allocates. */
int silumul_run(const void* x, void* out, int64_t M, int64_t d, int dtype, const addrms_cfg* cfg, void* stream);

int silumul_default_cfg(int64_t d, int dtype, addrms_cfg* out);
int silumul_cfg_feasible(const addrms_cfg* cfg, int64_t M, int64_t d, int dtype,
                         char* reason, size_t reason_len, addrms_resources* res);
int64_t silumul_enumerate_feasible(int64_t M, int64_t d, int dtype, addrms_cfg* out, int64_t cap, int64_t* n_grid);

/* Search on the current device (Algorithm 1 lines 18-23 for this kernel): same strategies,
 * gate (every candidate must reproduce the default cfg's output) and Top-K re-test as
 * addrms_tune; the winner goes to the specialised table under this operator. */
int silumul_tune(int64_t M, int64_t d, int dtype, const addrms_budget* budget,
                 addrms_cfg* out_cfg, addrms_tune_report* report);
int silumul_tune_with_backend(int64_t M, int64_t d, int dtype, const addrms_budget* budget,
                              const addrms_backend* backend, addrms_cfg* out_cfg, addrms_tune_report* report);

/* One general configuration over a set of shapes and the specialised table built on the way
 * (Algorithm 1 lines 22-23), as addrms_select_general does for add+RMSNorm: per-shape search,
 * pool of Top-K / defaults / universally feasible neighbours, every pool member timed on
 * every shape, arg-max of the geometric-mean speed-up over the per-shape defaults.
 * shapes: host, addrms_shape with M rows, N = d outputs per row.
 * Blocking; allocates and frees device memory. */
int silumul_select_general(const addrms_shape* shapes, int32_t n, int dtype, const addrms_budget* budget,
                           addrms_cfg* out_general, addrms_general_report* report);

/* The outer loop of Algorithm 1 with a fixed list of strategy families (base template, then the
 * streaming cache policy, the occupancy cap, the grid mapping), as addrms_tune_rounds: each round
 * validates the family it adds, searches every shape within the families enabled so far, selects
 * the general cfg and the specialised table, and scores the round. */
int silumul_tune_rounds(const addrms_shape* shapes, int32_t n, int dtype, const addrms_budget* budget,
                        addrms_cfg* out_general, addrms_rounds_report* report);

/* Mean time in microseconds over `reps` launches after `warmup`, on library-allocated
 * synthetic buffers rotated past the last-level cache (rotate != 0). */
int silumul_measure(const addrms_cfg* cfg, int64_t M, int64_t d, int dtype, int warmup, int reps, int rotate,
                    double* mean_us);

/* Exact (dtype, d, M) table entry of this operator, else the nearest tuned M; ADDRMS_ERR_NO_RESULT if none. */
int silumul_table_lookup(int64_t M, int64_t d, int dtype, addrms_cfg* out);

/* Bytes the operator must move: both halves of x read once, out written once. */
int64_t silumul_algorithmic_bytes(int64_t M, int64_t d, int dtype);

#ifdef __cplusplus
}
#endif
#endif /* SILUMUL_H */
