/*
 * merge_attn_states for AMD MI355X (gfx950) behind the same two-stage tuner as addrms:
 * the third of the serving kernels the paper evaluates (Section 4, "Kernels").
 *
 * Two partial attention results over disjoint key ranges -- outputs v_a, v_b [rows, d]
 * (rows = tokens x heads) and their log-sum-exp scores s_a, s_b [rows] (natural log) --
 * are merged per row:
 *     m = max(s_a, s_b);  e_a = exp(s_a - m);  e_b = exp(s_b - m)
 *     v_out = (e_a v_a + e_b v_b) / (e_a + e_b);   s_out = m + log(e_a + e_b)
 * v tensors are ADDRMS_BF16 or ADDRMS_FP16, row-major, contiguous; scores are fp32.
 * Arithmetic is fp32 with the hardware exponential, logarithm and reciprocal; v_out is
 * rounded once into the storage format.  Scores must be finite.
 *
 * Configurations, budgets, reports, feasibility rules, search and table are those of
 * addrms.h (addrms_cfg.reduce must be 0).  d plays the role of N.
 */
#ifndef MERGESTATES_H
#define MERGESTATES_H

#include "addrms.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One asynchronous launch.  All pointers device; outputs must not overlap inputs.
 * rows == 0 is a no-op.  cfg: host; NULL = specialised table, else default. */
int mergestates_run(const void* v_a, const float* s_a, const void* v_b, const float* s_b,
                    void* v_out, float* s_out, int64_t rows, int64_t d, int dtype,
                    const addrms_cfg* cfg, void* stream);

int mergestates_default_cfg(int64_t d, int dtype, addrms_cfg* out);
int mergestates_cfg_feasible(const addrms_cfg* cfg, int64_t rows, int64_t d, int dtype,
                             char* reason, size_t reason_len, addrms_resources* res);
int64_t mergestates_enumerate_feasible(int64_t rows, int64_t d, int dtype, addrms_cfg* out, int64_t cap,
                                       int64_t* n_grid);
int mergestates_tune(int64_t rows, int64_t d, int dtype, const addrms_budget* budget,
                     addrms_cfg* out_cfg, addrms_tune_report* report);
int mergestates_tune_with_backend(int64_t rows, int64_t d, int dtype, const addrms_budget* budget,
                                  const addrms_backend* backend, addrms_cfg* out_cfg, addrms_tune_report* report);

/* One general configuration over a set of shapes and the specialised table built on the way
 * (Algorithm 1 lines 22-23), as addrms_select_general does for add+RMSNorm: per-shape search,
 * pool of Top-K / defaults / universally feasible neighbours, every pool member timed on
 * every shape, arg-max of the geometric-mean speed-up over the per-shape defaults.
 * shapes: host, addrms_shape with M = rows (tokens x heads), N = d (head size).
 * Blocking; allocates and frees device memory. */
int mergestates_select_general(const addrms_shape* shapes, int32_t n, int dtype, const addrms_budget* budget,
                               addrms_cfg* out_general, addrms_general_report* report);

/* The outer loop of Algorithm 1 with a fixed list of strategy families (base template, then the
 * streaming cache policy, the occupancy cap, the grid mapping), as addrms_tune_rounds: each round
 * validates the family it adds, searches every shape within the families enabled so far, selects
 * the general cfg and the specialised table, and scores the round. */
int mergestates_tune_rounds(const addrms_shape* shapes, int32_t n, int dtype, const addrms_budget* budget,
                            addrms_cfg* out_general, addrms_rounds_report* report);

int mergestates_measure(const addrms_cfg* cfg, int64_t rows, int64_t d, int dtype, int warmup, int reps,
                        int rotate, double* mean_us);
int mergestates_table_lookup(int64_t rows, int64_t d, int dtype, addrms_cfg* out);
/* rows * (3 * d * element size + 12): v_a, v_b read, v_out written, three fp32 scores per row. */
int64_t mergestates_algorithmic_bytes(int64_t rows, int64_t d, int dtype);

#ifdef __cplusplus
}
#endif
#endif /* MERGESTATES_H */
