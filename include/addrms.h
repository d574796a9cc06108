/*
 * addrms -- fused residual-add + RMSNorm for AMD MI355X (gfx950), with the
 * paper's two-stage tuner: an explicitly parameterised kernel template, a
 * feasible-region deriver built on the hardware's resource limits, and a
 * measured search over that region (Algorithm 1, Level 2; Section 3.3).
 *
 * C ABI.  Every function returns 0 (ADDRMS_OK) or a negative addrms_status;
 * a message for the last failure on the calling thread is available from
 * addrms_last_error().  No exception crosses this boundary.
 *
 * Pointer kinds are stated per argument: "device" = HIP device memory owned by
 * the caller; "host" = ordinary host memory owned by the caller.  The library
 * owns its compiled kernels, the configuration table and the error string.
 *
 * The operator (Section 4, "Kernels": fused_add_rmsnorm), per row of N elements:
 *     h        = f32(x) + f32(residual)                    (one fp32 add)
 *     residual <- round_nearest_even(h -> residual dtype)  (in place)
 *     rstd     = fp32( 1 / sqrt( sum(h^2)/N + eps ) )      (sum of squares in fp64)
 *     x        <- round_nearest_even((h*rstd)*f32(weight) -> x dtype)  (in place)
 * Results do not depend on the configuration used to run it.
 */
#ifndef ADDRMS_H
#define ADDRMS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADDRMS_VERSION_STRING "0.2.0"

/* ---- status codes ------------------------------------------------------- */
typedef enum addrms_status {
    ADDRMS_OK = 0,
    ADDRMS_ERR_INVALID_ARG = -1,       /* null pointer, N <= 0, M < 0, bad enum, bad struct field */
    ADDRMS_ERR_UNSUPPORTED_DTYPE = -2,
    ADDRMS_ERR_INFEASIBLE_CFG = -3,    /* cfg outside the feasible region for (M, N, dtype) */
    ADDRMS_ERR_MISALIGNED = -4,        /* a tensor base is not aligned to cfg's vector width */
    ADDRMS_ERR_HIP = -5,               /* a HIP runtime call failed; text has the HIP error */
    ADDRMS_ERR_IO = -6,                /* table/log file could not be read or written, or is malformed */
    ADDRMS_ERR_NO_RESULT = -7,         /* budget ran out before any candidate was measured */
    ADDRMS_ERR_UNSUPPORTED_SHAPE = -8  /* no configuration of the template covers this N */
} addrms_status;

/* ---- storage formats ----------------------------------------------------- */
typedef enum addrms_dtype {
    ADDRMS_BF16 = 0,        /* x, residual, weight: bfloat16                       */
    ADDRMS_FP16 = 1,        /* x, residual, weight: IEEE binary16                  */
    ADDRMS_FP16_RES32 = 2,  /* x, weight: binary16; residual stream: fp32          */
    ADDRMS_FP32 = 3         /* x, residual, weight: fp32 (the paper's fp32 shapes) */
} addrms_dtype;

/* ---- the searchable parameter vector theta (Algorithm 1, Input) ------------ */
enum { ADDRMS_REDUCE_WAVE = 0,   /* wave64 cross-lane (DPP) sums, one LDS hop across waves */
       ADDRMS_REDUCE_LDS = 1 };  /* LDS-staged tree reduction                             */
enum { ADDRMS_FLAG_XCD_CONTIG = 1,    /* workgroups of one XCD cover a contiguous row range       */
       ADDRMS_FLAG_NONTEMPORAL = 2,   /* streaming cache policy on x/residual loads and stores    */
       ADDRMS_FLAG_PERSISTENT = 4,    /* grid = resident workgroups only; each walks several row
                                         blocks and prefetches the next block before reducing   */
       ADDRMS_FLAG_TWO_PASS = 8,      /* rows too long for the register row cache: read the row
                                         twice (sum of squares, then outputs); feasible only
                                         where no single-pass configuration covers N            */
       ADDRMS_FLAG_LDS_CACHE = 16,    /* rows somewhat too long for the registers: still one pass,
                                         the row cache continues in the workgroup's LDS (up to
                                         160 KB per CU: about 90 K elements per row at 1024 threads,
                                         about 110 K at 512 threads with 16-bit x, where a thread
                                         keeps 144 values in registers instead of 48).  Together
                                         with ADDRMS_FLAG_TWO_PASS: the hybrid form for rows beyond
                                         that -- registers and LDS hold what they can, and only the
                                         rest of each row is read twice                           */
       ADDRMS_FLAG_ALIGNED_SPAN = 64, /* rows that are not whole cache lines (N = 1000): a workgroup
                                         owns rows_per_wg rows that together ARE whole lines and walks
                                         them as one flat span of 16-byte pieces, so that every
                                         wave-wide access is aligned and every line is written whole
                                         by one instruction; row sums come from a segmented reduction
                                         in LDS.  threads_per_row x rows_per_wg threads share the span;
                                         vec x residual element size must be 16 bytes                */
       ADDRMS_FLAG_DEFER_STORE = 32 };/* the residual is written after the row reduction, the whole
                                         row at once and then the whole y row, instead of chunk by
                                         chunk while the row is still being read: a workgroup reads
                                         in one phase and writes in one phase (register-cached form
                                         only; results are the same bits)                         */

typedef struct addrms_cfg {
    int32_t vec;              /* elements per thread per vector access: 1, 2, 4, 8        */
    int32_t threads_per_row;  /* 8, 16, 32, or a multiple of 64 up to 1024                */
    int32_t rows_per_wg;      /* 1, 2, 4, 8, 16; threads_per_row*rows_per_wg <= 1024      */
    int32_t reduce;           /* ADDRMS_REDUCE_*                                          */
    int32_t unroll;           /* 1, 2, 4, 8: chunks whose loads are in flight together    */
    int32_t flags;            /* ADDRMS_FLAG_* bits                                       */
    int32_t max_waves_per_simd; /* 0 = as many as fit; 1..7 = cap on resident waves per SIMD,
                                 imposed by padding the workgroup's LDS allocation (fewer
                                 requests in flight can raise mixed read/write HBM efficiency) */
    int32_t walk;             /* persistent grids only: 0 = as many workgroups as are resident
                                 on the chip; 4, 16 = that many times more, so that each walks
                                 fewer row blocks (between the persistent and the ordinary grid) */
} addrms_cfg;

/* ---- run ------------------------------------------------------------------
 * addrms_run: one launch of the operator, in place, asynchronous on `stream`.
 *   x        device, [M, N] row-major (row stride N), x dtype.   in: x, out: y
 *   residual device, [M, N] row-major, residual dtype.            in: r, out: round(x+r)
 *   weight   device, [N], x dtype, read only
 *   eps      added to the mean of squares
 *   M, N     rows, row length.  M == 0 is a successful no-op; N <= 0 is INVALID_ARG;
 *            a row is held in registers between the reduction and the scaling
 *            (1024 threads x 32 cached values, at most 16 accesses per thread:
 *            even N up to 32768, odd N up to 16384); longer rows continue the
 *            cache in LDS (ADDRMS_FLAG_LDS_CACHE) while it fits and otherwise, up to
 *            2^28 elements, read what fits neither registers nor LDS twice (both flags)
 *            or the whole row twice (ADDRMS_FLAG_TWO_PASS); the default
 *            configuration selects these by itself; beyond that UNSUPPORTED_SHAPE
 *   dtype    addrms_dtype
 *   cfg      host; NULL = look (M, N, dtype) up in the specialised table
 *            (nearest tuned M for the same N and dtype), else the default cfg
 *   stream   a hipStream_t passed as void*; NULL = the default stream
 * Never synchronises, never allocates device memory.  Arguments are checked
 * before anything is launched (Section 3.3: invalid launches are pruned, not
 * attempted).  x, residual and weight must not overlap.  Re-entrant: host threads
 * may call it concurrently on their own streams.  It can be recorded into a HIP
 * graph (stream capture); the first launch of a cfg whose occupancy cap pads the
 * LDS allocation beyond 64 KiB raises that kernel's dynamic-LDS limit once per
 * process, so issue one such launch eagerly before capturing.
 */
int addrms_run(void* x, void* residual, const void* weight, float eps,
               int64_t M, int64_t N, int dtype, const addrms_cfg* cfg, void* stream);

/* The single untuned default configuration for (N, dtype): widest vector the
 * row length admits, 256 threads per row where the template covers N with
 * that, one row per workgroup, wave reduction. out: host. */
int addrms_default_cfg(int64_t N, int dtype, addrms_cfg* out);

/* ---- feasible region (Algorithm 1 line 18, DeriveFeasibleSpace; Section 3.3) */

/* Resources of the kernel instance a cfg selects, read back from the compiler
 * when the library was built, plus what the launch shape implies on one CU. */
typedef struct addrms_resources {
    int32_t chunks_per_thread;  /* ceil(N / (vec * threads_per_row))                   */
    int32_t vgprs;              /* architected vector registers per lane               */
    int32_t agprs;              /* accumulation registers per lane (same 512-entry file)*/
    int32_t sgprs;
    int32_t scratch_bytes;      /* per lane; nonzero means spills and is rejected      */
    int32_t lds_bytes;          /* per workgroup for this launch shape, occupancy padding included */
    int32_t max_threads;        /* workgroup-size bound the instance was compiled for  */
    int32_t waves_per_wg;
    int32_t waves_per_simd_regs;/* min(8, 512 / ceil8(vgprs + agprs))                  */
    int32_t wgs_per_cu;         /* resident workgroups per CU (registers, LDS, slots, cap) */
    int32_t waves_per_simd;     /* achieved = wgs_per_cu * waves_per_wg / 4 (rounded up)*/
    int32_t reserved[5];
} addrms_resources;

/* 0 if cfg is in the feasible region for (M, N, dtype), else ADDRMS_ERR_INFEASIBLE_CFG
 * (or INVALID_ARG / UNSUPPORTED_DTYPE).  `reason` (host, may be NULL) receives a
 * NUL-terminated constraint rationale, truncated to reason_len.  `res` (host, may be
 * NULL) receives the resources when the cfg got as far as selecting an instance. */
int addrms_cfg_feasible(const addrms_cfg* cfg, int64_t M, int64_t N, int dtype,
                        char* reason, size_t reason_len, addrms_resources* res);

/* Writes up to `cap` feasible cfgs into `out` (host, may be NULL when cap == 0)
 * and returns how many exist (>= 0), or a negative status.  `n_grid` (host, may be
 * NULL) receives the size of the knob grid that was pruned. Order is deterministic. */
int64_t addrms_enumerate_feasible(int64_t M, int64_t N, int dtype,
                                  addrms_cfg* out, int64_t cap, int64_t* n_grid);

/* ---- search (Algorithm 1 lines 19-23: Search, BuildSpecialized) -------------- */
enum { ADDRMS_SEARCH_GUIDED = 0, ADDRMS_SEARCH_EXHAUSTIVE = 1 };
/* Strategy families of the template beyond its base form (Level 1 of Algorithm 1 adds
 * them round by round; a search can be restricted to a subset). */
enum { ADDRMS_FAMILY_STREAMING = 1,      /* non-temporal cache policy (ADDRMS_FLAG_NONTEMPORAL)              */
       ADDRMS_FAMILY_OCCUPANCY_CAP = 2,  /* max_waves_per_simd != 0                                          */
       ADDRMS_FAMILY_GRID_MAPPING = 4,   /* XCD-contiguous mapping, the persistent grid and its walk length  */
       ADDRMS_FAMILY_BASE_ONLY = 8,      /* none of these: the base template only                            */
       ADDRMS_FAMILY_STORE_PHASE = 16 }; /* deferred residual store (ADDRMS_FLAG_DEFER_STORE)                */
/* Hints for the guided search, derived from profiler counters of an earlier round
 * (Algorithm 1 line 9, Suggest): they decide which neighbouring cfgs are tried first
 * and add a sweep mode; they never remove a candidate. */
enum { ADDRMS_HINT_LOWER_OCCUPANCY = 1,         /* memory system saturated: try fewer resident waves      */
       ADDRMS_HINT_HIGHER_OCCUPANCY = 2,        /* latency-bound: try more waves / more loads in flight   */
       ADDRMS_HINT_FEWER_LARGER_WORKGROUPS = 4, /* prefer whole rows per workgroup, persistent grids      */
       ADDRMS_HINT_WIDER_VECTORS = 8 };         /* instruction-bound: prefer wider vector accesses        */

typedef struct addrms_budget {
    double  max_wall_ms;     /* 0 = unlimited                                              */
    int32_t max_candidates;  /* distinct cfgs that may be measured; 0 = unlimited          */
    int32_t strategy;        /* ADDRMS_SEARCH_*                                            */
    int32_t top_k;           /* candidates re-tested at the end; 0 = 5 (max 8)             */
    int32_t warmup;          /* confirmation protocol; 0 = 20 (Section 4, "Performance     */
    int32_t reps;            /*   Measurement": 20 warm-up runs, mean of 100); 0 = 100.
                                The exhaustive strategy times every candidate with it.     */
    int32_t coarse_warmup;   /* screening protocol of the guided search; 0 = 3             */
    int32_t coarse_reps;     /* 0 = 15                                                     */
    int32_t skip_validation; /* nonzero: do not gate candidates on correctness (tests only)*/
    float   eps;             /* eps used for the tuning launches; 0 = 1e-6                 */
    int32_t hints;           /* ADDRMS_HINT_* bits; 0 = none                               */
    const char* log_path;    /* host; JSON-lines log of every candidate; NULL = none.  If the
                                file already holds a search of the same operator, shape and
                                format made on this architecture by this library version,
                                candidates it screened are not measured again (their logged
                                times and gate verdicts stand); only the Top-K confirmation
                                is repeated.  The search is appended to the file, one line
                                per candidate, flushed as written; a last line that a killed
                                search left incomplete is ignored, so searches cut short by
                                a signal or by max_wall_ms add up to a whole one.            */
    int32_t family_mask;     /* ADDRMS_FAMILY_* bits the search may use; 0 = all of them   */
    int32_t no_resume;       /* nonzero: ignore what log_path already holds, measure anew   */
} addrms_budget;

#define ADDRMS_MAX_TOPK 8
typedef struct addrms_tune_report {
    int64_t n_grid;          /* knob-grid points examined by the deriver                   */
    int64_t n_feasible;      /* size of the feasible region                                */
    int64_t n_measured;      /* distinct cfgs timed                                        */
    int64_t n_failed;        /* cfgs that failed the correctness gate or a launch          */
    int64_t best_found_at;   /* 1-based count of measured cfgs when the winner first ran   */
    double  best_us;         /* confirmed mean time of the returned cfg                    */
    double  default_us;      /* confirmed mean time of the default cfg                     */
    double  wall_ms;         /* whole call                                                 */
    double  time_to_best_ms; /* wall time until the winner was first measured              */
    addrms_cfg best;
    addrms_cfg default_cfg;
    int32_t n_topk;
    int32_t n_resumed;       /* candidates whose screening result came from the log         */
    addrms_cfg topk[ADDRMS_MAX_TOPK];    /* confirmed candidates (the default among them), fastest first */
    double  topk_us[ADDRMS_MAX_TOPK];
} addrms_tune_report;

/* addrms_tune: derive the feasible region for (M, N, dtype), search it on the
 * current HIP device with measured kernel time, gate every candidate on
 * agreement with the default configuration's output (bit-exact residual,
 * y within 1 unit in the last place), re-test the Top-K with the confirmation
 * protocol, store the winner in the specialised table and return it.
 * Blocking.  Allocates and frees its own device buffers (rotated so that the
 * timed launches stream from HBM rather than from cache).
 *   budget  host, may be NULL (all defaults)
 *   out_cfg host, required;  report host, may be NULL
 * With the environment variable ADDRMS_VERBOSE set (1: one line when a search starts and
 * one when it ends; 2: also one per candidate) every search reports on stderr, and the audit every
 * 500 candidates.
 */
int addrms_tune(int64_t M, int64_t N, int dtype, const addrms_budget* budget,
                addrms_cfg* out_cfg, addrms_tune_report* report);

/* The same search driven by caller-supplied measurement, so that its logic can
 * be exercised without a GPU.  measure returns 0 and a time in microseconds, or
 * nonzero if the candidate could not be run; validate returns 0 if the
 * candidate's output is acceptable.  Does not touch the specialised table. */
typedef struct addrms_backend {
    void* user;
    int (*validate)(void* user, const addrms_cfg* cfg);
    int (*measure)(void* user, const addrms_cfg* cfg, int warmup, int reps, double* mean_us);
} addrms_backend;

int addrms_tune_with_backend(int64_t M, int64_t N, int dtype, const addrms_budget* budget,
                             const addrms_backend* backend,
                             addrms_cfg* out_cfg, addrms_tune_report* report);

/* ---- general configuration (Algorithm 1 line 22, SelectGeneral) ----------------
 * One cfg for a whole set of shapes of one dtype: each shape is searched as in
 * addrms_tune (its winner goes to the specialised table, line 23); the Top-K of all
 * shapes, the default cfgs, and the universally feasible cfgs closest to each shape's
 * winner form the pool; every pool member that is feasible on every shape is timed on
 * every shape with the confirmation protocol; the winner maximises the geometric mean
 * over shapes of default_time / time (the aggregate of Section 3.1). */
#define ADDRMS_MAX_SHAPES 16
typedef struct addrms_shape { int64_t M, N; } addrms_shape;

typedef struct addrms_general_report {
    int32_t n_shapes;
    int32_t n_pool;                        /* universally feasible candidates that were timed  */
    double  geomean_speedup_general;       /* theta_gen against the default cfg of each shape  */
    double  geomean_speedup_specialized;   /* each shape's own winner against its default       */
    double  mean_speedup_general;          /* arithmetic mean of the same per-shape ratios      */
    double  wall_ms;
    double  default_us[ADDRMS_MAX_SHAPES];
    double  general_us[ADDRMS_MAX_SHAPES];
    double  specialized_us[ADDRMS_MAX_SHAPES];
    addrms_cfg specialized[ADDRMS_MAX_SHAPES];
} addrms_general_report;

/* shapes: host, n in 1..ADDRMS_MAX_SHAPES; out_general: host, required; report: host, may be NULL.
 * Blocking; allocates and frees device buffers shape by shape.  ADDRMS_ERR_NO_RESULT if no cfg is
 * feasible on all shapes. */
int addrms_select_general(const addrms_shape* shapes, int32_t n, int dtype, const addrms_budget* budget,
                          addrms_cfg* out_general, addrms_general_report* report);

/* The same selection over caller-supplied measurement: open() fills a backend for one
 * shape, close() releases it; at most one backend is open at a time. */
typedef struct addrms_backend_factory {
    void* user;
    int (*open)(void* user, int64_t M, int64_t N, int dtype, addrms_backend* out);
    void (*close)(void* user, addrms_backend* backend);
} addrms_backend_factory;

int addrms_select_general_with_backend(const addrms_shape* shapes, int32_t n, int dtype,
                                       const addrms_budget* budget, const addrms_backend_factory* factory,
                                       addrms_cfg* out_general, addrms_general_report* report);

/* ---- the outer loop (Algorithm 1 lines 6-32) with a fixed strategy list ----------
 * Round 0 uses the base template; each later round adds one strategy family (streaming
 * cache policy, occupancy cap, grid mapping, store phase) in that order -- the deterministic stand-in
 * for the planning agent's suggestions.  Per round: Validate the new family on the first
 * shape against the base default's output and roll it back if it fails (lines 13-14);
 * search every shape within the families enabled so far (lines 19-21); SelectGeneral and
 * BuildSpecialized (22-23); score = minus the geometric-mean speed-up of the specialised
 * table over the per-shape defaults (line 27); keep the incumbent (28-30).  Every round is
 * appended to budget->log_path as an "event":"round" line. */
#define ADDRMS_MAX_ROUNDS 5
typedef struct addrms_round_info {
    int32_t families;          /* ADDRMS_FAMILY_* bits enabled in this round (0 = base only)  */
    int32_t pass;              /* 1 if the family added in this round passed validation       */
    double  score;             /* -geomean speed-up of the specialised table                  */
    double  geomean_speedup_general;
    addrms_cfg general;
} addrms_round_info;
typedef struct addrms_rounds_report {
    int32_t n_rounds;
    int32_t best_round;
    double  wall_ms;
    addrms_round_info rounds[ADDRMS_MAX_ROUNDS];
    addrms_general_report best;   /* report of the incumbent round */
} addrms_rounds_report;

int addrms_tune_rounds(const addrms_shape* shapes, int32_t n, int dtype, const addrms_budget* budget,
                       addrms_cfg* out_general, addrms_rounds_report* report);
int addrms_tune_rounds_with_backend(const addrms_shape* shapes, int32_t n, int dtype, const addrms_budget* budget,
                                    const addrms_backend_factory* factory, addrms_cfg* out_general,
                                    addrms_rounds_report* report);

/* ---- audit of the feasible region's efficiency rules (Section 3.3) ----------------
 * The deriver prunes two kinds of configurations: invalid ones (a launch the hardware
 * or the compiled instance cannot take) and ones it calls obviously inefficient (at
 * most half the lanes of a row carrying data; fewer than two resident waves per SIMD;
 * an instance that spills registers; the two-pass or hybrid form or the LDS-continued cache where
 * the registers of a single pass would do; the aligned-span form where rows are whole cache
 * lines anyway).  The second kind is a judgement, and this
 * call puts it to the test: it enumerates the grid with those six rules switched off,
 * passes both the retained configurations and the ones each rule would have pruned
 * through the correctness gate and the screening protocol (budget.coarse_warmup /
 * coarse_reps, default 3 + 15 launches), and reports per rule how the pruned ones
 * compare.  A rule is sound on this shape if none of what it prunes is faster than
 * the best retained configuration (n_beating_best == 0, up to timing noise).
 * budget.max_candidates caps the configurations measured per PRUNED class (evenly
 * strided sample; 0 = all; the retained region is always measured in full, since its
 * best member is the yardstick); budget.max_wall_ms stops early (truncated = 1).  Nothing is added
 * to the table, and addrms_run still refuses the pruned configurations.  Blocking;
 * allocates and frees device memory. */
#define ADDRMS_AUDIT_RULES 6
typedef struct addrms_audit_rule {
    char    rule[24];          /* "lane_utilisation", "occupancy_floor", "scratch", "two_pass_needless",
                                  "lds_cache_needless", "span_needless"                                */
    int64_t n_pruned;          /* grid points this rule alone keeps out of the feasible region         */
    int32_t n_measured;        /* of those, validated and timed                                        */
    int32_t n_failed;          /* of those, failed the gate or the launch                              */
    int32_t n_in_top_decile;   /* timed pruned cfgs faster than the retained region's fastest decile   */
    int32_t n_beating_best;    /* timed pruned cfgs faster than the best retained cfg                  */
    double  best_us;           /* fastest pruned cfg (0 if none was timed)                             */
    double  median_us;
    addrms_cfg best;
} addrms_audit_rule;
typedef struct addrms_audit_report {
    int64_t n_retained;            /* size of the feasible region with every rule on                   */
    int32_t n_retained_measured;
    int32_t n_retained_failed;
    double  retained_best_us;
    double  retained_decile_us;    /* 10th percentile of the retained cfgs' times                      */
    double  retained_median_us;
    double  wall_ms;
    int32_t truncated;
    int32_t reserved;
    addrms_cfg retained_best;
    addrms_audit_rule rules[ADDRMS_AUDIT_RULES];
} addrms_audit_report;
int addrms_audit_rules(int64_t M, int64_t N, int dtype, const addrms_budget* budget, addrms_audit_report* report);
/* The same with validation and timing supplied by the caller (host-only; CPU tests). */
int addrms_audit_rules_with_backend(int64_t M, int64_t N, int dtype, const addrms_budget* budget,
                                    const addrms_backend* backend, addrms_audit_report* report);

/* addrms_measure: mean time in microseconds of `cfg` (NULL = table/default, as
 * in addrms_run) on (M, N, dtype) over `reps` launches after `warmup`, on
 * library-allocated synthetic buffers.  rotate != 0 cycles through enough
 * buffer sets to exceed the last-level caches; rotate == 0 reuses one set
 * (a cache-warm figure).  A batch shorter than 30 ms is preceded by that much
 * untimed running of the same kernel and then timed again, so that a call made
 * on an idle device does not time rising clocks.  Blocking; allocates and frees
 * device memory. */
int addrms_measure(const addrms_cfg* cfg, int64_t M, int64_t N, int dtype, float eps,
                   int warmup, int reps, int rotate, double* mean_us);

/* Timing statistics of one cfg: the batch mean of addrms_measure plus per-launch figures
 * from an event pair around every launch (which include the launch floor that back-to-back
 * launches hide).  out (host): mean_us = batch mean over `reps` launches, per_launch_mean_us,
 * median_us and min_us from the per-launch events.  Same arguments as addrms_measure. */
typedef struct addrms_time_stats {
    double mean_us, per_launch_mean_us, median_us, min_us, max_us;
    int32_t reps, buffer_sets;
} addrms_time_stats;
int addrms_measure_stats(const addrms_cfg* cfg, int64_t M, int64_t N, int dtype, float eps,
                         int warmup, int reps, int rotate, addrms_time_stats* out);

/* r(h): the resource upper bounds of the target the deriver works from (Algorithm 1, Input),
 * so that they can be checked against what the device reports. out: host. */
typedef struct addrms_hw_limits {
    int32_t compute_units, xcds, simds_per_cu, wave_size, max_waves_per_simd, regs_per_lane, reg_granule,
            lds_bytes_per_cu, lds_granule, max_threads_per_wg, max_access_bytes, reserved;
    double  hbm_bytes_per_s;
    int64_t last_level_cache_bytes, l2_bytes_per_xcd;
} addrms_hw_limits;
int addrms_get_hw_limits(addrms_hw_limits* out);

/* ---- specialised table D_spec: (dtype, N, M) -> cfg (Algorithm 1 line 23) ---- */
int addrms_table_insert(int64_t M, int64_t N, int dtype, const addrms_cfg* cfg, double mean_us);
/* Exact (dtype, N, M) entry if present, else the entry of the same (dtype, N)
 * whose M is nearest in ratio and whose cfg is feasible for the asked M.
 * Returns 0 and fills out (host), or ADDRMS_ERR_NO_RESULT. */
int addrms_table_lookup(int64_t M, int64_t N, int dtype, addrms_cfg* out);
int64_t addrms_table_size(void);
void addrms_table_clear(void);
/* Text file: a format line, "arch gfx950", "library <version>", then one entry per line.
 * load replaces nothing on failure: a missing or malformed file, one written for another
 * architecture or by a library of another major.minor version (whose kernel instances, and
 * with them feasibility and timings, differ) returns ADDRMS_ERR_IO and leaves the table as
 * it was.  save writes beside the target and renames over it.
 * Tune cache: if the environment variable ADDRMS_TABLE_FILE names a file, the library loads it once, before the
 * table is first consulted or extended (addrms_run with cfg == NULL, a lookup, an insertion, the end of a tuning
 * call), and rewrites it after every insertion, so that what one process tuned is what the next one runs.  A
 * file that exists but does not load is neither read nor overwritten. */
int addrms_table_save(const char* path);
int addrms_table_load(const char* path);

/* ---- probes used by tests and by the measurement report ------------------- */

/* rstd for each of n sums of squares: out[i] = fp32(1/sqrt(ss[i]/N + eps)),
 * computed by the same device routine the kernel uses.  ss: device, fp64[n];
 * out: device, fp32[n].  Asynchronous on stream. */
int addrms_rstd_probe(const double* ss, int64_t n, int64_t N, float eps, float* out, void* stream);

/* The correctness gate of the tuner (Algorithm 1 line 13, Validate; Section 3.1: d(S~(x), S(x)) <= eps over a
 * finite test set) applied to caller buffers: compares n elements of an output pair (y, residual) with a
 * reference pair.  residual must agree bit for bit; y may differ by at most `tol` units in the last place of
 * its storage format, +0 and -0 counting as equal.
 *   y, y_ref               device, n elements of the x dtype of `dtype`
 *   residual, residual_ref device, n elements of the residual dtype of `dtype`
 *   n                      0 .. 2^32-1 (the counters are 32 bits wide; more is INVALID_ARG)
 *   counts_out             device, 16-byte aligned; receives the verdict
 *   stream                 a hipStream_t passed as void*; NULL = the default stream
 * Blocking: allocates a buffer of per-workgroup partial counts (16 bytes per 4096 elements, at most 64 KiB),
 * runs the two kernels of the gate on `stream`, waits for them and frees the buffer.  The counts are exact and
 * cost the same whether nothing or everything disagrees (no atomics). */
typedef struct addrms_gate_counts {
    uint32_t residual_mismatches;  /* residual elements whose bits differ                          */
    uint32_t y_beyond_tol;         /* y elements further than tol units in the last place          */
    uint32_t y_max_distance;       /* largest y distance seen, in units in the last place          */
    uint32_t reserved;             /* written as 0                                                 */
} addrms_gate_counts;
int addrms_gate_probe(const void* y, const void* y_ref, const void* residual, const void* residual_ref, int64_t n,
                      int dtype, uint32_t tol, addrms_gate_counts* counts_out, void* stream);

/* addrms_gate_probe for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments and the same verdict in counts_out, but the
 * per-workgroup partial counts live in a 64 KiB array that is part of the library's device code (one copy per GPU,
 * held until the process ends), so this call allocates nothing, frees nothing and does not wait: both kernels
 * are only enqueued on `stream`, and counts_out is valid once the stream has reached them.  Nothing in it is a
 * memset, so a capturing caller records two kernel nodes.  n beyond 2^32-1 is INVALID_ARG as above (the array
 * itself never limits n: a launch uses at most 4096 slots whatever n is).  Every call on a GPU shares that GPU's
 * array: calls that may overlap in time on one GPU (different streams, concurrent graphs) race on it and must be
 * serialised by the caller; calls on one stream are ordered and safe. */
int addrms_gate_probe_noalloc(const void* y, const void* y_ref, const void* residual, const void* residual_ref,
                              int64_t n, int dtype, uint32_t tol, addrms_gate_counts* counts_out, void* stream);

/* Calibration kernel with the operator's traffic and none of its arithmetic:
 * reads [M,N] of x and of residual and writes both back (bitwise complemented),
 * 16 bytes per lane, streaming cache policy, three 256-thread workgroups per CU
 * (the fastest plain copy-like kernel found on MI355X; its rate is the practical
 * ceiling the operator is compared with, and its known byte counts calibrate the
 * profiler's HBM counters).  Same argument meaning as addrms_run. */
int addrms_stream_probe(void* x, void* residual, int64_t M, int64_t N, int dtype, void* stream);

/* The calibration traffic under the operator's constraint (Section 3.3: the organisation of registers and
 * shared memory is what a row-wise normalisation has to tune): one workgroup of threads_per_row threads owns one
 * row, every thread reads all its 16-byte pieces of both streams (at most 16 per stream), the workgroup meets at
 * a barrier -- where the operator has its row sum -- and only then writes the row back (bitwise complemented),
 * streaming cache policy.  wgs_per_cu > 0 caps the resident workgroups per CU through the dynamic LDS allocation
 * (0: no cap).  Swept over threads_per_row and wgs_per_cu it measures what holding a row across a reduction
 * costs by itself; the reports print its best beside the operator.  Same argument meaning and alignment rules
 * as addrms_stream_probe, except that each row of x must be a multiple of 16 bytes.  Asynchronous on `stream`;
 * allocates nothing.  threads_per_row must be a multiple of 64 in [64, 1024] that covers a row in at most 16
 * pieces per thread without idle whole chunks, else ADDRMS_ERR_INFEASIBLE_CFG. */
int addrms_row_probe(void* x, void* residual, int64_t M, int64_t N, int dtype, int threads_per_row, int wgs_per_cu,
                     void* stream);

/* What the HIP runtime on the current device reports for the kernel instance and
 * launch shape a cfg selects: registers and scratch from the loaded code object,
 * resident workgroups per CU from the runtime's occupancy query.  Fills vgprs
 * (architected + accumulation registers as the runtime counts them), scratch_bytes,
 * lds_bytes, max_threads, waves_per_wg, wgs_per_cu and waves_per_simd of `out` (host);
 * other fields are zero.  Used to pin the deriver's model against the device. */
int addrms_device_resources(const addrms_cfg* cfg, int64_t M, int64_t N, int dtype, addrms_resources* out);

/* Bytes the operator must move for (M, N, dtype): every x and residual element
 * read once and written once, weight read once.  Negative on bad arguments. */
int64_t addrms_algorithmic_bytes(int64_t M, int64_t N, int dtype);

/* Static storage owned by the library; valid until the thread's next failing call. */
const char* addrms_last_error(void);
const char* addrms_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ADDRMS_H */
