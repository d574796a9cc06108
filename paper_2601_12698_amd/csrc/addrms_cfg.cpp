// Feasible-region deriver (Algorithm 1 line 18, DeriveFeasibleSpace; Section 3.3:
// ranges and candidate sets are derived from the hardware's resource limits, and
// combinations that would fail to compile, launch invalidly or be obviously
// inefficient are pruned, each with a stated rationale).
//
// Host-only: no HIP call is made here, so the region can be derived on a machine
// without a GPU.  Register, scratch and LDS figures of every kernel instance
// come from the compiler's resource report captured when the library was built.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>
#include <unordered_map>

#include "addrms_internal.h"

namespace addrms_host {

// ---- error text -------------------------------------------------------------
static thread_local std::string g_error;

int fail(int status, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_error = buf;
    return status;
}
void clear_error() { g_error.clear(); }
static const char* last_error() { return g_error.c_str(); }

// ---- hardware ---------------------------------------------------------------
const HwLimits& hw()
{
    static const HwLimits limits;
    return limits;
}

// ---- instances ----------------------------------------------------------------
static const Instance kInstances[] = {
#include "gen_instances.inc"
};
static const InstanceRes kInstanceRes[] = {
#include "gen_resources.inc"
};
static_assert(sizeof(kInstances) / sizeof(kInstances[0]) == sizeof(kInstanceRes) / sizeof(kInstanceRes[0]),
              "instance list and resource report disagree");

int n_instances() { return static_cast<int>(sizeof(kInstances) / sizeof(kInstances[0])); }
const Instance& instance(int idx) { return kInstances[idx]; }
const InstanceRes& instance_res(int idx) { return kInstanceRes[idx]; }

const char* op_name(int op)
{
    return op == OP_SILUMUL ? "silu_and_mul" : op == OP_MERGE ? "merge_attn_states" : "add_rmsnorm";
}

static uint32_t inst_key(int op, int dt, int vec, int cpt, int unr, int nt, int df)
{
    return (static_cast<uint32_t>(op) << 28) | (static_cast<uint32_t>(dt) << 25) | (static_cast<uint32_t>(vec) << 20) |
           (static_cast<uint32_t>(cpt) << 8) | (static_cast<uint32_t>(unr) << 2) | (static_cast<uint32_t>(df) << 1) |
           static_cast<uint32_t>(nt);      // cpt codes reach 300 + 32: twelve bits
}

int find_instance(int op, int dt, int vec, int cpt, int unr, int nt, int df)
{
    static const std::unordered_map<uint32_t, int> index = [] {
        std::unordered_map<uint32_t, int> m;
        for (int i = 0; i < n_instances(); ++i)
            m[inst_key(kInstances[i].op, kInstances[i].dt, kInstances[i].vec, kInstances[i].cpt, kInstances[i].unr, kInstances[i].nt,
                       kInstances[i].df)] = i;
        return m;
    }();
    auto it = index.find(inst_key(op, dt, vec, cpt, unr, nt, df));
    return it == index.end() ? -1 : it->second;
}

bool cpt_supported(int op, int cpt)
{
    for (int i = 0; i < n_instances(); ++i)
        if (kInstances[i].op == op && kInstances[i].cpt == cpt) return true;
    return false;
}

// ---- formats -------------------------------------------------------------------
bool dtype_valid(int dtype, int op)
{
    if (dtype < ADDRMS_BF16 || dtype > ADDRMS_FP32) return false;
    if (op == OP_MERGE) return dtype == ADDRMS_BF16 || dtype == ADDRMS_FP16;   // 16-bit partial outputs
    return op == OP_ADDRMS || dtype != ADDRMS_FP16_RES32;     // only add+RMSNorm has a separate residual stream
}

int64_t algorithmic_bytes(int op, int64_t M, int64_t N, int dtype)
{
    if (op == OP_SILUMUL) return M * N * 3 * x_bytes(dtype);                   // read gate and up, write out
    if (op == OP_MERGE) return M * (N * 3 * x_bytes(dtype) + 12);              // two parts in, one out, three fp32 scores
    return M * N * (2 * x_bytes(dtype) + 2 * r_bytes(dtype)) + N * x_bytes(dtype);
}
int x_bytes(int dtype) { return dtype == ADDRMS_FP32 ? 4 : 2; }
int r_bytes(int dtype) { return (dtype == ADDRMS_FP32 || dtype == ADDRMS_FP16_RES32) ? 4 : 2; }
const char* dtype_name(int dtype)
{
    switch (dtype) {
    case ADDRMS_BF16: return "bf16";
    case ADDRMS_FP16: return "fp16";
    case ADDRMS_FP16_RES32: return "fp16_res32";
    case ADDRMS_FP32: return "fp32";
    default: return "?";
    }
}

// ---- small helpers -----------------------------------------------------------
static const int kVecs[] = {8, 4, 2, 1};
static const int kRows[] = {1, 2, 4, 8, 16};
static const int kUnrolls[] = {1, 2, 4, 8};
static const int kWalks[] = {0, 4, 16};

static bool in_set(int v, const int* set, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        if (set[i] == v) return true;
    return false;
}
static bool tpr_valid(int t) { return t == 8 || t == 16 || t == 32 || (t >= 64 && t <= 1024 && t % 64 == 0); }
static int round_up(int v, int g) { return (v + g - 1) / g * g; }

bool cfg_equal(const addrms_cfg& a, const addrms_cfg& b)
{
    return a.vec == b.vec && a.threads_per_row == b.threads_per_row && a.rows_per_wg == b.rows_per_wg &&
           a.reduce == b.reduce && a.unroll == b.unroll && a.flags == b.flags &&
           a.max_waves_per_simd == b.max_waves_per_simd && a.walk == b.walk;
}
uint64_t cfg_key(const addrms_cfg& c)
{
    return (static_cast<uint64_t>(c.vec) << 40) | (static_cast<uint64_t>(c.threads_per_row) << 28) |
           (static_cast<uint64_t>(c.rows_per_wg) << 20) | (static_cast<uint64_t>(c.reduce) << 16) |
           (static_cast<uint64_t>(c.unroll) << 12) | (static_cast<uint64_t>(c.max_waves_per_simd & 0xf) << 8) |
           static_cast<uint64_t>(c.flags & 0xff) | (static_cast<uint64_t>(c.walk & 0xff) << 48);
}
std::string cfg_json(const addrms_cfg& c)
{
    char buf[256];
    snprintf(buf, sizeof buf,
             "{\"vec\":%d,\"threads_per_row\":%d,\"rows_per_wg\":%d,\"reduce\":%d,\"unroll\":%d,\"flags\":%d,"
             "\"max_waves_per_simd\":%d,\"walk\":%d}",
             c.vec, c.threads_per_row, c.rows_per_wg, c.reduce, c.unroll, c.flags, c.max_waves_per_simd, c.walk);
    return buf;
}

int reduction_lds_bytes(const addrms_cfg& c, int op)
{
    if (op != OP_ADDRMS) return 0;          // no reduction, no LDS
    // a persistent workgroup alternates between two regions from one row block to the next
    const int regions = (c.flags & ADDRMS_FLAG_PERSISTENT) ? 2 : 1;
    if (c.reduce == ADDRMS_REDUCE_LDS) return regions * c.threads_per_row * c.rows_per_wg * 8;
    return c.threads_per_row > 64 ? regions * c.rows_per_wg * 16 * 8 : 0;   // one fp64 slot per wave of a row
}

int capped_wgs_per_cu(const addrms_cfg& c)
{
    if (c.max_waves_per_simd <= 0) return 0;
    const int waves_per_wg = std::max(1, c.threads_per_row * c.rows_per_wg / hw().wave_size);
    return c.max_waves_per_simd * hw().simds_per_cu / waves_per_wg;   // 0: one workgroup already exceeds the cap
}

// LDS padding such that exactly `wgs` workgroups fit the CU's LDS: the largest
// whole number of allocation granules g with wgs * g <= total; it binds only if
// (wgs + 1) * g exceeds the total.  Returns 0 if no such padding exists.
static int lds_padding_for_wgs(int wgs)
{
    const int total = hw().lds_bytes_per_cu / hw().lds_granule;
    const int g = total / wgs;
    if (g < 1 || (wgs + 1) * g <= total) return 0;
    return g * hw().lds_granule;
}

bool cfg_in_families(const addrms_cfg& c, int mask)
{
    if (mask == 0) return true;
    if ((c.flags & ADDRMS_FLAG_NONTEMPORAL) && !(mask & ADDRMS_FAMILY_STREAMING)) return false;
    if (c.max_waves_per_simd != 0 && !(mask & ADDRMS_FAMILY_OCCUPANCY_CAP)) return false;
    if ((c.flags & (ADDRMS_FLAG_XCD_CONTIG | ADDRMS_FLAG_PERSISTENT)) && !(mask & ADDRMS_FAMILY_GRID_MAPPING)) return false;
    if ((c.flags & ADDRMS_FLAG_DEFER_STORE) && !(mask & ADDRMS_FAMILY_STORE_PHASE)) return false;
    return true;
}

int lds_bytes_for(const addrms_cfg& c, int op)
{
    const int need = reduction_lds_bytes(c, op);
    const int wgs = capped_wgs_per_cu(c);
    if (c.max_waves_per_simd <= 0) return need;
    if (wgs == 0) return 0;
    const int pad = lds_padding_for_wgs(wgs);
    return pad == 0 ? 0 : std::max(need, pad);
}
int64_t n_row_blocks(const addrms_cfg& c, int64_t M) { return (M + c.rows_per_wg - 1) / c.rows_per_wg; }
int64_t n_workgroups(const addrms_cfg& c, int64_t M, int wgs_per_cu)
{
    const int64_t blocks = n_row_blocks(c, M);
    if (!(c.flags & ADDRMS_FLAG_PERSISTENT)) return blocks;
    return std::min<int64_t>(blocks, static_cast<int64_t>(hw().compute_units) * std::max(1, wgs_per_cu) * std::max(1, c.walk));
}

// ---- the rules ------------------------------------------------------------------
static Feas infeasible(const char* rule, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
// Walking the whole grid rejects millions of points whose rationale nobody reads: the walk
// switches the text off and keeps only the rule tag.
static thread_local bool g_rationale_wanted = true;
static Feas infeasible(const char* rule, const char* fmt, ...)
{
    Feas f;
    f.status = ADDRMS_ERR_INFEASIBLE_CFG;
    f.rule = rule;
    if (g_rationale_wanted) {
        char buf[384];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        f.reason = buf;
    }
    return f;
}

// True if the single-pass form has a default configuration for rows of N elements, i.e. if
// some launch shape holds such a row in its register cache and passes every rule.
static bool single_pass_default(int64_t N, int dtype, int op, addrms_cfg* out);
static bool single_pass_covers(int64_t N, int dtype, int op)
{
    static thread_local int64_t last_n = -1;
    static thread_local int last_dt = -1, last_op = -1;
    static thread_local bool last = false;
    if (N == last_n && dtype == last_dt && op == last_op) return last;
    addrms_cfg unused{};
    const bool found = single_pass_default(N, dtype, op, &unused);
    last_n = N; last_dt = dtype; last_op = op; last = found;
    return found;
}

Feas check_cfg(const addrms_cfg& c, int64_t M, int64_t N, int dtype, int op, int relax)
{
    const HwLimits& L = hw();
    Feas f;
    if (!dtype_valid(dtype, op)) {
        f.status = ADDRMS_ERR_UNSUPPORTED_DTYPE;
        f.reason = op == OP_ADDRMS ? "dtype is not one of bf16, fp16, fp16_res32, fp32"
                   : op == OP_MERGE ? "dtype is not one of bf16, fp16" : "dtype is not one of bf16, fp16, fp32";
        return f;
    }
    if (M < 0 || N <= 0) {
        f.status = ADDRMS_ERR_INVALID_ARG;
        f.reason = "M must be >= 0 and N must be > 0";
        return f;
    }
    // -- the knob grid itself
    if (!in_set(c.vec, kVecs, 4)) return infeasible("grid", "vec=%d: vector width must be 1, 2, 4 or 8 elements", c.vec);
    if (!tpr_valid(c.threads_per_row))
        return infeasible("grid", "threads_per_row=%d: a row is reduced either inside one wave64 (8, 16 or 32 lanes) or by "
                          "whole waves (a multiple of 64 up to %d)", c.threads_per_row, L.max_threads_per_wg);
    if (!in_set(c.rows_per_wg, kRows, 5)) return infeasible("grid", "rows_per_wg=%d: must be 1, 2, 4, 8 or 16", c.rows_per_wg);
    if (c.reduce != ADDRMS_REDUCE_WAVE && c.reduce != ADDRMS_REDUCE_LDS)
        return infeasible("grid", "reduce=%d: must be wave (0) or lds (1)", c.reduce);
    if (op != OP_ADDRMS && c.reduce != 0)
        return infeasible("grid", "reduce=%d: %s has no reduction; the knob must stay 0", c.reduce, op_name(op));
    if (!in_set(c.unroll, kUnrolls, 4)) return infeasible("grid", "unroll=%d: must be 1, 2, 4 or 8", c.unroll);
    if (c.flags & ~(ADDRMS_FLAG_XCD_CONTIG | ADDRMS_FLAG_NONTEMPORAL | ADDRMS_FLAG_PERSISTENT | ADDRMS_FLAG_TWO_PASS |
                    ADDRMS_FLAG_LDS_CACHE | ADDRMS_FLAG_DEFER_STORE | ADDRMS_FLAG_ALIGNED_SPAN))
        return infeasible("grid", "flags=0x%x: unknown bits set", c.flags);
    const bool span = (c.flags & ADDRMS_FLAG_ALIGNED_SPAN) != 0;
    if (span && op != OP_ADDRMS)
        return infeasible("grid", "flags=0x%x: only add+RMSNorm has the aligned-span form", c.flags);
    if (span && (c.flags & (ADDRMS_FLAG_TWO_PASS | ADDRMS_FLAG_LDS_CACHE | ADDRMS_FLAG_PERSISTENT)))
        return infeasible("grid", "flags=0x%x: the aligned-span form is a register-cached single pass over an ordinary grid", c.flags);
    if (span && c.reduce != ADDRMS_REDUCE_WAVE)
        return infeasible("grid", "reduce=%d: the aligned-span form has its own segmented reduction; the knob must stay 0", c.reduce);
    // both long-row flags together name the hybrid form: what fits stays on the chip, the rest is read twice
    const bool hybrid = (c.flags & ADDRMS_FLAG_TWO_PASS) && (c.flags & ADDRMS_FLAG_LDS_CACHE);
    const bool two_pass = (c.flags & ADDRMS_FLAG_TWO_PASS) != 0 && !hybrid;
    const bool lds_cache = (c.flags & ADDRMS_FLAG_LDS_CACHE) != 0 && !hybrid;
    const bool defer = (c.flags & ADDRMS_FLAG_DEFER_STORE) != 0;
    if (defer && op != OP_ADDRMS)
        return infeasible("grid", "flags=0x%x: %s has no residual stream whose store could be deferred", c.flags, op_name(op));
    if (defer && (two_pass || lds_cache || hybrid))
        return infeasible("grid", "flags=0x%x: the deferred residual store exists for the register-cached form only (the "
                          "two-pass form writes everything in its second pass anyway)", c.flags);
    if (c.walk != 0 && c.walk != 4 && c.walk != 16)
        return infeasible("grid", "walk=%d: must be 0 (grid = resident workgroups) or 4 or 16 times as many", c.walk);
    if (c.walk != 0 && !(c.flags & ADDRMS_FLAG_PERSISTENT))
        return infeasible("grid", "walk=%d sizes a persistent grid; without ADDRMS_FLAG_PERSISTENT there is one workgroup per "
                          "row block and nothing to size", c.walk);
    if ((two_pass || lds_cache || hybrid) && op != OP_ADDRMS)
        return infeasible("grid", "flags=0x%x: only add+RMSNorm has forms for long rows", c.flags);
    if ((two_pass || lds_cache || hybrid) && (c.flags & ADDRMS_FLAG_PERSISTENT))
        return infeasible("grid", "flags=0x%x: the long-row forms have no persistent grid", c.flags);
    if (c.max_waves_per_simd < 0 || c.max_waves_per_simd >= L.max_waves_per_simd)
        return infeasible("grid", "max_waves_per_simd=%d: must be 0 (no cap) or 1..%d", c.max_waves_per_simd,
                          L.max_waves_per_simd - 1);

    const int xb = x_bytes(dtype), rb = r_bytes(dtype);
    // -- vectorisation and alignment
    if (N % c.vec != 0)
        return infeasible("vec_divides_n", "vec=%d does not divide N=%lld: rows after the first would start misaligned and the last "
                          "vector of a row would straddle two rows", c.vec, (long long)N);
    if (c.vec * xb > L.max_access_bytes)
        return infeasible("access_width", "vec=%d x %d-byte elements is %d bytes per lane: wider than the %d-byte global access",
                          c.vec, xb, c.vec * xb, L.max_access_bytes);
    // (the residual stream may take two accesses: fp32 residual at vec=8; not so in the aligned-span form)
    if (span) {
        if (c.vec * rb != L.max_access_bytes)
            return infeasible("span_piece", "vec=%d x %d-byte residual elements is %d bytes: the aligned-span form moves the residual "
                              "in %d-byte pieces, one access per lane", c.vec, rb, c.vec * rb, L.max_access_bytes);
        const int64_t xspan = static_cast<int64_t>(c.rows_per_wg) * N * xb, rspan = static_cast<int64_t>(c.rows_per_wg) * N * rb;
        if (xspan % kLineBytes != 0 || rspan % kLineBytes != 0)
            return infeasible("span_alignment", "%d rows of N=%lld are %lld and %lld bytes: not whole %d-byte cache lines, so "
                              "consecutive workgroups would still share lines", c.rows_per_wg, (long long)N, (long long)xspan,
                              (long long)rspan, kLineBytes);
        if ((N * xb) % kLineBytes == 0 && (N * rb) % kLineBytes == 0) {
            if (!(relax & RELAX_SPAN_NEEDLESS))
                return infeasible("span_needless", "rows of N=%lld are whole cache lines already (%lld and %lld bytes): the ordinary "
                                  "form is aligned and needs no segmented reduction", (long long)N, (long long)(N * xb), (long long)(N * rb));
            if (!f.soft_rule[0]) f.soft_rule = "span_needless";
        }
    }

    // -- launch validity
    const int threads = c.threads_per_row * c.rows_per_wg;
    if (threads > L.max_threads_per_wg)
        return infeasible("wg_size", "workgroup of %d x %d = %d threads exceeds the %d-thread limit (invalid launch)",
                          c.threads_per_row, c.rows_per_wg, threads, L.max_threads_per_wg);
    if (threads % L.wave_size != 0)
        return infeasible("whole_waves", "workgroup of %d threads is not a whole number of %d-lane waves: the cross-lane reduction "
                          "needs full waves", threads, L.wave_size);

    // -- register row cache: the row slice of a thread must fit in registers (single-pass form)
    const int64_t per_pass = static_cast<int64_t>(c.vec) * c.threads_per_row;
    const int64_t need = (N + per_pass - 1) / per_pass;
    int64_t lds_cache_bytes = 0;
    // Long-row forms: values per thread kept in registers.  The instance compiled for at most 512 threads keeps 144
    // instead of 48; it is taken where the 48-value instance cannot hold the whole row on the chip (registers + LDS)
    // at this launch shape, the workgroup is small enough, and the instance exists and does not spill.
    int64_t long_row_reg_elems = kLdsCacheRegElems;
    int long_row_cpt_base = kLdsCacheCptBase;
    if ((lds_cache || hybrid) && threads <= kLdsCacheBigMaxThreads && kLdsCacheBigRegElems % c.vec == 0) {
        const int64_t chunk_bytes = static_cast<int64_t>(c.rows_per_wg) * per_pass * 4;
        const int64_t fit = (L.lds_bytes_per_cu - reduction_lds_bytes(c, op)) / chunk_bytes;
        const int big = find_instance(op, dtype, c.vec, kLdsCacheBigCptBase + kLdsCacheBigRegElems / c.vec, c.unroll,
                                      (c.flags & ADDRMS_FLAG_NONTEMPORAL) ? 1 : 0, 0);
        if (need > kLdsCacheRegElems / c.vec + fit && big >= 0 && kInstanceRes[big].scratch == 0) {
            long_row_reg_elems = kLdsCacheBigRegElems;
            long_row_cpt_base = kLdsCacheBigCptBase;
        }
    }
    if (two_pass) {
        if (N * c.rows_per_wg > kMaxTwoPassElemsPerWg)
            return infeasible("row_too_long", "N=%lld x rows_per_wg=%d exceeds the %lld elements a workgroup addresses with "
                              "32-bit offsets", (long long)N, c.rows_per_wg, (long long)kMaxTwoPassElemsPerWg);
        if (single_pass_covers(N, dtype, op)) {
            if (!(relax & RELAX_TWO_PASS_NEEDLESS))
                return infeasible("two_pass_needless", "N=%lld fits the register row cache of a single-pass configuration: "
                                  "reading every row twice is obviously inefficient", (long long)N);
            if (!f.soft_rule[0]) f.soft_rule = "two_pass_needless";
        }
    } else if (lds_cache) {
        const int64_t reg_chunks = long_row_reg_elems / c.vec;
        // Needless where the plain form takes the same launch shape: it has an instance for this chunk count and that
        // instance admits this workgroup size (32 cached values up to 1024 threads, 64 up to 256).  A chunk count that
        // fits this form's 48 register values but not a plain instance - 17 to 32 one-element chunks, or 33 to 48
        // values in a workgroup of more than 256 threads - runs here with nothing parked: the register part clamps
        // its unused chunks.
        const bool plain_takes_it = cpt_supported(op, static_cast<int>(need)) && need * c.vec <= kMaxElemsPerThread &&
                                    (need * c.vec <= kMaxElemsPerThread / 2 || c.threads_per_row * c.rows_per_wg <= 256);
        if (need <= reg_chunks && plain_takes_it)
            return infeasible("lds_cache_needless", "N=%lld over %d threads at vec=%d is %lld chunks per thread: they fit the "
                              "registers of the plain form, there is nothing to park in LDS", (long long)N, c.threads_per_row,
                              c.vec, (long long)need);
        f.lds_chunks = static_cast<int>(std::max<int64_t>(0, need - reg_chunks));
        lds_cache_bytes = static_cast<int64_t>(c.rows_per_wg) * f.lds_chunks * per_pass * 4;
        if (lds_cache_bytes + reduction_lds_bytes(c, op) > L.lds_bytes_per_cu)
            return infeasible("lds_cache_too_big", "parking %lld chunks per thread takes %lld bytes of LDS per workgroup; a CU has %d",
                              (long long)std::max<int64_t>(0, need - reg_chunks), (long long)lds_cache_bytes, L.lds_bytes_per_cu);
        if (single_pass_covers(N, dtype, op)) {
            if (!(relax & RELAX_LDS_CACHE_NEEDLESS))
                return infeasible("lds_cache_needless", "N=%lld fits the register row cache of a single-pass configuration: "
                                  "a detour through LDS is obviously inefficient", (long long)N);
            if (!f.soft_rule[0]) f.soft_rule = "lds_cache_needless";
        }
    } else if (hybrid) {
        const int64_t reg_chunks = long_row_reg_elems / c.vec;
        if (N * c.rows_per_wg > kMaxTwoPassElemsPerWg)
            return infeasible("row_too_long", "N=%lld x rows_per_wg=%d exceeds the %lld elements a workgroup addresses with "
                              "32-bit offsets", (long long)N, c.rows_per_wg, (long long)kMaxTwoPassElemsPerWg);
        const int64_t chunk_bytes = static_cast<int64_t>(c.rows_per_wg) * per_pass * 4;     // one parked chunk of every thread
        const int64_t fit = (L.lds_bytes_per_cu - reduction_lds_bytes(c, op)) / chunk_bytes;
        if (need <= reg_chunks + fit)
            return infeasible("hybrid_needless", "N=%lld over %d threads at vec=%d is %lld chunks per thread: registers (%lld) and "
                              "LDS (%lld) hold them all, nothing has to be read twice", (long long)N, c.threads_per_row, c.vec,
                              (long long)need, (long long)reg_chunks, (long long)fit);
        if (single_pass_covers(N, dtype, op)) {
            if (!(relax & RELAX_TWO_PASS_NEEDLESS))
                return infeasible("two_pass_needless", "N=%lld fits the register row cache of a single-pass configuration: "
                                  "reading part of every row twice is obviously inefficient", (long long)N);
            if (!f.soft_rule[0]) f.soft_rule = "two_pass_needless";
        }
        if (fit < 1)
            return infeasible("hybrid_no_lds", "not one chunk per thread fits the LDS of a CU at this workgroup size: this is the "
                              "two-pass form");
        f.lds_chunks = static_cast<int>(fit);
        lds_cache_bytes = fit * chunk_bytes;
    } else if (need * c.vec > kMaxElemsPerThread)
        return infeasible("row_cache", "N=%lld over %d threads at vec=%d needs %lld values per thread in registers; the row cache "
                          "holds %d (more would spill or leave under %d waves per SIMD)",
                          (long long)N, c.threads_per_row, c.vec, (long long)(need * c.vec), kMaxElemsPerThread,
                          kMinWavesPerSimd);
    if (span && need != 1 && need != 2 && need != 4)
        return infeasible("no_instance", "chunks per thread = %lld: the aligned-span form exists for 1, 2 and 4", (long long)need);
    if (!two_pass && !lds_cache && !hybrid && !cpt_supported(op, static_cast<int>(need)))
        return infeasible("no_instance", "chunks per thread = %lld has no compiled instance (%s)", (long long)need,
                          op == OP_ADDRMS ? "1-8, 10, 12, 14, 16 exist" : op == OP_MERGE ? "1-4 exist" : "1-8 exist");
    f.res.chunks_per_thread = static_cast<int>(need);
    const double util = static_cast<double>(N) / static_cast<double>(per_pass * need);
    if (util <= 0.5 && (relax & RELAX_LANE_UTILISATION)) {
        if (!f.soft_rule[0]) f.soft_rule = "lane_utilisation";
    } else if (util <= 0.5)
        return infeasible("lane_utilisation", "only %.0f%% of the %lld lane slots of a row would carry data (obviously inefficient: a "
                          "narrower row does the same work)", util * 100.0, (long long)(per_pass * need));
    if (c.unroll > need)
        return infeasible("unroll_gt_chunks", "unroll=%d exceeds the %lld chunks a thread has", c.unroll, (long long)need);

    // -- problem-size rules
    const int min_rows = std::max(1, L.wave_size / c.threads_per_row);
    if (c.rows_per_wg > std::max<int64_t>(M, min_rows) && c.rows_per_wg > min_rows)
        return infeasible("rows_gt_m", "rows_per_wg=%d exceeds the %lld rows there are", c.rows_per_wg, (long long)M);
    if ((c.flags & ADDRMS_FLAG_XCD_CONTIG) && n_row_blocks(c, M) < 2 * L.xcds)
        return infeasible("xcd_identity", "XCD-contiguous mapping with fewer than %d workgroups is the identity mapping",
                          2 * L.xcds);

    // -- compiled instance and its resources
    const int cpt_code = two_pass ? 0 : (hybrid || lds_cache) ? long_row_cpt_base + static_cast<int>(long_row_reg_elems) / c.vec
                         : span ? kSpanCptBase + static_cast<int>(need) : static_cast<int>(need);
    const int idx = find_instance(op, dtype, c.vec, cpt_code, c.unroll, (c.flags & ADDRMS_FLAG_NONTEMPORAL) ? 1 : 0, defer ? 1 : 0);
    if (idx < 0)
        return infeasible("no_instance", "no compiled instance for dtype=%s vec=%d chunks=%lld unroll=%d", dtype_name(dtype), c.vec,
                          (long long)need, c.unroll);
    f.inst = idx;
    const Instance& in = kInstances[idx];
    const InstanceRes& r = kInstanceRes[idx];
    addrms_resources& o = f.res;
    o.vgprs = r.vgprs; o.agprs = r.agprs; o.sgprs = r.sgprs; o.scratch_bytes = r.scratch;
    o.max_threads = in.maxt;
    o.lds_bytes = reduction_lds_bytes(c, op) + static_cast<int>(lds_cache_bytes) + r.lds_static;
    if (span)   // one fp64 sum per piece slot, then one fp32 rstd per row (rounded up to whole doubles)
        o.lds_bytes = threads * static_cast<int>(need) * 8 + round_up(c.rows_per_wg * 4, 8) + r.lds_static;
    o.waves_per_wg = threads / L.wave_size;
    if (r.scratch > 0 && (relax & RELAX_SCRATCH)) {
        if (!f.soft_rule[0]) f.soft_rule = "scratch";
    } else if (r.scratch > 0)
        return infeasible("scratch", "instance spills %d bytes per lane to scratch memory", r.scratch);
    if (threads > in.maxt)
        return infeasible("wg_bound", "instance holds %d values per thread and was compiled for workgroups of at most %d threads; "
                          "%d requested", c.vec * static_cast<int>(need), in.maxt, threads);

    // -- occupancy on one CU
    const int regs = round_up(std::max(1, r.vgprs + r.agprs), L.reg_granule);
    o.waves_per_simd_regs = std::min(L.max_waves_per_simd, L.regs_per_lane / regs);
    const int waves_cu_regs = o.waves_per_simd_regs * L.simds_per_cu;
    int wgs = waves_cu_regs / o.waves_per_wg;
    if (o.lds_bytes > 0) wgs = std::min(wgs, L.lds_bytes_per_cu / round_up(o.lds_bytes, L.lds_granule));
    wgs = std::min(wgs, o.waves_per_wg > 1 ? L.max_multiwave_wgs_per_cu : L.max_wgs_per_cu);
    // -- requested occupancy cap: must bind, and must be imposable by LDS padding
    if (c.max_waves_per_simd > 0) {
        const int cap = capped_wgs_per_cu(c);
        if (cap < 1)
            return infeasible("cap_below_one_wg", "max_waves_per_simd=%d is less than one %d-wave workgroup spread over "
                              "%d SIMDs", c.max_waves_per_simd, o.waves_per_wg, L.simds_per_cu);
        if ((c.max_waves_per_simd - 1) * L.simds_per_cu / o.waves_per_wg == cap)
            return infeasible("cap_redundant", "max_waves_per_simd=%d and %d both leave %d workgroups per CU",
                              c.max_waves_per_simd, c.max_waves_per_simd - 1, cap);
        if (cap >= wgs)
            return infeasible("cap_not_binding", "max_waves_per_simd=%d allows %d workgroups per CU but only %d fit anyway: "
                              "the cap changes nothing", c.max_waves_per_simd, cap, wgs);
        const int pad = lds_padding_for_wgs(cap);
        if (pad == 0 || pad < o.lds_bytes)
            return infeasible("cap_not_imposable", "no LDS padding leaves exactly %d workgroups per CU", cap);
        o.lds_bytes = pad;
        wgs = cap;
    }
    o.wgs_per_cu = wgs;
    if (wgs < 1)
        return infeasible("occupancy", "workgroup of %d waves at %d registers per lane does not fit one CU (%d wave slots by "
                          "registers, %d bytes of LDS)", o.waves_per_wg, regs, waves_cu_regs, o.lds_bytes);
    o.waves_per_simd = (wgs * o.waves_per_wg + L.simds_per_cu - 1) / L.simds_per_cu;
    if ((c.flags & ADDRMS_FLAG_PERSISTENT) &&
        n_row_blocks(c, M) <= static_cast<int64_t>(L.compute_units) * wgs * std::max(1, c.walk))
        return infeasible("persistent_identity", "all %lld row blocks get a workgroup of their own (%d CUs x %d workgroups x "
                          "walk %d): this persistent grid is the ordinary grid", (long long)n_row_blocks(c, M),
                          L.compute_units, wgs, std::max(1, c.walk));
    if (o.waves_per_simd < kMinWavesPerSimd && (relax & RELAX_OCCUPANCY_FLOOR)) {
        if (!f.soft_rule[0]) f.soft_rule = "occupancy_floor";
    } else if (o.waves_per_simd < kMinWavesPerSimd)
        return infeasible("occupancy", "only %d wave per SIMD would be resident (%d registers per lane, %d-wave workgroups): too "
                          "few loads in flight to cover HBM latency", o.waves_per_simd, regs, o.waves_per_wg);
    f.dyn_lds = o.lds_bytes - r.lds_static;
    return f;
}

void enumerate(int64_t M, int64_t N, int dtype, std::vector<addrms_cfg>* out, int64_t* n_grid,
               std::map<std::string, int64_t>* pruned, int op, int relax)
{
    int64_t grid = 0;
    struct Quiet { bool was; Quiet() : was(g_rationale_wanted) { g_rationale_wanted = false; } ~Quiet() { g_rationale_wanted = was; } } quiet;
    std::vector<int> tprs = {8, 16, 32};
    for (int t = 64; t <= hw().max_threads_per_wg; t += 64) tprs.push_back(t);
    for (int vec : kVecs)
        for (int tpr : tprs)
            for (int rows : kRows)
                for (int red = 0; red < 2; ++red)
                    for (int unr : kUnrolls)
                        for (int flags = 0; flags < 128; ++flags)
                            for (int cap = 0; cap < hw().max_waves_per_simd; ++cap) {
                                // A longer grid (walk) exists for persistent cfgs only, and whatever rejects the
                                // resident-size grid rejects the longer ones as well (a grid that already covers
                                // every row block still does when it is longer): they are checked one by one only
                                // where walk = 0 is feasible, and counted under the same rule otherwise.
                                const Feas* base = nullptr;
                                Feas f0;
                                for (int walk : kWalks) {
                                    if (walk != 0 && !(flags & ADDRMS_FLAG_PERSISTENT)) continue;   // no such grid point
                                    ++grid;
                                    if (base && base->status != ADDRMS_OK) { if (pruned) ++(*pruned)[base->rule]; continue; }
                                    addrms_cfg c{};
                                    c.vec = vec; c.threads_per_row = tpr; c.rows_per_wg = rows;
                                    c.reduce = red; c.unroll = unr; c.flags = flags; c.max_waves_per_simd = cap;
                                    c.walk = walk;
                                    const Feas f = check_cfg(c, M, N, dtype, op, relax);
                                    if (walk == 0) { f0 = f; base = &f0; }
                                    if (f.status == ADDRMS_OK) { if (out) out->push_back(c); }
                                    else if (pruned) ++(*pruned)[f.rule];
                                }
                            }
    if (n_grid) *n_grid = grid;
}

static bool single_pass_default(int64_t N, int dtype, int op, addrms_cfg* out)
{
    // Preference order: widest vector; 256 threads per row, then wider, then
    // narrower rows; one row per workgroup (more only to fill a wave).
    static const int tprs[] = {256, 512, 1024, 384, 768, 128, 192, 320, 448, 576, 640, 704, 832, 896, 960,
                               64, 32, 16, 8};
    const int64_t big_m = 1 << 20;   // feasibility of the default must not depend on M
    for (int vec : kVecs)
        for (int tpr : tprs) {
            addrms_cfg c{};
            c.vec = vec; c.threads_per_row = tpr;
            c.rows_per_wg = std::max(1, hw().wave_size / tpr);
            c.reduce = ADDRMS_REDUCE_WAVE;
            const int64_t need = (N + static_cast<int64_t>(vec) * tpr - 1) / (static_cast<int64_t>(vec) * tpr);
            c.unroll = need >= 2 ? 2 : 1;
            if (check_cfg(c, big_m, N, dtype, op).status == ADDRMS_OK) { *out = c; return true; }
        }
    return false;
}

int default_cfg(int64_t N, int dtype, addrms_cfg* out, std::string* why, int op)
{
    if (!dtype_valid(dtype, op)) { if (why) *why = "unsupported dtype"; return ADDRMS_ERR_UNSUPPORTED_DTYPE; }
    if (N <= 0) { if (why) *why = "N must be > 0"; return ADDRMS_ERR_INVALID_ARG; }
    const int64_t big_m = 1 << 20;
    if (single_pass_default(N, dtype, op, out)) return ADDRMS_OK;
    if (op == OP_ADDRMS)   // rows somewhat beyond the register cache: one pass, the cache continued in LDS
        for (int vec : kVecs) {
            addrms_cfg c{};
            c.vec = vec; c.threads_per_row = hw().max_threads_per_wg; c.rows_per_wg = 1;
            c.reduce = ADDRMS_REDUCE_WAVE; c.unroll = 2; c.flags = ADDRMS_FLAG_LDS_CACHE;
            if (check_cfg(c, big_m, N, dtype, op).status == ADDRMS_OK) { *out = c; return ADDRMS_OK; }
        }
    if (op == OP_ADDRMS)   // longer still: registers and LDS hold what they can, only the rest of a row is read twice
        for (int vec : kVecs) {
            addrms_cfg c{};
            c.vec = vec; c.threads_per_row = hw().max_threads_per_wg; c.rows_per_wg = 1;
            c.reduce = ADDRMS_REDUCE_WAVE; c.unroll = 2; c.flags = ADDRMS_FLAG_LDS_CACHE | ADDRMS_FLAG_TWO_PASS;
            if (check_cfg(c, big_m, N, dtype, op).status == ADDRMS_OK) { *out = c; return ADDRMS_OK; }
        }
    if (op == OP_ADDRMS)   // (kept for completeness: the plain two-pass form, widest vector, largest workgroup)
        for (int vec : kVecs) {
            addrms_cfg c{};
            c.vec = vec; c.threads_per_row = hw().max_threads_per_wg; c.rows_per_wg = 1;
            c.reduce = ADDRMS_REDUCE_WAVE; c.unroll = 2; c.flags = ADDRMS_FLAG_TWO_PASS;
            if (check_cfg(c, big_m, N, dtype, op).status == ADDRMS_OK) { *out = c; return ADDRMS_OK; }
        }
    if (why) {
        char buf[160];
        snprintf(buf, sizeof buf, "no configuration of the template covers N=%lld for %s (row cache holds %d values "
                 "per thread, %d threads per row at most)", (long long)N, dtype_name(dtype), kMaxElemsPerThread,
                 hw().max_threads_per_wg);
        *why = buf;
    }
    return ADDRMS_ERR_UNSUPPORTED_SHAPE;
}

// ---- the host-only entry points, once for all three operators ------------------------
int export_default_cfg(int op, int64_t N, int dtype, addrms_cfg* out)
{
    if (!out) return fail(ADDRMS_ERR_INVALID_ARG, "out is NULL");
    std::string why;
    const int st = default_cfg(N, dtype, out, &why, op);
    return st == ADDRMS_OK ? st : fail(st, "%s", why.c_str());
}

int export_cfg_feasible(int op, const addrms_cfg* cfg, int64_t M, int64_t N, int dtype, char* reason, size_t reason_len,
                        addrms_resources* res)
{
    if (reason && reason_len) reason[0] = '\0';
    if (!cfg) return fail(ADDRMS_ERR_INVALID_ARG, "cfg is NULL");
    const Feas f = check_cfg(*cfg, M, N, dtype, op);
    if (res) *res = f.res;
    if (f.status != ADDRMS_OK) {
        if (reason && reason_len) snprintf(reason, reason_len, "%s", f.reason.c_str());
        return fail(f.status, "%s", f.reason.c_str());
    }
    return ADDRMS_OK;
}

int64_t export_enumerate_feasible(int op, int64_t M, int64_t N, int dtype, addrms_cfg* out, int64_t cap, int64_t* n_grid)
{
    if (!dtype_valid(dtype, op)) return fail(ADDRMS_ERR_UNSUPPORTED_DTYPE, "unsupported dtype %d for %s", dtype, op_name(op));
    if (M < 0 || N <= 0) return fail(ADDRMS_ERR_INVALID_ARG, "the number of rows must be >= 0 and the row length > 0");
    if (cap < 0 || (cap > 0 && !out)) return fail(ADDRMS_ERR_INVALID_ARG, "out is NULL with cap > 0");
    std::vector<addrms_cfg> v;
    enumerate(M, N, dtype, &v, n_grid, nullptr, op);
    const int64_t n = static_cast<int64_t>(v.size());
    for (int64_t i = 0; i < std::min(n, cap); ++i) out[i] = v[i];
    return n;
}

int export_table_lookup(int op, int64_t M, int64_t N, int dtype, addrms_cfg* out)
{
    if (!out) return fail(ADDRMS_ERR_INVALID_ARG, "out is NULL");
    const int st = table_lookup(M, N, dtype, out, op);
    return st == ADDRMS_OK ? st : fail(st, "no %s table entry usable for %lld rows of %lld, dtype=%d", op_name(op),
                                       (long long)M, (long long)N, dtype);
}

int64_t export_algorithmic_bytes(int op, int64_t M, int64_t N, int dtype)
{
    if (!dtype_valid(dtype, op)) return fail(ADDRMS_ERR_UNSUPPORTED_DTYPE, "unsupported dtype %d for %s", dtype, op_name(op));
    if (M < 0 || N <= 0) return fail(ADDRMS_ERR_INVALID_ARG, "the number of rows must be >= 0 and the row length > 0");
    return algorithmic_bytes(op, M, N, dtype);
}

}  // namespace addrms_host

// ---- C ABI -------------------------------------------------------------------------
using namespace addrms_host;

extern "C" {

const char* addrms_last_error(void) { return last_error(); }
const char* addrms_version(void) { return ADDRMS_VERSION_STRING " (gfx950)"; }

int64_t addrms_algorithmic_bytes(int64_t M, int64_t N, int dtype) { return export_algorithmic_bytes(OP_ADDRMS, M, N, dtype); }

int addrms_get_hw_limits(addrms_hw_limits* out)
{
    if (!out) return fail(ADDRMS_ERR_INVALID_ARG, "out is NULL");
    const HwLimits& L = hw();
    memset(out, 0, sizeof *out);
    out->compute_units = L.compute_units; out->xcds = L.xcds; out->simds_per_cu = L.simds_per_cu;
    out->wave_size = L.wave_size; out->max_waves_per_simd = L.max_waves_per_simd;
    out->regs_per_lane = L.regs_per_lane; out->reg_granule = L.reg_granule;
    out->lds_bytes_per_cu = L.lds_bytes_per_cu; out->lds_granule = L.lds_granule;
    out->max_threads_per_wg = L.max_threads_per_wg; out->max_access_bytes = L.max_access_bytes;
    out->hbm_bytes_per_s = L.hbm_bytes_per_s;
    out->last_level_cache_bytes = L.last_level_cache_bytes; out->l2_bytes_per_xcd = L.l2_bytes_per_xcd;
    return ADDRMS_OK;
}

int addrms_default_cfg(int64_t N, int dtype, addrms_cfg* out) { return export_default_cfg(OP_ADDRMS, N, dtype, out); }

int addrms_cfg_feasible(const addrms_cfg* cfg, int64_t M, int64_t N, int dtype,
                        char* reason, size_t reason_len, addrms_resources* res)
{
    return export_cfg_feasible(OP_ADDRMS, cfg, M, N, dtype, reason, reason_len, res);
}

int64_t addrms_enumerate_feasible(int64_t M, int64_t N, int dtype, addrms_cfg* out, int64_t cap, int64_t* n_grid)
{
    return export_enumerate_feasible(OP_ADDRMS, M, N, dtype, out, cap, n_grid);
}

}  // extern "C"
