// Audit of the deriver's efficiency rules (Section 3.3: the feasible region excludes
// "obviously inefficient" configurations as well as invalid ones).  Validity rules
// cannot be questioned by measurement - an invalid launch has no time - but an
// efficiency rule can: switch it off, run what it would have pruned through the same
// gate and the same timing protocol as the retained configurations, and compare.  A
// rule is sound if nothing it prunes beats the best retained configuration.
//
// Host-only: validation and timing come through a backend.
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <string>
#include <vector>

#include "addrms_internal.h"

namespace addrms_host {

int run_audit_rules(int64_t M, int64_t N, int dtype, const addrms_budget* budget, const addrms_backend& be,
                    addrms_audit_report* report)
{
    using Clock = std::chrono::steady_clock;
    const auto t0 = Clock::now();
    auto elapsed_ms = [&] { return std::chrono::duration<double, std::milli>(Clock::now() - t0).count(); };
    if (!report) return fail(ADDRMS_ERR_INVALID_ARG, "report is NULL");
    if (!dtype_valid(dtype)) return fail(ADDRMS_ERR_UNSUPPORTED_DTYPE, "unsupported dtype %d", dtype);
    if (M <= 0 || N <= 0) return fail(ADDRMS_ERR_INVALID_ARG, "the audit needs M > 0 and N > 0");
    if (!be.measure) return fail(ADDRMS_ERR_INVALID_ARG, "backend has no measure function");
    const int warm = budget && budget->coarse_warmup > 0 ? budget->coarse_warmup : 3;
    const int reps = budget && budget->coarse_reps > 0 ? budget->coarse_reps : 15;
    const int per_class = budget && budget->max_candidates > 0 ? budget->max_candidates : 0;   // pruned classes; 0 = all
    const double wall_cap = budget ? budget->max_wall_ms : 0.0;
    const bool gate = !(budget && budget->skip_validation) && be.validate;

    memset(report, 0, sizeof *report);
    static const char* kRules[ADDRMS_AUDIT_RULES] = {"lane_utilisation", "occupancy_floor", "scratch", "two_pass_needless",
                                                      "lds_cache_needless", "span_needless"};
    for (int r = 0; r < ADDRMS_AUDIT_RULES; ++r) snprintf(report->rules[r].rule, sizeof report->rules[r].rule, "%s", kRules[r]);

    // class 0 = retained by every rule; class 1 + r = let through only because rule r was switched off
    std::vector<addrms_cfg> all;
    enumerate(M, N, dtype, &all, nullptr, nullptr, OP_ADDRMS, RELAX_ALL);
    std::vector<std::vector<addrms_cfg>> cls(1 + ADDRMS_AUDIT_RULES);
    for (const addrms_cfg& c : all) {
        const Feas f = check_cfg(c, M, N, dtype, OP_ADDRMS, RELAX_ALL);
        int k = 0;
        for (int r = 0; r < ADDRMS_AUDIT_RULES; ++r)
            if (!strcmp(f.soft_rule, kRules[r])) k = 1 + r;
        cls[k].push_back(c);
    }
    report->n_retained = static_cast<int64_t>(cls[0].size());
    if (cls[0].empty()) return fail(ADDRMS_ERR_UNSUPPORTED_SHAPE, "feasible region is empty");

    bool out_of_time = false;
    const int verbose = verbosity();
    int64_t n_done = 0;
    auto run_class = [&](const std::vector<addrms_cfg>& v, bool sample, std::vector<double>* times, addrms_cfg* best_cfg,
                         int32_t* n_failed) {
        const size_t stride = (sample && per_class > 0) ? std::max<size_t>(1, (v.size() + per_class - 1) / per_class) : 1;
        double best = 0.0;
        for (size_t i = 0; i < v.size(); i += stride) {
            if (wall_cap > 0.0 && elapsed_ms() >= wall_cap) { out_of_time = true; break; }
            if (verbose && ++n_done % 500 == 0)
                fprintf(stderr, "[addrms] audit of %lld x %lld %s: %lld candidates after %.0f ms\n", (long long)M, (long long)N,
                        dtype_name(dtype), (long long)n_done, elapsed_ms());
            if (gate && be.validate(be.user, &v[i]) != 0) { ++*n_failed; continue; }
            double us = 0.0;
            if (be.measure(be.user, &v[i], warm, reps, &us) != 0 || !(us > 0.0)) { ++*n_failed; continue; }
            times->push_back(us);
            if (best == 0.0 || us < best) { best = us; *best_cfg = v[i]; }
        }
        return best;
    };

    std::vector<double> t_ret;
    int32_t failed_ret = 0;
    report->retained_best_us = run_class(cls[0], false, &t_ret, &report->retained_best, &failed_ret);
    report->n_retained_measured = static_cast<int32_t>(t_ret.size());
    report->n_retained_failed = failed_ret;
    if (t_ret.empty()) return fail(ADDRMS_ERR_NO_RESULT, "no retained configuration could be measured");
    std::sort(t_ret.begin(), t_ret.end());
    report->retained_decile_us = t_ret[t_ret.size() / 10];
    report->retained_median_us = t_ret[t_ret.size() / 2];

    for (int r = 0; r < ADDRMS_AUDIT_RULES; ++r) {
        addrms_audit_rule& o = report->rules[r];
        o.n_pruned = static_cast<int64_t>(cls[1 + r].size());
        std::vector<double> t;
        o.best_us = run_class(cls[1 + r], true, &t, &o.best, &o.n_failed);
        o.n_measured = static_cast<int32_t>(t.size());
        for (double us : t) {
            if (us < report->retained_decile_us) ++o.n_in_top_decile;
            if (us < report->retained_best_us) ++o.n_beating_best;
        }
        if (!t.empty()) {
            std::sort(t.begin(), t.end());
            o.median_us = t[t.size() / 2];
        }
    }
    report->truncated = out_of_time ? 1 : 0;
    report->wall_ms = elapsed_ms();
    return ADDRMS_OK;
}

}  // namespace addrms_host

extern "C" int addrms_audit_rules_with_backend(int64_t M, int64_t N, int dtype, const addrms_budget* budget,
                                               const addrms_backend* backend, addrms_audit_report* report)
{
    if (!backend) return addrms_host::fail(ADDRMS_ERR_INVALID_ARG, "backend is NULL");
    return addrms_host::run_audit_rules(M, N, dtype, budget, *backend, report);
}
