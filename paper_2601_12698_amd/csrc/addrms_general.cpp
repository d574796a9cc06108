// General configuration (Algorithm 1 line 22, SelectGeneral; Section 4, "Performance
// Measurement": besides the best specialised cfg per shape, report the one general
// cfg with the best average performance across shapes).  The aggregate is the
// geometric-mean speed-up of Section 3.1, taken against each shape's default cfg.
//
// Host-only: measurement comes through a backend factory, one backend per shape.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <unordered_set>

#include "addrms_internal.h"

namespace addrms_host {
namespace {

double knob_distance(const addrms_cfg& a, const addrms_cfg& b)
{
    auto l2 = [](int v) { return log2(static_cast<double>(std::max(1, v))); };
    return fabs(l2(a.vec) - l2(b.vec)) * 2.0 + fabs(l2(a.threads_per_row) - l2(b.threads_per_row)) +
           fabs(l2(a.rows_per_wg) - l2(b.rows_per_wg)) + fabs(l2(a.unroll) - l2(b.unroll)) * 0.5 +
           (a.reduce != b.reduce ? 1.0 : 0.0) + __builtin_popcount(static_cast<unsigned>(a.flags ^ b.flags)) +
           0.25 * abs(a.max_waves_per_simd - b.max_waves_per_simd);
}

bool feasible_everywhere(const addrms_cfg& c, const addrms_shape* shapes, int n, int dtype, int op)
{
    for (int i = 0; i < n; ++i)
        if (check_cfg(c, shapes[i].M, shapes[i].N, dtype, op).status != ADDRMS_OK) return false;
    return true;
}

struct OpenBackend {
    const addrms_backend_factory& f;
    addrms_backend be{};
    bool open = false;
    explicit OpenBackend(const addrms_backend_factory& fac) : f(fac) {}
    int start(int64_t M, int64_t N, int dtype)
    {
        const int st = f.open(f.user, M, N, dtype, &be);
        open = st == 0;
        return st;
    }
    ~OpenBackend() { if (open && f.close) f.close(f.user, &be); }
};

}  // namespace

int run_select_general(const addrms_shape* shapes, int n, int dtype, const addrms_budget* budget,
                       const addrms_backend_factory& factory, bool insert_in_table,
                       addrms_cfg* out_general, addrms_general_report* report, int op)
{
    using Clock = std::chrono::steady_clock;
    const auto t0 = Clock::now();
    if (!shapes || !out_general) return fail(ADDRMS_ERR_INVALID_ARG, "shapes and out_general must not be NULL");
    if (n < 1 || n > ADDRMS_MAX_SHAPES) return fail(ADDRMS_ERR_INVALID_ARG, "n must be 1..%d", ADDRMS_MAX_SHAPES);
    if (!factory.open) return fail(ADDRMS_ERR_INVALID_ARG, "backend factory has no open function");
    if (!dtype_valid(dtype, op)) return fail(ADDRMS_ERR_UNSUPPORTED_DTYPE, "unsupported dtype %d for %s", dtype, op_name(op));
    for (int i = 0; i < n; ++i)
        if (shapes[i].M <= 0 || shapes[i].N <= 0) return fail(ADDRMS_ERR_INVALID_ARG, "shape %d needs M > 0 and N > 0", i);
    addrms_budget b{};
    if (budget) b = *budget;
    const int warmup = b.warmup > 0 ? b.warmup : 20, reps = b.reps > 0 ? b.reps : 100;

    // ---- per-shape search (lines 19-21), specialised table (line 23)
    addrms_general_report rep{};
    rep.n_shapes = n;
    std::vector<addrms_cfg> pool;
    std::unordered_set<uint64_t> seen;
    auto add = [&](const addrms_cfg& c) { if (seen.insert(cfg_key(c)).second) pool.push_back(c); };
    std::vector<addrms_cfg> defaults(n);
    for (int i = 0; i < n; ++i) {
        OpenBackend ob(factory);
        if (ob.start(shapes[i].M, shapes[i].N, dtype) != 0)
            return fail(ADDRMS_ERR_HIP, "could not open a measurement backend for shape %d (%lld x %lld)", i,
                        (long long)shapes[i].M, (long long)shapes[i].N);
        addrms_cfg best{};
        addrms_tune_report tr{};
        const int st = run_search(shapes[i].M, shapes[i].N, dtype, budget, ob.be, &best, &tr, op);
        if (st != ADDRMS_OK) return st;
        rep.specialized[i] = best;
        rep.specialized_us[i] = tr.best_us;
        rep.default_us[i] = tr.default_us;
        defaults[i] = tr.default_cfg;
        for (int k = 0; k < tr.n_topk; ++k) add(tr.topk[k]);
        add(tr.default_cfg);
    }

    // ---- candidates that are one theta for every shape
    std::vector<addrms_cfg> cands;
    for (const addrms_cfg& c : pool)
        if (feasible_everywhere(c, shapes, n, dtype, op)) cands.push_back(c);
    {
        // widen: the universally feasible cfgs nearest (in knob steps) to each shape's winner, so that a
        // compromise lying between the specialised winners is in the pool even if no winner fits every shape
        std::vector<addrms_cfg> all;
        enumerate(shapes[0].M, shapes[0].N, dtype, &all, nullptr, nullptr, op);
        std::vector<addrms_cfg> common;
        for (const addrms_cfg& c : all)
            if (feasible_everywhere(c, shapes, n, dtype, op)) common.push_back(c);
        if (common.empty() && cands.empty())
            return fail(ADDRMS_ERR_NO_RESULT, "no configuration is feasible on all %d shapes", n);
        std::unordered_set<uint64_t> have;
        for (const addrms_cfg& c : cands) have.insert(cfg_key(c));
        for (int i = 0; i < n; ++i) {
            std::vector<std::pair<double, int>> near;
            for (int j = 0; j < static_cast<int>(common.size()); ++j)
                near.push_back({knob_distance(common[j], rep.specialized[i]), j});
            std::stable_sort(near.begin(), near.end());
            for (int k = 0; k < std::min<int>(3, near.size()); ++k)
                if (have.insert(cfg_key(common[near[k].second])).second) cands.push_back(common[near[k].second]);
        }
    }
    rep.n_pool = static_cast<int32_t>(cands.size());

    // ---- time every candidate on every shape; defaults again with the same protocol.  Three rounds, the default
    // and every candidate once per round, each cfg keeping its fastest round: on launch-bound shapes one batch of a
    // 3 us kernel scatters by several per cent, and a default timed once beside candidates timed once made the
    // same cfg come out 8 % apart from itself.
    constexpr int kRounds = 3;
    std::vector<std::vector<double>> us(cands.size(), std::vector<double>(n, -1.0));
    for (int i = 0; i < n; ++i) {
        OpenBackend ob(factory);
        if (ob.start(shapes[i].M, shapes[i].N, dtype) != 0)
            return fail(ADDRMS_ERR_HIP, "could not open a measurement backend for shape %d", i);
        std::vector<char> usable(cands.size(), 1);
        double dbest = -1.0;
        for (int round = 0; round < kRounds; ++round) {
            double d = 0.0;
            if (ob.be.measure(ob.be.user, &defaults[i], warmup, reps, &d) == 0 && d > 0.0 && (dbest < 0.0 || d < dbest)) dbest = d;
            for (size_t k = 0; k < cands.size(); ++k) {
                if (!usable[k]) continue;
                if (round == 0 && !b.skip_validation && ob.be.validate && ob.be.validate(ob.be.user, &cands[k]) != 0) {
                    usable[k] = 0;
                    continue;
                }
                double t = 0.0;
                if (ob.be.measure(ob.be.user, &cands[k], warmup, reps, &t) == 0 && t > 0.0) {
                    if (us[k][i] < 0.0 || t < us[k][i]) us[k][i] = t;
                } else {
                    usable[k] = 0;
                    us[k][i] = -1.0;
                }
            }
        }
        if (dbest > 0.0) rep.default_us[i] = dbest;
    }
    int win = -1;
    double win_score = 0.0;
    for (size_t k = 0; k < cands.size(); ++k) {
        double logsum = 0.0;
        bool ok = true;
        for (int i = 0; i < n && ok; ++i) {
            ok = us[k][i] > 0.0 && rep.default_us[i] > 0.0;
            if (ok) logsum += log(rep.default_us[i] / us[k][i]);
        }
        if (!ok) continue;
        const double score = exp(logsum / n);
        if (win < 0 || score > win_score) { win = static_cast<int>(k); win_score = score; }
    }
    if (win < 0) return fail(ADDRMS_ERR_NO_RESULT, "no candidate could be measured on all %d shapes", n);
    *out_general = cands[win];
    rep.geomean_speedup_general = win_score;
    double logspec = 0.0, mean = 0.0;
    for (int i = 0; i < n; ++i) {
        rep.general_us[i] = us[win][i];
        // a shape's specialised time can never be reported worse than the general cfg measured on it
        if (rep.specialized_us[i] <= 0.0 || us[win][i] < rep.specialized_us[i]) {
            rep.specialized_us[i] = us[win][i];
            rep.specialized[i] = cands[win];
        }
        logspec += log(rep.default_us[i] / rep.specialized_us[i]);
        mean += rep.default_us[i] / us[win][i];
        // the table gets what the report calls specialised (line 23), after the replacement above
        if (insert_in_table) table_insert(shapes[i].M, shapes[i].N, dtype, rep.specialized[i], rep.specialized_us[i], op);
    }
    rep.geomean_speedup_specialized = exp(logspec / n);
    rep.mean_speedup_general = mean / n;
    rep.wall_ms = std::chrono::duration<double, std::milli>(Clock::now() - t0).count();
    if (report) *report = rep;
    return ADDRMS_OK;
}

// ---- the outer loop with a fixed strategy list ------------------------------------
int run_tune_rounds(const addrms_shape* shapes, int n, int dtype, const addrms_budget* budget,
                    const addrms_backend_factory& factory, bool insert_in_table,
                    addrms_cfg* out_general, addrms_rounds_report* report, int op)
{
    using Clock = std::chrono::steady_clock;
    const auto t0 = Clock::now();
    if (!shapes || !out_general) return fail(ADDRMS_ERR_INVALID_ARG, "shapes and out_general must not be NULL");
    if (n < 1 || n > ADDRMS_MAX_SHAPES) return fail(ADDRMS_ERR_INVALID_ARG, "n must be 1..%d", ADDRMS_MAX_SHAPES);
    if (!factory.open) return fail(ADDRMS_ERR_INVALID_ARG, "backend factory has no open function");
    if (!dtype_valid(dtype, op)) return fail(ADDRMS_ERR_UNSUPPORTED_DTYPE, "unsupported dtype %d for %s", dtype, op_name(op));
    addrms_budget b{};
    if (budget) b = *budget;
    static const int kOrder[ADDRMS_MAX_ROUNDS] = {0, ADDRMS_FAMILY_STREAMING, ADDRMS_FAMILY_OCCUPANCY_CAP,
                                                  ADDRMS_FAMILY_GRID_MAPPING, ADDRMS_FAMILY_STORE_PHASE};
    addrms_rounds_report rep{};
    rep.best_round = -1;
    double best_score = 0.0;
    int enabled = 0;
    for (int r = 0; r < ADDRMS_MAX_ROUNDS; ++r) {
        addrms_round_info& info = rep.rounds[r];
        info.pass = 1;
        if (kOrder[r] != 0) {
            // Validate the rewritten kernel (the family just added) on the first shape: the cheapest
            // feasible cfg that uses it must reproduce the reference output; otherwise roll back.
            std::vector<addrms_cfg> all;
            enumerate(shapes[0].M, shapes[0].N, dtype, &all, nullptr, nullptr, op);
            const addrms_cfg* probe = nullptr;
            for (const addrms_cfg& c : all)
                if (cfg_in_families(c, enabled | kOrder[r]) && !cfg_in_families(c, enabled ? enabled : ADDRMS_FAMILY_BASE_ONLY)) {
                    probe = &c;
                    break;
                }
            if (probe) {
                OpenBackend ob(factory);
                if (ob.start(shapes[0].M, shapes[0].N, dtype) != 0)
                    return fail(ADDRMS_ERR_HIP, "could not open a measurement backend for validation");
                if (ob.be.validate && ob.be.validate(ob.be.user, probe) != 0) info.pass = 0;
            } else {
                info.pass = 0;      // the family has no feasible member on this shape: nothing to add
            }
            if (info.pass) enabled |= kOrder[r];
        }
        info.families = enabled;
        addrms_budget rb = b;
        rb.family_mask = enabled ? enabled : ADDRMS_FAMILY_BASE_ONLY;
        addrms_cfg general{};
        addrms_general_report gr{};
        int st = ADDRMS_OK;
        if (r == 0 || info.pass) {
            st = run_select_general(shapes, n, dtype, &rb, factory, false, &general, &gr, op);
            if (st != ADDRMS_OK) return st;
            info.general = general;
            info.geomean_speedup_general = gr.geomean_speedup_general;
            info.score = -gr.geomean_speedup_specialized;
            if (rep.best_round < 0 || info.score < best_score) {
                rep.best_round = r;
                best_score = info.score;
                rep.best = gr;
                *out_general = general;
            }
        } else {            // rolled back: this round is the previous round again
            info.general = rep.rounds[r - 1].general;
            info.geomean_speedup_general = rep.rounds[r - 1].geomean_speedup_general;
            info.score = rep.rounds[r - 1].score;
        }
        rep.n_rounds = r + 1;
        if (b.log_path) {
            if (FILE* f = fopen(b.log_path, "a")) {
                fprintf(f, "{\"event\":\"round\",\"round\":%d,\"families\":%d,\"pass\":%s,\"general\":%s,"
                           "\"geomean_speedup_general\":%.5f,\"score\":%.5f,\"incumbent\":%d}\n",
                        r, info.families, info.pass ? "true" : "false", cfg_json(info.general).c_str(),
                        info.geomean_speedup_general, info.score, rep.best_round);
                fclose(f);
            }
        }
    }
    if (insert_in_table)
        for (int i = 0; i < n; ++i)
            table_insert(shapes[i].M, shapes[i].N, dtype, rep.best.specialized[i], rep.best.specialized_us[i], op);
    rep.wall_ms = std::chrono::duration<double, std::milli>(Clock::now() - t0).count();
    if (report) *report = rep;
    return ADDRMS_OK;
}

}  // namespace addrms_host

extern "C" int addrms_tune_rounds_with_backend(const addrms_shape* shapes, int32_t n, int dtype,
                                               const addrms_budget* budget, const addrms_backend_factory* factory,
                                               addrms_cfg* out_general, addrms_rounds_report* report)
{
    if (!factory) return addrms_host::fail(ADDRMS_ERR_INVALID_ARG, "factory is NULL");
    return addrms_host::run_tune_rounds(shapes, n, dtype, budget, *factory, false, out_general, report);
}

extern "C" int addrms_select_general_with_backend(const addrms_shape* shapes, int32_t n, int dtype,
                                                  const addrms_budget* budget, const addrms_backend_factory* factory,
                                                  addrms_cfg* out_general, addrms_general_report* report)
{
    if (!factory) return addrms_host::fail(ADDRMS_ERR_INVALID_ARG, "factory is NULL");
    return addrms_host::run_select_general(shapes, n, dtype, budget, *factory, false, out_general, report);
}
