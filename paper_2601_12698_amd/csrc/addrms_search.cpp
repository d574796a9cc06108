// Search over the feasible region (Algorithm 1 lines 19-21: for each input x,
// theta*(x) = argmin over Theta_feasible of measured runtime; Section 3.2, Tuning
// agent: candidates are compiled, run and timed, ranked, and the Top-K are
// submitted for re-testing; Testing agent: every candidate passes a correctness
// gate first).
//
// The search only sees a backend with two calls, validate(cfg) and
// measure(cfg, warmup, reps), so the same code runs against the GPU and against
// a synthetic cost function in the CPU tests.
//
// Strategies:
//   exhaustive  the plain definition: time every feasible cfg with the
//               confirmation protocol, then re-test the Top-K;
//   guided      (1) coarse sweep: one representative launch shape per
//               (vec, threads_per_row, form) class, short protocol, in up to four
//               modes (plain, streaming, deferred store, persistent) because those
//               corners are not connected by single-knob moves;
//               (2) descent: from the best few classes, move one knob at a time
//               to the best unmeasured neighbour, trying first the moves that
//               the static signals favour (more resident waves when the kernel
//               is register-limited, more workgroups when the grid underfills
//               the chip); then every occupancy cap and load batching around the best cfg of the
//               three leading classes;
//               (3) Top-K re-test with the confirmation protocol, interleaved
//               so that clock drift hits all candidates alike.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <map>
#include <unordered_map>

#include "addrms_internal.h"

namespace addrms_host {
namespace {

using Clock = std::chrono::steady_clock;
constexpr double kShortKernelUs = 100.0;
constexpr double kScreenTargetUs = 2000.0;
constexpr int kFormBits = ADDRMS_FLAG_TWO_PASS | ADDRMS_FLAG_LDS_CACHE | ADDRMS_FLAG_ALIGNED_SPAN;
constexpr int kLongRowBits = ADDRMS_FLAG_TWO_PASS | ADDRMS_FLAG_LDS_CACHE;

struct Cand {
    addrms_cfg cfg{};
    addrms_resources res{};
    bool tried = false;      // validate and/or measure was attempted
    bool failed = false;     // gate or launch failure: never ranked
    double us = -1.0;        // screening time
    int64_t order = 0;       // 1-based count of measured cfgs when first timed
    double at_ms = 0.0;      // wall time of the first measurement
};

struct Searcher {
    int64_t M, N;
    int dtype;
    addrms_budget b;
    const addrms_backend& be;
    std::vector<Cand> cands;
    std::unordered_map<uint64_t, int> index;
    int64_t n_measured = 0, n_failed = 0;
    int32_t n_resumed = 0;
    std::unordered_map<uint64_t, std::pair<double, bool>> resumed;   // cfg key -> (screening time, passed) from an earlier log
    Clock::time_point t0 = Clock::now();
    FILE* log = nullptr;
    double bytes = 0.0;
    int verbose = 0;

    Searcher(int64_t m, int64_t n, int dt, const addrms_budget& bud, const addrms_backend& backend)
        : M(m), N(n), dtype(dt), b(bud), be(backend) {}

    double elapsed_ms() const { return std::chrono::duration<double, std::milli>(Clock::now() - t0).count(); }
    bool budget_left() const
    {
        if (b.max_candidates > 0 && n_measured >= b.max_candidates) return false;
        if (b.max_wall_ms > 0.0 && elapsed_ms() >= b.max_wall_ms) return false;
        return true;
    }
    int find(const addrms_cfg& c) const
    {
        auto it = index.find(cfg_key(c));
        return it == index.end() ? -1 : it->second;
    }

    void log_eval(const char* phase, const Cand& c, bool pass, double us, int warmup, int reps)
    {
        if (!log) return;
        fprintf(log,
                "{\"event\":\"eval\",\"phase\":\"%s\",\"cfg\":%s,\"pass\":%s,\"us\":%.4f,\"gbps\":%.2f,"
                "\"warmup\":%d,\"reps\":%d,\"signals\":{\"chunks_per_thread\":%d,\"vgprs\":%d,\"agprs\":%d,"
                "\"lds_bytes\":%d,\"waves_per_wg\":%d,\"wgs_per_cu\":%d,\"waves_per_simd\":%d,\"workgroups\":%lld},"
                "\"n_measured\":%lld,\"t_ms\":%.3f}\n",
                phase, cfg_json(c.cfg).c_str(), pass ? "true" : "false", us, us > 0 ? bytes / us * 1e-3 : 0.0,
                warmup, reps, c.res.chunks_per_thread, c.res.vgprs, c.res.agprs, c.res.lds_bytes, c.res.waves_per_wg,
                c.res.wgs_per_cu, c.res.waves_per_simd, (long long)n_workgroups(c.cfg, M, c.res.wgs_per_cu),
                (long long)n_measured, elapsed_ms());
        fflush(log);    // a search that is killed loses at most the line being written
    }

    // Gate + screening measurement of candidate i.  Returns true if it now has a time.
    bool eval(int i, const char* phase, int warmup, int reps)
    {
        Cand& c = cands[i];
        if (c.tried) return !c.failed;
        c.tried = true;
        {   // measured in an earlier run of the same search (same architecture, library, operator, shape): take that
            auto it = resumed.find(cfg_key(c.cfg));
            if (it != resumed.end()) {
                ++n_resumed;
                if (!it->second.second) { c.failed = true; return false; }
                c.us = it->second.first;
                c.order = 0;
                c.at_ms = elapsed_ms();
                return true;
            }
        }
        if (!b.skip_validation && be.validate && be.validate(be.user, &c.cfg) != 0) {
            c.failed = true;
            ++n_failed;
            log_eval(phase, c, false, -1.0, 0, 0);
            return false;
        }
        double us = 0.0;
        if (be.measure(be.user, &c.cfg, warmup, reps, &us) != 0 || !(us > 0.0)) {
            c.failed = true;
            ++n_failed;
            log_eval(phase, c, false, -1.0, warmup, reps);
            return false;
        }
        // Short kernels time noisily with a short protocol and cost next to nothing to time longer: repeat the
        // screening with as many repetitions as fill about two milliseconds (at most eight times as many).
        if (us < kShortKernelUs && reps <= b.coarse_reps) {
            const int more = std::min(reps * 8, std::max(reps, static_cast<int>(kScreenTargetUs / us)));
            double again = 0.0;
            if (more > reps && be.measure(be.user, &c.cfg, warmup, more, &again) == 0 && again > 0.0) us = again;
        }
        ++n_measured;
        c.us = us;
        c.order = n_measured;
        c.at_ms = elapsed_ms();
        log_eval(phase, c, true, us, warmup, reps);
        if (verbose > 1) fprintf(stderr, "[addrms] %-16s %s %.3f us\n", phase, cfg_json(c.cfg).c_str(), us);
        return true;
    }

    std::vector<int> ranked() const
    {
        std::vector<int> v;
        for (int i = 0; i < static_cast<int>(cands.size()); ++i)
            if (cands[i].tried && !cands[i].failed) v.push_back(i);
        std::stable_sort(v.begin(), v.end(), [&](int a, int c) { return cands[a].us < cands[c].us; });
        return v;
    }

    // ---- guided: stage 1 -------------------------------------------------------
    // One representative per (vec, threads_per_row) class and per mode.  The modes are
    // the corners of the space that one-knob moves do not connect well:
    //   plain       default cache policy, workgroup nearest 256 threads, two chunks in flight
    //   streaming   the same launch shape with the non-temporal policy
    //   persistent  non-temporal, persistent grid (XCD-contiguous when available), the
    //               largest workgroup and the deepest load batching the class admits
    //   capped      (only with the lower-occupancy hint) streaming with about half the
    //               resident waves
    //   deferred    streaming with the residual store deferred to the write phase
    enum Mode { kPlain = 0, kStreaming = 1, kPersistent = 2, kCapped = 3, kDeferred = 4 };
    std::vector<int> class_representatives(Mode mode) const
    {
        std::map<std::pair<int, int>, std::pair<double, int>> best;   // class -> (score, index)
        for (int i = 0; i < static_cast<int>(cands.size()); ++i) {
            const addrms_cfg& c = cands[i].cfg;
            if (c.reduce != ADDRMS_REDUCE_WAVE || (c.max_waves_per_simd != 0) != (mode == kCapped)) continue;
            const double threads = static_cast<double>(c.threads_per_row) * c.rows_per_wg;
            double score;
            if (c.walk != 0) continue;                  // walk lengths are reached by descent only
            if (mode == kPersistent) {
                if (!(c.flags & ADDRMS_FLAG_PERSISTENT) || !(c.flags & ADDRMS_FLAG_NONTEMPORAL) ||
                    (c.flags & ADDRMS_FLAG_DEFER_STORE)) continue;
                score = -threads - 0.1 * c.unroll - ((c.flags & ADDRMS_FLAG_XCD_CONTIG) ? 0.01 : 0.0);
            } else {
                // (the long-row form is part of the class, not of the mode)
                const int want_flags = mode == kPlain ? 0
                                       : mode == kDeferred ? (ADDRMS_FLAG_NONTEMPORAL | ADDRMS_FLAG_DEFER_STORE)
                                                           : ADDRMS_FLAG_NONTEMPORAL;
                if ((c.flags & ~kFormBits) != want_flags) continue;
                const int want_unroll = std::min(2, cands[i].res.chunks_per_thread);
                score = fabs(log2(threads / 256.0)) + 0.1 * fabs(log2((double)c.unroll) - log2((double)want_unroll));
                if (mode == kCapped) score += 0.5 * fabs(static_cast<double>(c.max_waves_per_simd) - 4.0);
            }
            // widest vector first; the long-row forms (two-pass, cache continued in LDS, hybrid) are classes of their own
            auto key = std::make_pair(-c.vec - 16 * (c.flags & kFormBits), c.threads_per_row);
            auto it = best.find(key);
            if (it == best.end() || score < it->second.first) best[key] = {score, i};
        }
        std::vector<int> out;
        for (auto& kv : best) out.push_back(kv.second.second);
        return out;
    }

    // ---- guided: stage 2 -------------------------------------------------------
    std::vector<int> neighbours(int i) const
    {
        const addrms_cfg c = cands[i].cfg;
        std::vector<addrms_cfg> raw;
        auto push = [&](addrms_cfg n) { raw.push_back(n); };
        { addrms_cfg n = c; n.rows_per_wg *= 2; push(n); }
        { addrms_cfg n = c; n.rows_per_wg /= 2; if (n.rows_per_wg >= 1) push(n); }
        { addrms_cfg n = c; n.unroll *= 2; push(n); }
        { addrms_cfg n = c; n.unroll /= 2; if (n.unroll >= 1) push(n); }
        { addrms_cfg n = c; n.reduce ^= 1; push(n); }
        { addrms_cfg n = c; n.flags ^= ADDRMS_FLAG_XCD_CONTIG; push(n); }
        { addrms_cfg n = c; n.flags ^= ADDRMS_FLAG_NONTEMPORAL; push(n); }
        { addrms_cfg n = c; n.flags ^= ADDRMS_FLAG_PERSISTENT; n.walk = 0; push(n); }
        { addrms_cfg n = c; n.flags ^= ADDRMS_FLAG_DEFER_STORE; push(n); }
        if (c.flags & ADDRMS_FLAG_PERSISTENT) {        // walk length: one step longer, one step shorter
            { addrms_cfg n = c; n.walk = c.walk == 0 ? 4 : c.walk * 4; push(n); }
            if (c.walk != 0) { addrms_cfg n = c; n.walk = c.walk == 4 ? 0 : c.walk / 4; push(n); }
        }
        if (c.flags & kLongRowBits) {                                // the other long-row forms
            { addrms_cfg n = c; n.flags ^= ADDRMS_FLAG_TWO_PASS; push(n); }
            { addrms_cfg n = c; n.flags ^= ADDRMS_FLAG_LDS_CACHE; push(n); }
            { addrms_cfg n = c; n.flags ^= kLongRowBits; push(n); }
        }
        else { addrms_cfg n = c; n.flags ^= ADDRMS_FLAG_ALIGNED_SPAN; n.reduce = 0; push(n); }   // into or out of the aligned-span form
        // occupancy cap: one step tighter, one step looser (0 = uncapped sits above the natural occupancy)
        {
            const int natural = cands[i].res.waves_per_simd;
            const int cur = c.max_waves_per_simd == 0 ? natural + 1 : c.max_waves_per_simd;
            for (int k = cur - 1; k >= 1; --k) {            // next tighter cap that is feasible
                addrms_cfg n = c; n.max_waves_per_simd = k;
                if (find(n) >= 0) { push(n); break; }
            }
            bool found = false;
            for (int k = cur + 1; k < hw().max_waves_per_simd && !found; ++k) {
                addrms_cfg n = c; n.max_waves_per_simd = k;
                if (find(n) >= 0) { push(n); found = true; }
            }
            if (!found && c.max_waves_per_simd != 0) { addrms_cfg n = c; n.max_waves_per_simd = 0; push(n); }
        }
        // threads_per_row: nearest feasible values above and below at this vec
        int up = 0, down = 0;
        for (const Cand& o : cands) {
            if (o.cfg.vec != c.vec) continue;
            const int t = o.cfg.threads_per_row;
            if (t > c.threads_per_row && (up == 0 || t < up)) up = t;
            if (t < c.threads_per_row && t > down) down = t;
        }
        for (int t : {up, down}) {
            if (t == 0) continue;
            addrms_cfg n = c; n.threads_per_row = t; push(n);
            // keep the workgroup size when the row gets wider or narrower
            n.rows_per_wg = std::max(1, c.rows_per_wg * c.threads_per_row / t); push(n);
        }
        // vec: same threads (more or fewer chunks), or same chunks (threads scaled)
        for (int v : {c.vec * 2, c.vec / 2}) {
            if (v < 1 || v > 8) continue;
            addrms_cfg n = c; n.vec = v; push(n);
            n.threads_per_row = c.threads_per_row * c.vec / v; push(n);
        }
        std::vector<int> out;
        for (addrms_cfg n : raw) {
            int j = find(n);
            if (j < 0) {   // the unroll may no longer fit the new chunk count: clamp down once
                for (int u = n.unroll / 2; u >= 1 && j < 0; u /= 2) { n.unroll = u; j = find(n); }
            }
            if (j >= 0 && j != i && std::find(out.begin(), out.end(), j) == out.end()) out.push_back(j);
        }
        return out;
    }

    // Static signals decide which neighbours are tried first.
    int move_priority(const Cand& from, const Cand& to) const
    {
        int p = 0;
        if (from.res.waves_per_simd < 4 && to.res.waves_per_simd > from.res.waves_per_simd) p += 2;
        const int64_t resident = static_cast<int64_t>(hw().compute_units) * std::max(1, from.res.wgs_per_cu);
        if (n_row_blocks(from.cfg, M) < resident && n_row_blocks(to.cfg, M) > n_row_blocks(from.cfg, M)) p += 2;
        if (to.cfg.vec > from.cfg.vec) p += 1;
        // hints from the previous round's profiler counters
        if ((b.hints & ADDRMS_HINT_LOWER_OCCUPANCY) && to.res.waves_per_simd < from.res.waves_per_simd) p += 3;
        if ((b.hints & ADDRMS_HINT_HIGHER_OCCUPANCY) &&
            (to.res.waves_per_simd > from.res.waves_per_simd || to.cfg.unroll > from.cfg.unroll)) p += 3;
        if ((b.hints & ADDRMS_HINT_FEWER_LARGER_WORKGROUPS) &&
            (n_row_blocks(to.cfg, M) < n_row_blocks(from.cfg, M) ||
             ((to.cfg.flags & ~from.cfg.flags) & ADDRMS_FLAG_PERSISTENT))) p += 3;
        if ((b.hints & ADDRMS_HINT_WIDER_VECTORS) && to.cfg.vec > from.cfg.vec) p += 3;
        return p;
    }

    void descend(int seed, int warmup, int reps)
    {
        int cur = seed;
        for (int step = 0; step < 64 && budget_left(); ++step) {
            std::vector<int> nb = neighbours(cur);
            std::stable_sort(nb.begin(), nb.end(), [&](int a, int c) {
                return move_priority(cands[cur], cands[a]) > move_priority(cands[cur], cands[c]);
            });
            int best = -1;
            for (int j : nb) {
                if (!cands[j].tried) {
                    if (!budget_left()) break;
                    eval(j, "descent", warmup, reps);
                }
                if (cands[j].tried && !cands[j].failed && (best < 0 || cands[j].us < cands[best].us)) best = j;
            }
            if (best < 0 || !(cands[best].us < cands[cur].us * 0.995)) break;
            cur = best;
        }
    }

    // The occupancy cap and the load batching each move a good cfg by about one per cent either way, which is less
    // than a descent step must gain to be taken next to the screening noise, so the descent often leaves them where
    // it happened to start.  Around a leading cfg every combination of the two is cheap to try (a few dozen
    // candidates at most).
    void sweep_fine(int i, int warmup, int reps)
    {
        const addrms_cfg c = cands[i].cfg;
        for (int u = 1; u <= 8; u *= 2)
            for (int k = 0; k < hw().max_waves_per_simd && budget_left(); ++k) {
                addrms_cfg n = c;
                n.unroll = u;
                n.max_waves_per_simd = k;
                const int j = find(n);
                if (j >= 0 && !cands[j].tried) eval(j, "fine", warmup, reps);
            }
    }
};


// ---- resume: what an earlier run already measured ---------------------------------------
// The log is a list of searches, each opened by a "begin" line that names architecture, library
// version, operator, shape and format.  Screening results ("eval" lines other than the
// confirmation re-tests) that follow a matching "begin" are facts about this very search problem
// and need not be measured again; anything else in the file is ignored.
bool json_str(const char* line, const char* key, char* out, size_t cap)
{
    char pat[48];
    snprintf(pat, sizeof pat, "\"%s\":\"", key);
    const char* p = strstr(line, pat);
    if (!p) return false;
    p += strlen(pat);
    size_t n = 0;
    while (*p && *p != '"' && n + 1 < cap) out[n++] = *p++;
    out[n] = '\0';
    return *p == '"';
}
bool json_num(const char* line, const char* key, double* out)
{
    char pat[48];
    snprintf(pat, sizeof pat, "\"%s\":", key);
    const char* p = strstr(line, pat);
    if (!p) return false;
    char* end = nullptr;
    const double v = strtod(p + strlen(pat), &end);
    if (end == p + strlen(pat)) return false;
    *out = v;
    return true;
}
bool version_compatible(const char* a, const char* b)      // same major.minor
{
    int dots = 0;
    for (; *a && *b; ++a, ++b) {
        if (*a != *b) return false;
        if (*a == '.' && ++dots == 2) return true;
    }
    return *a == *b;
}
void load_resume(const char* path, int op, int64_t M, int64_t N, int dtype,
                 std::unordered_map<uint64_t, std::pair<double, bool>>* out)
{
    FILE* f = fopen(path, "r");
    if (!f) return;
    char line[2048];
    bool active = false;
    while (fgets(line, sizeof line, f)) {
        char ev[16] = "";
        if (!json_str(line, "event", ev, sizeof ev)) continue;
        if (!strcmp(ev, "begin")) {
            char s_op[32] = "", s_dt[16] = "", s_arch[16] = "", s_lib[16] = "";
            double m = 0, n = 0;
            active = json_str(line, "op", s_op, sizeof s_op) && json_str(line, "dtype", s_dt, sizeof s_dt) &&
                     json_str(line, "arch", s_arch, sizeof s_arch) && json_str(line, "library", s_lib, sizeof s_lib) &&
                     json_num(line, "M", &m) && json_num(line, "N", &n) && !strcmp(s_op, op_name(op)) &&
                     !strcmp(s_dt, dtype_name(dtype)) && !strcmp(s_arch, "gfx950") &&
                     version_compatible(s_lib, ADDRMS_VERSION_STRING) && static_cast<int64_t>(m) == M &&
                     static_cast<int64_t>(n) == N;
            continue;
        }
        if (!active || strcmp(ev, "eval")) continue;
        {   // a line cut short (the writer was killed) says nothing about its candidate
            const size_t len = strlen(line);
            if (len < 2 || line[len - 1] != '\n' || line[len - 2] != '}') continue;
        }
        char phase[24] = "";
        if (!json_str(line, "phase", phase, sizeof phase) || !strcmp(phase, "confirm")) continue;
        const char* p = strstr(line, "\"cfg\":{");
        addrms_cfg c{};
        if (!p || sscanf(p, "\"cfg\":{\"vec\":%d,\"threads_per_row\":%d,\"rows_per_wg\":%d,\"reduce\":%d,\"unroll\":%d,"
                            "\"flags\":%d,\"max_waves_per_simd\":%d,\"walk\":%d}", &c.vec, &c.threads_per_row, &c.rows_per_wg,
                         &c.reduce, &c.unroll, &c.flags, &c.max_waves_per_simd, &c.walk) != 8) continue;
        double us = 0.0;
        const bool pass = strstr(line, "\"pass\":true") != nullptr;
        if (pass && !(json_num(line, "us", &us) && us > 0.0)) continue;
        (*out)[cfg_key(c)] = {us, pass};
    }
    fclose(f);
}

void fill_defaults(addrms_budget* b)
{
    if (b->top_k <= 0) b->top_k = 5;
    if (b->top_k > ADDRMS_MAX_TOPK) b->top_k = ADDRMS_MAX_TOPK;
    if (b->warmup <= 0) b->warmup = 20;
    if (b->reps <= 0) b->reps = 100;
    if (b->coarse_warmup <= 0) b->coarse_warmup = 3;
    if (b->coarse_reps <= 0) b->coarse_reps = 15;
    if (!(b->eps > 0.0f)) b->eps = 1e-6f;
}

}  // namespace

// Progress on stderr when the environment variable ADDRMS_VERBOSE is set to something other than "0": one line
// when a search starts and one when it ends (2: also one per candidate); the audit reports every 500 candidates.
int verbosity()
{
    static const int v = [] { const char* e = getenv("ADDRMS_VERBOSE"); return (e && *e && strcmp(e, "0") != 0) ? atoi(e) > 1 ? 2 : 1 : 0; }();
    return v;
}

int run_search(int64_t M, int64_t N, int dtype, const addrms_budget* budget, const addrms_backend& be,
               addrms_cfg* out_cfg, addrms_tune_report* report, int op)
{
    if (!out_cfg) return fail(ADDRMS_ERR_INVALID_ARG, "out_cfg is NULL");
    if (!be.measure) return fail(ADDRMS_ERR_INVALID_ARG, "backend has no measure function");
    if (!dtype_valid(dtype, op)) return fail(ADDRMS_ERR_UNSUPPORTED_DTYPE, "unsupported dtype %d for %s", dtype, op_name(op));
    if (M <= 0 || N <= 0) return fail(ADDRMS_ERR_INVALID_ARG, "tuning needs M > 0 and N > 0");
    addrms_budget b{};
    if (budget) b = *budget;
    if (b.strategy != ADDRMS_SEARCH_GUIDED && b.strategy != ADDRMS_SEARCH_EXHAUSTIVE)
        return fail(ADDRMS_ERR_INVALID_ARG, "unknown search strategy %d", b.strategy);
    fill_defaults(&b);

    Searcher s(M, N, dtype, b, be);
    s.bytes = static_cast<double>(algorithmic_bytes(op, M, N, dtype));
    std::vector<addrms_cfg> feasible;
    int64_t n_grid = 0;
    std::map<std::string, int64_t> pruned;   // which rule removed how many grid points
    enumerate(M, N, dtype, &feasible, &n_grid, &pruned, op);
    if (b.family_mask != 0) {   // Level-1 rounds restrict the search to the strategy families enabled so far
        std::vector<addrms_cfg> kept;
        for (const addrms_cfg& c : feasible)
            if (cfg_in_families(c, b.family_mask)) kept.push_back(c);
        pruned["family_not_enabled"] += static_cast<int64_t>(feasible.size() - kept.size());
        feasible.swap(kept);
    }
    addrms_cfg dflt{};
    std::string why;
    const int dst = default_cfg(N, dtype, &dflt, &why, op);
    if (dst != ADDRMS_OK || feasible.empty())
        return fail(ADDRMS_ERR_UNSUPPORTED_SHAPE, "feasible region is empty for M=%lld N=%lld %s: %s", (long long)M,
                    (long long)N, dtype_name(dtype), why.c_str());
    // The default is feasible for any M except that a wave-filling row count may exceed a tiny M; keep it anyway.
    if (check_cfg(dflt, M, N, dtype, op).status != ADDRMS_OK) {
        bool found = false;
        for (const addrms_cfg& c : feasible)
            if (c.vec == dflt.vec && c.threads_per_row == dflt.threads_per_row) { dflt = c; found = true; break; }
        if (!found) dflt = feasible.front();
    }
    s.cands.reserve(feasible.size());
    for (const addrms_cfg& c : feasible) {
        Cand cd;
        cd.cfg = c;
        cd.res = check_cfg(c, M, N, dtype, op).res;
        s.index[cfg_key(c)] = static_cast<int>(s.cands.size());
        s.cands.push_back(cd);
    }
    const int i_default = s.find(dflt);
    s.verbose = verbosity();
    if (s.verbose)
        fprintf(stderr, "[addrms] %s search of %s %lld x %lld %s: %lld feasible of %lld grid points\n",
                b.strategy == ADDRMS_SEARCH_GUIDED ? "guided" : "exhaustive", op_name(op), (long long)M, (long long)N,
                dtype_name(dtype), (long long)feasible.size(), (long long)n_grid);

    if (b.log_path) {
        if (!b.no_resume) load_resume(b.log_path, op, M, N, dtype, &s.resumed);
        s.log = fopen(b.log_path, "a");
        if (!s.log) return fail(ADDRMS_ERR_IO, "cannot open log %s", b.log_path);
        fprintf(s.log, "{\"event\":\"begin\",\"arch\":\"gfx950\",\"library\":\"" ADDRMS_VERSION_STRING "\",\"op\":\"%s\",\"M\":%lld,"
                       "\"N\":%lld,\"dtype\":\"%s\",\"strategy\":\"%s\",\"n_grid\":%lld,"
                       "\"n_feasible\":%lld,\"default\":%s,\"pruned\":{",
                op_name(op), (long long)M, (long long)N, dtype_name(dtype),
                b.strategy == ADDRMS_SEARCH_GUIDED ? "guided" : "exhaustive",
                (long long)n_grid, (long long)feasible.size(), cfg_json(dflt).c_str());
        bool first = true;
        for (auto& kv : pruned) { fprintf(s.log, "%s\"%s\":%lld", first ? "" : ",", kv.first.c_str(), (long long)kv.second); first = false; }
        fprintf(s.log, "}}\n");
    }

    // ---- screening ---------------------------------------------------------------
    if (b.strategy == ADDRMS_SEARCH_EXHAUSTIVE) {
        if (i_default >= 0) s.eval(i_default, "default", b.warmup, b.reps);
        for (int i = 0; i < static_cast<int>(s.cands.size()) && s.budget_left(); ++i)
            s.eval(i, "exhaustive", b.warmup, b.reps);
    } else {
        if (i_default >= 0) s.eval(i_default, "default", b.coarse_warmup, b.coarse_reps);
        // plain mode for every class; the other modes only for classes within a factor two of the best plain time
        std::map<std::pair<int, int>, double> plain_us;
        double best_plain = 0.0;
        for (int i : s.class_representatives(Searcher::kPlain)) {
            if (!s.budget_left()) break;
            if (s.eval(i, "sweep", b.coarse_warmup, b.coarse_reps)) {
                const addrms_cfg& c = s.cands[i].cfg;
                plain_us[{c.vec + 16 * (c.flags & kFormBits), c.threads_per_row}] = s.cands[i].us;
                if (best_plain == 0.0 || s.cands[i].us < best_plain) best_plain = s.cands[i].us;
            }
        }
        std::vector<Searcher::Mode> modes = {Searcher::kStreaming, Searcher::kDeferred, Searcher::kPersistent};
        if (b.hints & ADDRMS_HINT_LOWER_OCCUPANCY) modes.push_back(Searcher::kCapped);
        for (Searcher::Mode mode : modes)
            for (int i : s.class_representatives(mode)) {
                if (!s.budget_left()) break;
                const addrms_cfg& c = s.cands[i].cfg;
                auto it = plain_us.find({c.vec + 16 * (c.flags & kFormBits), c.threads_per_row});
                if (it != plain_us.end() && it->second > 2.0 * best_plain) continue;
                s.eval(i, mode == Searcher::kStreaming ? "sweep_streaming"
                          : mode == Searcher::kDeferred ? "sweep_deferred"
                          : mode == Searcher::kPersistent ? "sweep_persistent" : "sweep_capped",
                       b.coarse_warmup, b.coarse_reps);
            }
        std::vector<int> seeds = s.ranked();
        // descend from the best three distinct (vec, threads_per_row, persistent) corners
        std::vector<int> starts;
        for (int i : seeds) {
            bool dup = false;
            for (int j : starts)
                dup = dup || (s.cands[j].cfg.vec == s.cands[i].cfg.vec &&
                              s.cands[j].cfg.threads_per_row == s.cands[i].cfg.threads_per_row &&
                              ((s.cands[j].cfg.flags ^ s.cands[i].cfg.flags) & (ADDRMS_FLAG_PERSISTENT | kFormBits)) == 0);
            if (!dup) starts.push_back(i);
            if (starts.size() == 3) break;
        }
        for (int i : starts) s.descend(i, b.coarse_warmup, b.coarse_reps);
        // ... around the best cfg of each of the three leading (vec, threads_per_row, form) classes
        std::vector<int> lead;
        for (int i : s.ranked()) {
            bool dup = false;
            for (int j : lead)
                dup = dup || (s.cands[j].cfg.vec == s.cands[i].cfg.vec &&
                              s.cands[j].cfg.threads_per_row == s.cands[i].cfg.threads_per_row &&
                              ((s.cands[j].cfg.flags ^ s.cands[i].cfg.flags) & kFormBits) == 0);
            if (!dup) lead.push_back(i);
            if (lead.size() == 3) break;
        }
        for (int i : lead) s.sweep_fine(i, b.coarse_warmup, b.coarse_reps);
    }

    std::vector<int> order = s.ranked();
    if (order.empty()) {
        if (s.log) { fprintf(s.log, "{\"event\":\"end\",\"status\":\"no_result\"}\n"); fclose(s.log); }
        return fail(ADDRMS_ERR_NO_RESULT, "no candidate could be measured within the budget (%lld failed)",
                    (long long)s.n_failed);
    }

    // ---- Top-K confirmation re-test ----------------------------------------------
    std::vector<int> top(order.begin(), order.begin() + std::min<size_t>(order.size(), b.top_k));
    bool default_in_top = std::find(top.begin(), top.end(), i_default) != top.end();
    std::vector<int> confirm = top;
    if (i_default >= 0 && !default_in_top && s.cands[i_default].tried && !s.cands[i_default].failed)
        confirm.push_back(i_default);
    std::vector<double> sum(confirm.size(), 0.0);
    std::vector<int> cnt(confirm.size(), 0);
    const int rounds = 2;
    for (int r = 0; r < rounds; ++r)
        for (size_t k = 0; k < confirm.size(); ++k) {
            double us = 0.0;
            if (be.measure(be.user, &s.cands[confirm[k]].cfg, b.warmup, b.reps, &us) == 0 && us > 0.0) {
                sum[k] += us;
                ++cnt[k];
                s.log_eval("confirm", s.cands[confirm[k]], true, us, b.warmup, b.reps);
            }
        }
    std::vector<std::pair<double, int>> confirmed;   // (mean us, cand index)
    double default_us = -1.0;
    for (size_t k = 0; k < confirm.size(); ++k) {
        if (cnt[k] == 0) continue;
        const double mean = sum[k] / cnt[k];
        if (confirm[k] == i_default) default_us = mean;
        confirmed.push_back({mean, confirm[k]});      // the default competes too: the winner is the argmin of what was confirmed
    }
    if (confirmed.empty()) {
        if (s.log) { fprintf(s.log, "{\"event\":\"end\",\"status\":\"no_result\"}\n"); fclose(s.log); }
        return fail(ADDRMS_ERR_NO_RESULT, "confirmation re-test failed for every Top-K candidate");
    }
    std::stable_sort(confirmed.begin(), confirmed.end());
    const Cand& win = s.cands[confirmed.front().second];
    *out_cfg = win.cfg;

    if (report) {
        memset(report, 0, sizeof *report);
        report->n_grid = n_grid;
        report->n_feasible = static_cast<int64_t>(feasible.size());
        report->n_measured = s.n_measured;
        report->n_failed = s.n_failed;
        report->best_found_at = win.order;
        report->best_us = confirmed.front().first;
        report->default_us = default_us;
        report->time_to_best_ms = win.at_ms;
        report->best = win.cfg;
        report->default_cfg = dflt;
        report->n_topk = static_cast<int32_t>(std::min<size_t>(confirmed.size(), ADDRMS_MAX_TOPK));
        report->n_resumed = s.n_resumed;
        for (size_t k = 0; k < static_cast<size_t>(report->n_topk); ++k) {
            report->topk[k] = s.cands[confirmed[k].second].cfg;
            report->topk_us[k] = confirmed[k].first;
        }
        report->wall_ms = s.elapsed_ms();
    }
    if (s.verbose)
        fprintf(stderr, "[addrms] best %s %.3f us (default %.3f us) after %lld candidates (%d taken from the log, %lld failed) "
                        "in %.0f ms\n", cfg_json(win.cfg).c_str(), confirmed.front().first, default_us, (long long)s.n_measured,
                s.n_resumed, (long long)s.n_failed, s.elapsed_ms());
    if (s.log) {
        fprintf(s.log, "{\"event\":\"end\",\"status\":\"ok\",\"best\":%s,\"best_us\":%.4f,\"default_us\":%.4f,"
                       "\"n_measured\":%lld,\"n_resumed\":%d,\"n_failed\":%lld,\"best_found_at\":%lld,\"time_to_best_ms\":%.3f,"
                       "\"wall_ms\":%.3f}\n",
                cfg_json(win.cfg).c_str(), confirmed.front().first, default_us, (long long)s.n_measured, s.n_resumed,
                (long long)s.n_failed, (long long)win.order, win.at_ms, s.elapsed_ms());
        fclose(s.log);
    }
    return ADDRMS_OK;
}

}  // namespace addrms_host

extern "C" int addrms_tune_with_backend(int64_t M, int64_t N, int dtype, const addrms_budget* budget,
                                        const addrms_backend* backend, addrms_cfg* out_cfg,
                                        addrms_tune_report* report)
{
    if (!backend) return addrms_host::fail(ADDRMS_ERR_INVALID_ARG, "backend is NULL");
    return addrms_host::run_search(M, N, dtype, budget, *backend, out_cfg, report);
}
