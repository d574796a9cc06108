// Exercises the host-only part of the library (deriver, table, search, general selection, outer loop,
// rule audit) through its C entry points, with synthetic measurement backends.  Built with the address and
// undefined-behaviour sanitizers by tests/test_host_sanitizers.py; any report makes the run fail.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <string>
#include <vector>

#include "addrms.h"

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "CHECK failed at line %d: %s (last error: %s)\n", __LINE__, #cond, addrms_last_error()); exit(1); } } while (0)

static int g_calls = 0;
static double cost(const addrms_cfg* c)
{
    double us = 20.0;
    us *= 1.0 + 0.3 * fabs(log2(c->threads_per_row / 512.0));
    us *= 1.0 + 0.25 * fabs(log2(c->vec / 8.0));
    us *= 1.0 + 0.05 * fabs(log2(c->rows_per_wg / 2.0));
    us *= c->reduce ? 1.1 : 1.0;
    us *= (c->flags & ADDRMS_FLAG_NONTEMPORAL) ? 0.85 : 1.0;
    us *= (c->flags & ADDRMS_FLAG_TWO_PASS) ? 1.5 : (c->flags & ADDRMS_FLAG_LDS_CACHE) ? 1.1 : 1.0;
    return us;
}
static int measure(void*, const addrms_cfg* c, int, int, double* us)
{
    ++g_calls;
    if (c->unroll == 8 && c->rows_per_wg == 4) return 1;          // a candidate that fails to launch
    *us = cost(c);
    return 0;
}
static int validate(void*, const addrms_cfg* c) { return (c->vec == 2 && c->reduce == 1) ? 1 : 0; }   // a wrong result
static int open_be(void*, int64_t, int64_t, int, addrms_backend* out) { out->user = nullptr; out->measure = measure; out->validate = validate; return 0; }
static void close_be(void*, addrms_backend*) {}

int main(int argc, char** argv)
{
    const char* tmp = argc > 1 ? argv[1] : "/tmp";
    // ---- deriver
    const int dts[] = {ADDRMS_BF16, ADDRMS_FP16, ADDRMS_FP16_RES32, ADDRMS_FP32};
    const int64_t ns[] = {8, 24, 1000, 1001, 4096, 7168, 11008, 20001, 32768, 32770, 65536, 100001, 1 << 20, (1ll << 28) + 8};
    for (int dt : dts)
        for (int64_t n : ns) {
            addrms_cfg c{};
            const int st = addrms_default_cfg(n, dt, &c);
            if (st == ADDRMS_OK) {
                char why[8];                                       // deliberately tiny: the text must be truncated safely
                addrms_resources res{};
                CHECK(addrms_cfg_feasible(&c, 64, n, dt, why, sizeof why, &res) == ADDRMS_OK);
                CHECK(addrms_cfg_feasible(&c, 64, n, dt, nullptr, 0, nullptr) == ADDRMS_OK);
            } else {
                CHECK(st == ADDRMS_ERR_UNSUPPORTED_SHAPE);
            }
        }
    {
        addrms_cfg bad{8, 1024, 2, 0, 1, 0, 0, 0};
        char why[600];
        CHECK(addrms_cfg_feasible(&bad, 64, 4096, ADDRMS_BF16, why, sizeof why, nullptr) == ADDRMS_ERR_INFEASIBLE_CFG);
        CHECK(strlen(why) > 10);
        CHECK(addrms_cfg_feasible(nullptr, 64, 4096, ADDRMS_BF16, why, sizeof why, nullptr) == ADDRMS_ERR_INVALID_ARG);
        int64_t grid = 0;
        const int64_t n = addrms_enumerate_feasible(4096, 4096, ADDRMS_BF16, nullptr, 0, &grid);
        CHECK(n > 1000 && grid > n);
        std::vector<addrms_cfg> some(100);                          // a buffer smaller than the region
        CHECK(addrms_enumerate_feasible(4096, 4096, ADDRMS_BF16, some.data(), 100, nullptr) == n);
        std::vector<addrms_cfg> all(n);
        CHECK(addrms_enumerate_feasible(4096, 4096, ADDRMS_BF16, all.data(), n, nullptr) == n);
        CHECK(addrms_enumerate_feasible(4096, 4096, ADDRMS_BF16, nullptr, 5, nullptr) == ADDRMS_ERR_INVALID_ARG);
        addrms_hw_limits lim{};
        CHECK(addrms_get_hw_limits(&lim) == ADDRMS_OK && lim.compute_units == 256);
    }
    // ---- table
    {
        const std::string path = std::string(tmp) + "/host_sanitize_table.txt";
        addrms_cfg a{8, 576, 1, 0, 1, ADDRMS_FLAG_NONTEMPORAL, 5, 0}, got{};
        addrms_table_clear();
        CHECK(addrms_table_insert(4096, 4096, ADDRMS_BF16, &a, 23.5) == ADDRMS_OK);
        CHECK(addrms_table_insert(4096, 4096, ADDRMS_BF16, nullptr, 1.0) == ADDRMS_ERR_INVALID_ARG);
        CHECK(addrms_table_lookup(100, 4096, ADDRMS_BF16, &got) == ADDRMS_OK && got.threads_per_row == 576);
        CHECK(addrms_table_save(path.c_str()) == ADDRMS_OK);
        addrms_table_clear();
        CHECK(addrms_table_size() == 0);
        CHECK(addrms_table_load(path.c_str()) == ADDRMS_OK && addrms_table_size() == 1);
        FILE* f = fopen(path.c_str(), "w");
        CHECK(f != nullptr);
        fputs("addrms-table 3 gfx950\n0 0 1 8192 8 1024 1 0 1 0\n", f);      // truncated entry
        fclose(f);
        CHECK(addrms_table_load(path.c_str()) == ADDRMS_ERR_IO && addrms_table_size() == 1);
        CHECK(addrms_table_load((path + ".missing").c_str()) == ADDRMS_ERR_IO);
        CHECK(addrms_table_save("/nonexistent-dir/x/y.txt") == ADDRMS_ERR_IO);
        remove(path.c_str());
    }
    // ---- search, both strategies, with failing candidates; and on the long-row forms
    addrms_backend be{nullptr, validate, measure};
    {
        addrms_cfg best{};
        addrms_tune_report rep{};
        addrms_budget b{};
        const std::string log = std::string(tmp) + "/host_sanitize_log.jsonl";
        b.log_path = log.c_str();
        CHECK(addrms_tune_with_backend(4096, 4096, ADDRMS_BF16, &b, &be, &best, &rep) == ADDRMS_OK);
        CHECK(rep.n_measured > 20 && rep.n_failed > 0 && rep.best_us > 0);
        b.strategy = ADDRMS_SEARCH_EXHAUSTIVE;
        b.log_path = nullptr;
        CHECK(addrms_tune_with_backend(64, 1000, ADDRMS_FP16_RES32, &b, &be, &best, &rep) == ADDRMS_OK);
        CHECK(rep.n_measured + rep.n_failed == rep.n_feasible);
        b.strategy = ADDRMS_SEARCH_GUIDED;
        CHECK(addrms_tune_with_backend(64, 65536, ADDRMS_BF16, &b, &be, &best, nullptr) == ADDRMS_OK);
        CHECK(best.flags & (ADDRMS_FLAG_TWO_PASS | ADDRMS_FLAG_LDS_CACHE));
        b.max_candidates = 3;
        CHECK(addrms_tune_with_backend(4096, 4096, ADDRMS_BF16, &b, &be, &best, &rep) == ADDRMS_OK && rep.n_measured <= 3);
        CHECK(addrms_tune_with_backend(4096, 4096, ADDRMS_BF16, &b, nullptr, &best, &rep) == ADDRMS_ERR_INVALID_ARG);
        CHECK(addrms_tune_with_backend(4096, 4096, ADDRMS_BF16, &b, &be, nullptr, &rep) == ADDRMS_ERR_INVALID_ARG);
        remove(log.c_str());
    }
    // ---- general selection, outer loop, rule audit
    {
        addrms_backend_factory fac{nullptr, open_be, close_be};
        const addrms_shape shapes[3] = {{4096, 4096}, {2048, 8192}, {512, 7168}};
        addrms_cfg g{};
        addrms_general_report grep{};
        CHECK(addrms_select_general_with_backend(shapes, 3, ADDRMS_BF16, nullptr, &fac, &g, &grep) == ADDRMS_OK);
        CHECK(grep.n_shapes == 3 && grep.geomean_speedup_general > 0.9);
        CHECK(addrms_select_general_with_backend(shapes, 0, ADDRMS_BF16, nullptr, &fac, &g, &grep) == ADDRMS_ERR_INVALID_ARG);
        addrms_rounds_report rr{};
        CHECK(addrms_tune_rounds_with_backend(shapes, 2, ADDRMS_BF16, nullptr, &fac, &g, &rr) == ADDRMS_OK);
        CHECK(rr.n_rounds == ADDRMS_MAX_ROUNDS && rr.best_round >= 0);
        addrms_audit_report ar{};
        addrms_budget b{};
        b.max_candidates = 200;
        CHECK(addrms_audit_rules_with_backend(2048, 1000, ADDRMS_FP16_RES32, &b, &be, &ar) == ADDRMS_OK);
        CHECK(ar.n_retained > 1000 && ar.n_retained_measured + ar.n_retained_failed == ar.n_retained);
        CHECK(addrms_audit_rules_with_backend(2048, 1000, ADDRMS_FP16_RES32, &b, &be, nullptr) == ADDRMS_ERR_INVALID_ARG);
    }
    printf("host sanitize driver: ok (%d backend calls)\n", g_calls);
    return 0;
}
