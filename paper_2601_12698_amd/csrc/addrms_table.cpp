// Specialised configuration table D_spec (Algorithm 1 line 23, BuildSpecialized):
// (dtype, N, M) -> configuration, with a nearest-M fallback for row counts that
// were never tuned, and a plain-text file form so a tuning run can be reused.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <map>
#include <mutex>
#include <string>
#include <tuple>

#include "addrms_internal.h"

namespace addrms_host {

struct Entry { addrms_cfg cfg; double us; };
using Key = std::tuple<int, int, int64_t, int64_t>;   // operator, dtype, N, M

static std::mutex g_mu;
static std::map<Key, Entry>& table()
{
    static std::map<Key, Entry> t;
    return t;
}

// The table file named by the environment variable ADDRMS_TABLE_FILE, if any, is the tune cache of the process:
// read once before the table is first consulted or extended, rewritten after every insertion.  A file that exists
// but cannot be loaded (another architecture, another library version, malformed) is left alone: nothing is read
// from it and nothing is written over it.
static std::once_flag g_cache_once;
static std::string g_cache_path;     // empty: no cache file in use
static void open_cache_once()
{
    std::call_once(g_cache_once, [] {
        const char* p = getenv("ADDRMS_TABLE_FILE");
        if (!p || !*p) return;
        FILE* f = fopen(p, "r");
        if (!f) { g_cache_path = p; return; }          // not there yet: the first insertion creates it
        fclose(f);
        if (addrms_table_load(p) == ADDRMS_OK) g_cache_path = p;
    });
}

int table_insert(int64_t M, int64_t N, int dtype, const addrms_cfg& cfg, double mean_us, int op)
{
    const Feas f = check_cfg(cfg, M, N, dtype, op);
    if (f.status != ADDRMS_OK) return fail(f.status, "%s", f.reason.c_str());
    open_cache_once();
    {
        std::lock_guard<std::mutex> lock(g_mu);
        table()[Key(op, dtype, N, M)] = Entry{cfg, mean_us};
    }
    if (!g_cache_path.empty()) return addrms_table_save(g_cache_path.c_str());
    return ADDRMS_OK;
}

int table_lookup(int64_t M, int64_t N, int dtype, addrms_cfg* out, int op)
{
    open_cache_once();
    std::lock_guard<std::mutex> lock(g_mu);
    auto& t = table();
    auto it = t.find(Key(op, dtype, N, M));
    if (it != t.end()) { *out = it->second.cfg; return ADDRMS_OK; }
    // Same (dtype, N): nearest M in ratio whose cfg is still feasible at this M.
    double best = 0.0;
    const Entry* pick = nullptr;
    for (auto lo = t.lower_bound(Key(op, dtype, N, INT64_MIN)); lo != t.end(); ++lo) {
        if (std::get<0>(lo->first) != op || std::get<1>(lo->first) != dtype || std::get<2>(lo->first) != N) break;
        const double d = fabs(log(static_cast<double>(std::max<int64_t>(std::get<3>(lo->first), 1)) /
                                  static_cast<double>(std::max<int64_t>(M, 1))));
        if (pick && d >= best) continue;
        if (check_cfg(lo->second.cfg, M, N, dtype, op).status != ADDRMS_OK) continue;
        best = d;
        pick = &lo->second;
    }
    if (!pick) return ADDRMS_ERR_NO_RESULT;
    *out = pick->cfg;
    return ADDRMS_OK;
}

// File form: a format line, the architecture the entries were measured on, the library
// version that wrote them, then one entry per line.  Timings and feasibility are facts
// about one architecture and one set of compiled kernel instances, so a file written for
// another architecture or by a library of another major.minor version is refused whole.
static const char kMagic[] = "addrms-table 4";
static const char kArch[] = "gfx950";

static bool same_major_minor(const char* a, const char* b)
{
    int dots = 0;
    for (; *a && *b; ++a, ++b) {
        if (*a != *b) return false;
        if (*a == '.' && ++dots == 2) return true;
    }
    return *a == *b;
}

}  // namespace addrms_host

using namespace addrms_host;

extern "C" {

int addrms_table_insert(int64_t M, int64_t N, int dtype, const addrms_cfg* cfg, double mean_us)
{
    if (!cfg) return fail(ADDRMS_ERR_INVALID_ARG, "cfg is NULL");
    return table_insert(M, N, dtype, *cfg, mean_us, OP_ADDRMS);
}

int addrms_table_lookup(int64_t M, int64_t N, int dtype, addrms_cfg* out) { return export_table_lookup(OP_ADDRMS, M, N, dtype, out); }

int64_t addrms_table_size(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    return static_cast<int64_t>(table().size());
}

void addrms_table_clear(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    table().clear();
}

int addrms_table_save(const char* path)
{
    if (!path) return fail(ADDRMS_ERR_INVALID_ARG, "path is NULL");
    std::lock_guard<std::mutex> lock(g_mu);
    // written beside the target and renamed over it, so that a reader never sees half a file
    const std::string tmp = std::string(path) + ".tmp";
    FILE* f = fopen(tmp.c_str(), "w");
    if (!f) return fail(ADDRMS_ERR_IO, "cannot open %s for writing", tmp.c_str());
    fprintf(f, "%s\narch %s\nlibrary %s\n# operator dtype M N vec threads_per_row rows_per_wg reduce unroll flags "
               "max_waves_per_simd walk mean_us\n", kMagic, kArch, ADDRMS_VERSION_STRING);
    for (const auto& kv : table()) {
        const addrms_cfg& c = kv.second.cfg;
        fprintf(f, "%d %d %lld %lld %d %d %d %d %d %d %d %d %.6f\n", std::get<0>(kv.first), std::get<1>(kv.first),
                (long long)std::get<3>(kv.first), (long long)std::get<2>(kv.first), c.vec, c.threads_per_row,
                c.rows_per_wg, c.reduce, c.unroll, c.flags, c.max_waves_per_simd, c.walk, kv.second.us);
    }
    const bool bad = ferror(f) != 0;
    if (fclose(f) != 0 || bad) { remove(tmp.c_str()); return fail(ADDRMS_ERR_IO, "write to %s failed", tmp.c_str()); }
    if (rename(tmp.c_str(), path) != 0) { remove(tmp.c_str()); return fail(ADDRMS_ERR_IO, "cannot move %s to %s", tmp.c_str(), path); }
    return ADDRMS_OK;
}

int addrms_table_load(const char* path)
{
    if (!path) return fail(ADDRMS_ERR_INVALID_ARG, "path is NULL");
    FILE* f = fopen(path, "r");
    if (!f) return fail(ADDRMS_ERR_IO, "cannot open %s", path);
    char line[512];
    std::map<Key, Entry> staged;
    int lineno = 0;
    bool have_magic = false, have_arch = false, have_version = false;
    while (fgets(line, sizeof line, f)) {
        ++lineno;
        size_t len = strlen(line);
        while (len && (line[len - 1] == '\n' || line[len - 1] == '\r')) line[--len] = '\0';
        if (!have_magic) {
            if (strcmp(line, kMagic) != 0) {
                fclose(f);
                return fail(ADDRMS_ERR_IO, "%s: not an addrms table of this format (first line is not \"%s\")", path, kMagic);
            }
            have_magic = true;
            continue;
        }
        if (!have_arch) {
            if (strncmp(line, "arch ", 5) != 0 || strcmp(line + 5, kArch) != 0) {
                fclose(f);
                return fail(ADDRMS_ERR_IO, "%s: written for \"%s\", this library runs on \"arch %s\": timings and feasible "
                            "regions do not carry over", path, line, kArch);
            }
            have_arch = true;
            continue;
        }
        if (!have_version) {
            if (strncmp(line, "library ", 8) != 0 || !same_major_minor(line + 8, ADDRMS_VERSION_STRING)) {
                fclose(f);
                return fail(ADDRMS_ERR_IO, "%s: written by \"%s\", this is library %s: the kernel instances differ", path, line,
                            ADDRMS_VERSION_STRING);
            }
            have_version = true;
            continue;
        }
        if (len == 0 || line[0] == '#') continue;
        int op, dtype; long long M, N; addrms_cfg c{}; double us; int used = 0;
        const int got = sscanf(line, "%d %d %lld %lld %d %d %d %d %d %d %d %d %lf %n", &op, &dtype, &M, &N, &c.vec,
                               &c.threads_per_row, &c.rows_per_wg, &c.reduce, &c.unroll, &c.flags,
                               &c.max_waves_per_simd, &c.walk, &us, &used);
        if (got != 13 || op < 0 || op >= kNumOps || static_cast<size_t>(used) != len) {
            fclose(f);
            return fail(ADDRMS_ERR_IO, "%s:%d: malformed entry", path, lineno);
        }
        const Feas fe = check_cfg(c, M, N, dtype, op);
        if (fe.status != ADDRMS_OK) {
            fclose(f);
            return fail(ADDRMS_ERR_IO, "%s:%d: entry is not feasible: %s", path, lineno, fe.reason.c_str());
        }
        staged[Key(op, dtype, N, M)] = Entry{c, us};
    }
    fclose(f);
    if (!have_magic || !have_arch || !have_version) return fail(ADDRMS_ERR_IO, "%s: header incomplete (format, arch and library lines)", path);
    std::lock_guard<std::mutex> lock(g_mu);
    for (const auto& kv : staged) table()[kv.first] = kv.second;
    return ADDRMS_OK;
}

}  // extern "C"
