// Internal declarations shared by the host-side translation units of libaddrms.
// Nothing here is part of the ABI.
#pragma once
#include <stdarg.h>
#include <stdint.h>

#include <map>
#include <string>
#include <vector>

#include "addrms.h"

namespace addrms_host {

// ---- r(h): resource upper bounds of the target (Algorithm 1, Input) --------
// MI355X / gfx950 (CDNA4), public figures.
struct HwLimits {
    int compute_units = 256;
    int xcds = 8;
    int simds_per_cu = 4;
    int wave_size = 64;
    int max_waves_per_simd = 8;
    int regs_per_lane = 512;        // unified VGPR+AGPR file entries per lane per SIMD
    int reg_granule = 8;            // allocation granularity of that file
    int lds_bytes_per_cu = 160 * 1024;
    int lds_granule = 1280;         // LDS allocation granularity in bytes
    int max_threads_per_wg = 1024;
    int max_wgs_per_cu = 32;        // workgroup slots per CU (16 when a workgroup has several waves)
    int max_multiwave_wgs_per_cu = 16;
    int max_access_bytes = 16;      // widest single global load/store per lane
    double hbm_bytes_per_s = 8.0e12;
    int64_t last_level_cache_bytes = 256ll << 20;  // Infinity Cache
    int64_t l2_bytes_per_xcd = 4ll << 20;
};
const HwLimits& hw();

// Floors below which a launch shape is pruned as obviously inefficient.
constexpr int kMinWavesPerSimd = 2;
constexpr int kMaxElemsPerThread = 64;   // register row cache, fp32 values per thread
constexpr int kSpanCptBase = 200;        // aligned-span form: cpt = 200 + chunks per thread
constexpr int kLdsCacheCptBase = 300;    // forms with the row cache continued in LDS: cpt = 300 + register-held chunks
constexpr int kLdsCacheRegElems = 48;    // their values per thread kept in registers (a 1024-thread workgroup leaves each lane
                                         // 128 registers; 64 cached values spill)
// The same body compiled for workgroups of at most 512 threads, where each lane has 256 registers: 144 values per
// thread stay in registers (vec 4 and 8 only; cpt = 400 + register-held chunks).  No knob selects it: check_cfg takes
// it where the 48-value instance cannot keep the whole row on the chip at the launch shape asked for.
constexpr int kLdsCacheBigCptBase = 400;
constexpr int kLdsCacheBigRegElems = 144;
constexpr int kLdsCacheBigMaxThreads = 512;
constexpr int kLineBytes = 128;          // cache line of the L2 / memory side
constexpr int64_t kMaxTwoPassElemsPerWg = 1ll << 28;   // two-pass form: rows_per_wg * N elements, 32-bit byte offsets

// ---- operators that go through the tuner ------------------------------------
enum Op : int { OP_ADDRMS = 0, OP_SILUMUL = 1, OP_MERGE = 2 };
constexpr int kNumOps = 3;
const char* op_name(int op);

// ---- kernel instances ------------------------------------------------------
struct Instance { int op, dt, vec, cpt, unr, nt, df, maxt; };
struct InstanceRes { int vgprs, agprs, sgprs, scratch, lds_static, occupancy; };

int n_instances();
const Instance& instance(int idx);
const InstanceRes& instance_res(int idx);
// Index of the instance with exactly these knob values, or -1.
int find_instance(int op, int dt, int vec, int cpt, int unr, int nt, int df = 0);
bool cpt_supported(int op, int cpt);

// ---- storage formats -------------------------------------------------------
bool dtype_valid(int dtype, int op = OP_ADDRMS);
// Bytes the operator must move for (M rows, N outputs per row).
int64_t algorithmic_bytes(int op, int64_t M, int64_t N, int dtype);
int x_bytes(int dtype);
int r_bytes(int dtype);
const char* dtype_name(int dtype);

// ---- feasibility -----------------------------------------------------------
// Efficiency rules that an audit may switch off to measure what they prune.  Rules that
// keep a launch valid (sizes, alignment, instance limits, LDS, at least one workgroup per
// CU) and rules that only remove duplicates of another cfg can never be switched off.
enum Relax : int { RELAX_LANE_UTILISATION = 1, RELAX_OCCUPANCY_FLOOR = 2, RELAX_SCRATCH = 4, RELAX_TWO_PASS_NEEDLESS = 8,
                   RELAX_LDS_CACHE_NEEDLESS = 16, RELAX_SPAN_NEEDLESS = 32, RELAX_ALL = 63 };

struct Feas {
    int status = ADDRMS_OK;
    const char* rule = "";      // short tag of the rule that rejected the cfg
    const char* soft_rule = ""; // first efficiency rule that a relaxed check let the cfg past
    std::string reason;
    int inst = -1;              // instance index when one was selected
    int dyn_lds = 0;            // dynamic LDS bytes of the launch (reduction scratch, row cache, occupancy padding)
    int lds_chunks = -1;        // forms with the cache continued in LDS: chunks per thread parked there (-1: another form)
    addrms_resources res{};
};
Feas check_cfg(const addrms_cfg& c, int64_t M, int64_t N, int dtype, int op = OP_ADDRMS, int relax = 0);
// Walks the whole knob grid; `pruned` (optional) counts rejected points by rule tag.
void enumerate(int64_t M, int64_t N, int dtype, std::vector<addrms_cfg>* out, int64_t* n_grid,
               std::map<std::string, int64_t>* pruned = nullptr, int op = OP_ADDRMS, int relax = 0);
int default_cfg(int64_t N, int dtype, addrms_cfg* out, std::string* why, int op = OP_ADDRMS);
// Dynamic LDS bytes of a launch: what the reduction needs, raised to the padding that
// imposes cfg.max_waves_per_simd (0 if the cap cannot be imposed; check_cfg rejects that).
int lds_bytes_for(const addrms_cfg& c, int op = OP_ADDRMS);
int reduction_lds_bytes(const addrms_cfg& c, int op = OP_ADDRMS);
// Workgroups per CU that cfg.max_waves_per_simd allows (0 = no cap requested).
int capped_wgs_per_cu(const addrms_cfg& c);
// Blocks of rows_per_wg rows; and the grid size: one workgroup per block, or for a
// persistent cfg the number of workgroups resident on the chip (wgs_per_cu from check_cfg).
int64_t n_row_blocks(const addrms_cfg& c, int64_t M);
int64_t n_workgroups(const addrms_cfg& c, int64_t M, int wgs_per_cu);

bool cfg_equal(const addrms_cfg& a, const addrms_cfg& b);
uint64_t cfg_key(const addrms_cfg& c);
std::string cfg_json(const addrms_cfg& c);

// ---- specialised table -----------------------------------------------------
int table_lookup(int64_t M, int64_t N, int dtype, addrms_cfg* out, int op = OP_ADDRMS);
int table_insert(int64_t M, int64_t N, int dtype, const addrms_cfg& cfg, double mean_us, int op);

// ---- search ----------------------------------------------------------------
int run_search(int64_t M, int64_t N, int dtype, const addrms_budget* budget,
               const addrms_backend& be, addrms_cfg* out_cfg, addrms_tune_report* report, int op = OP_ADDRMS);

// ---- general configuration ---------------------------------------------------
// insert_in_table: store each shape's winner in the specialised table (device runs only).
int run_select_general(const addrms_shape* shapes, int n, int dtype, const addrms_budget* budget,
                       const addrms_backend_factory& factory, bool insert_in_table,
                       addrms_cfg* out_general, addrms_general_report* report, int op = OP_ADDRMS);

int run_tune_rounds(const addrms_shape* shapes, int n, int dtype, const addrms_budget* budget,
                    const addrms_backend_factory& factory, bool insert_in_table,
                    addrms_cfg* out_general, addrms_rounds_report* report, int op = OP_ADDRMS);
// Measures what the efficiency rules of the deriver prune (see addrms_audit_rules).
int run_audit_rules(int64_t M, int64_t N, int dtype, const addrms_budget* budget, const addrms_backend& be,
                    addrms_audit_report* report);
// True if cfg only uses strategy families allowed by mask (0 = all).
bool cfg_in_families(const addrms_cfg& c, int family_mask);

// ---- host-only entry points, operator-indexed (the exported names are thin wrappers) ----
int export_default_cfg(int op, int64_t N, int dtype, addrms_cfg* out);
int export_cfg_feasible(int op, const addrms_cfg* cfg, int64_t M, int64_t N, int dtype, char* reason, size_t reason_len,
                        addrms_resources* res);
int64_t export_enumerate_feasible(int op, int64_t M, int64_t N, int dtype, addrms_cfg* out, int64_t cap, int64_t* n_grid);
int export_table_lookup(int op, int64_t M, int64_t N, int dtype, addrms_cfg* out);
int64_t export_algorithmic_bytes(int op, int64_t M, int64_t N, int dtype);

// 0, 1 or 2: what the environment variable ADDRMS_VERBOSE asks the searches and the audit to report on stderr.
int verbosity();

// ---- error text ------------------------------------------------------------
int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

}  // namespace addrms_host
