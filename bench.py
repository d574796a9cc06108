#!/usr/bin/env python3
"""Benchmark of the fused residual-add + RMSNorm hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--op addrms|silumul|mergestates]

Headline workload: the large prefill shape M=32768, N=7168, bf16 storage with 1 % outliers
(seed 3), the largest of the benchmark configurations that one GPU holds (1.88 GB moved per
step).  One step = one in-place launch of the operator through the C ABI over one batch that
is already resident in HBM.  The launches rotate through enough buffer sets that every step
streams from HBM rather than from the 256 MB last-level cache.

Before the timed region the library's guided search tunes the launch configuration and its
Top-K are re-tested once on the workload's own buffers, the fastest being kept (the cost of
both is reported, not timed as steps).  Then, for the headline workload:
  * W untimed warm-up steps and exactly K timed steps of the tuned configuration, bracketed
    by device synchronisation (`value`, `ms_per_step`), with HIP events on the launch stream
    around the same K steps (`roofline`);
  * the same for the untuned default configuration (`default_cfg`);
  * blocks of launches of the default and the tuned configuration in alternation, each block
    timed with events, and the median block of each (`interleaved`): clock or thermal drift
    hits both alike and a slow first block does not decide the ratio;
  * the library's copy-like calibration kernel over the same buffers (`copy_probe`): the
    same bytes with none of the arithmetic, the practical ceiling of this traffic pattern;
  * the same copy under the operator's constraint (`row_probe`): a workgroup holds a whole
    row of both streams across a barrier before it writes anything, best over workgroup
    sizes and occupancy caps -- what the row-wise reduction costs by its structure alone.
All five benchmark configurations (smoke, prefill, the decode sweep, large prefill, the three
odd-width mixed-precision shapes) are then tuned and timed by the library's own measurement
harness (20 warm-up + 100 timed launches, twice, rotated buffers) and listed under `configs`.
One JSON line is printed.

--op silumul / --op mergestates time the two further operators that sit behind the same
tuner with the same protocol and print the same kind of line.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
LLC_BYTES = 256 << 20           # Infinity Cache
L2_TOTAL_BYTES = 8 * (4 << 20)
SKEW_BYTES = 4096               # residual base is skewed against x by one 4 KiB interleave unit
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "addrms_hbm_traffic.md")
METRIC = "fused add+RMSNorm achieved HBM GB/s (% of peak), tuned vs default cfg"


def measured_traffic(workload_name, cfg=None):
    """HBM bytes per launch on `workload_name`, as the profiler's FETCH_SIZE and WRITE_SIZE counters measured them
    (rows of the table in profiles/addrms_hbm_traffic.md, which `python -m paper_2601_12698_amd.signals
    --traffic-report` writes): the row of exactly this cfg if the table has one, else the row of the cfg that was
    the tuned one when the table was written.  None if the workload was not measured."""
    want = ",".join(str(v) for v in cfg) if cfg is not None else None
    found = None
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                cells = [c.strip() for c in line.split("|")]
                if len(cells) >= 9 and cells[1] == workload_name and (cells[3] == want or (cells[2] == "tuned" and found is None)):
                    found = {"bytes": int(cells[6]), "cfg": cells[3], "over_algorithmic": float(cells[8])}
                    if cells[3] == want:
                        break
    except (OSError, ValueError):
        pass
    return found


def recorded_regret(label="prefill"):
    """Regret of the guided search against the exhaustive one on prefill 4096 x 4096 (`label` "prefill") or on the
    headline shape ("large prefill"), as the last run of `python -m paper_2601_12698_amd.report --exhaustive-prefill`
    (`--exhaustive-large`) recorded it: the exhaustive searches take two minutes and half an hour of GPU time, too
    long to repeat in every bench run."""
    import re
    path = os.path.join(ROOT, "profiles", "addrms_tuned_vs_default_all_configs.md")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(label + ": guided"):
                    r = re.findall(r"regret ([0-9.]+)", line)
                    n = re.findall(r"after (\d+) cfgs / (\d+) ms", line)
                    if len(r) == 2 and len(n) == 2:
                        out = {"confirmed_in_search": float(r[0]), "re_measured_in_alternation": float(r[1]),
                               "guided_cfgs": int(n[0][0]), "guided_ms": int(n[0][1]),
                               "exhaustive_cfgs": int(n[1][0]), "exhaustive_ms": int(n[1][1]),
                               "source": "profiles/" + os.path.basename(path)}
                        earlier = re.search(r"and (\d+) taken from the log of earlier runs", line)
                        if earlier:
                            out["exhaustive_cfgs_from_the_log_of_earlier_runs"] = int(earlier.group(1))
                        return out
    except OSError:
        pass
    return None


def device_info(torch):
    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "arch": getattr(p, "gcnArchName", ""), "compute_units": p.multi_processor_count,
            "memory_gib": round(p.total_memory / 2 ** 30, 1)}
    # clocks as far as the runtime exposes them (kHz); the driver's own power-state records sit beside this line
    for key in ("clock_rate", "memory_clock_rate", "memory_bus_width", "L2_cache_size"):
        v = getattr(p, key, None)
        if v:
            info[key] = v
    return info


def pick_workload(W, name):
    if name == "prefill":
        return W.PREFILL
    if name == "large_prefill":
        return W.LARGE_PREFILL
    if name == "smoke":
        return W.SMOKE
    if name.startswith("odd_width_") and int(name[10:]) in W.ODD_WIDTH_N:
        return W.ODD_WIDTH.with_cols(int(name[10:]))
    if name.startswith("decode_") and int(name[7:]) in W.DECODE_M:
        return W.DECODE.with_rows(int(name[7:]))
    print(f"unknown workload {name}", file=sys.stderr)
    sys.exit(2)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the table of all five benchmark configurations (profiler runs want the headline kernels only)")
    ap.add_argument("--tune-log", default=None, help="write the search's JSON-lines log here")
    ap.add_argument("--exhaustive", action="store_true", help="tune by exhaustive search instead of guided")
    ap.add_argument("--cfg", default=None,
                    help="skip the search and time this configuration: vec,threads_per_row,rows_per_wg,reduce,unroll,"
                         "flags,max_waves_per_simd[,walk] (used for profiler runs, whose overhead would mislead the search)")
    ap.add_argument("--workload", default="large_prefill",
                    help="addrms workload of the headline: large_prefill (default; the largest benchmark configuration "
                         "one GPU holds), prefill, smoke, odd_width_5120, odd_width_2880, odd_width_1000 or decode_<M>")
    ap.add_argument("--op", default="addrms", choices=("addrms", "silumul", "mergestates"),
                    help="operator to time (default: the fused add+RMSNorm hot path)")
    ap.add_argument("--probe", action="store_true",
                    help="time only the library's copy-like calibration kernel (same traffic, no arithmetic) over the "
                         "same buffers; used to calibrate profiler byte counters")
    return ap.parse_args()


def carve_sets(torch, wl, W, nsets):
    """One pool, `nsets` (x, r) pairs; r is skewed by SKEW_BYTES against x so that the
    two streams of a lane do not map to the same HBM channel at the same time."""
    xb = wl.M * wl.N * W.x_bytes(wl.dtype)
    rb = wl.M * wl.N * W.r_bytes(wl.dtype)
    align = 1 << 16
    def up(v):
        return (v + align - 1) // align * align
    stride = up(xb) + up(rb) + 2 * align
    pool = torch.empty(stride * nsets + align, dtype=torch.uint8, device="cuda")
    base = (-pool.data_ptr()) % align
    xs, rs = [], []
    for i in range(nsets):
        o = base + i * stride
        xs.append(pool[o:o + xb].view(W.x_torch_dtype(wl.dtype)).view(wl.M, wl.N))
        o2 = o + up(xb) + SKEW_BYTES
        rs.append(pool[o2:o2 + rb].view(W.r_torch_dtype(wl.dtype)).view(wl.M, wl.N))
    return pool, xs, rs


def make_sets(torch, W, wl, d, dtype_id):
    """Resident inputs, rotated so that each step misses the last-level cache."""
    set_bytes = wl.M * wl.N * (W.x_bytes(wl.dtype) + W.r_bytes(wl.dtype))
    nsets = min(256, max(2, -(-4 * (LLC_BYTES + L2_TOTAL_BYTES) // set_bytes)))
    pool, xs, rs = carve_sets(torch, wl, W, nsets)
    w = d["w"].cuda()
    x0, r0 = d["x"].cuda(), d["r"].cuda()
    for x, r in zip(xs, rs):
        x.copy_(x0)
        r.copy_(r0)
    args = [(x.data_ptr(), r.data_ptr(), w.data_ptr(), wl.eps, wl.M, wl.N, dtype_id) for x, r in zip(xs, rs)]
    return (pool, xs, rs, w), nsets, args


class Runner:
    """Enqueues launches on one stream, rotating over the buffer sets."""

    def __init__(self, torch, lib, B, args_per_set, stream):
        self.torch, self.lib, self.B, self.args, self.stream = torch, lib, B, args_per_set, stream
        self.sp = int(stream.cuda_stream)
        self.k = 0

    def run(self, cfg, count):
        ref = ctypes.byref(cfg) if cfg is not None else None
        run, args, n, sp = self.lib.addrms_run, self.args, len(self.args), self.sp
        for _ in range(count):
            a = args[self.k % n]
            self.k += 1
            if run(a[0], a[1], a[2], a[3], a[4], a[5], a[6], ref, sp) != 0:
                raise RuntimeError(self.B.addrms_last_error())

    def probe(self, count):
        fn, args, n, sp = self.lib.addrms_stream_probe, self.args, len(self.args), self.sp
        for _ in range(count):
            a = args[self.k % n]
            self.k += 1
            if fn(a[0], a[1], a[4], a[5], a[6], sp) != 0:
                raise RuntimeError(self.B.addrms_last_error())

    def row_probe(self, threads, wgs, count):
        fn, args, n, sp = self.lib.addrms_row_probe, self.args, len(self.args), self.sp
        for _ in range(count):
            a = args[self.k % n]
            self.k += 1
            if fn(a[0], a[1], a[4], a[5], a[6], threads, wgs, sp) != 0:
                raise RuntimeError(self.B.addrms_last_error())

    def best_row_probe(self, row_x_bytes, launches=12):
        """The row-holding copy over its workgroup sizes and occupancy caps: (us, threads, wgs per CU) of the fastest,
        or None where a row is not a whole number of 16-byte pieces."""
        if row_x_bytes % 16:
            return None
        pieces = row_x_bytes // 16
        shapes = sorted({min(1024, -(-(-(-pieces // c)) // 64) * 64) for c in (1, 2, 3, 4, 6, 8, 12, 16)})
        best = None
        for t in shapes:
            chunks = -(-pieces // t)
            if chunks > 16 or (chunks - 1) * t >= pieces:
                continue
            for wgs in (1, 2, 3, 4, 6, 8):
                if wgs * t > 2048:
                    continue
                _, ev = self.timed(lambda n: self.row_probe(t, wgs, n), 3, launches)
                us = ev * 1e3 / launches
                if best is None or us < best[0]:
                    best = (us, t, wgs)
        if best is None:
            return None
        _, ev = self.timed(lambda n: self.row_probe(best[1], best[2], n), 5, 4 * launches)     # the winner, timed longer
        return (ev * 1e3 / (4 * launches), best[1], best[2])

    def timed(self, launch, warmup, steps):
        """`launch(count)` enqueues count steps.  Returns (wall seconds, event milliseconds) for exactly `steps`
        steps after `warmup` untimed ones, the timed region bracketed by device synchronisation."""
        torch = self.torch
        launch(warmup)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(self.stream)
        launch(steps)
        e1.record(self.stream)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, e0.elapsed_time(e1)

    def interleaved(self, launchers, blocks, per_block):
        """Alternates between the launchers, `blocks` blocks each of `per_block` launches, one event pair per block;
        returns the per-launch microseconds of every block, per launcher."""
        torch = self.torch
        ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(blocks)]
              for _ in launchers]
        for launch in launchers:
            launch(min(per_block, 5))
        for b in range(blocks):
            for i, launch in enumerate(launchers):
                ev[i][b][0].record(self.stream)
                launch(per_block)
                ev[i][b][1].record(self.stream)
        torch.cuda.synchronize()
        return [[e0.elapsed_time(e1) * 1e3 / per_block for e0, e1 in row] for row in ev]


def cpu_baseline(W, wl, d, nbytes):
    """The oracle as it stands, timed on the host cores: a bounded number of
    passes over the same workload, all cores (rows split over threads)."""
    import oracle
    oracle.build()
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))
    xb, rb, wb = W.to_bits(d["x"]), W.to_bits(d["r"]), W.to_bits(d["w"])
    dt = {"bf16": 0, "fp16": 1, "fp16_res32": 2, "fp32": 3}[wl.dtype]
    oracle.addrms(xb[:64], rb[:64], wb, wl.eps, dt, nthreads=cores)            # load + page in
    passes, spent = 0, 0.0
    t_budget = 12.0
    while spent < t_budget and passes < 5000:
        t0 = time.perf_counter()
        oracle.addrms(xb, rb, wb, wl.eps, dt, nthreads=cores)
        spent += time.perf_counter() - t0
        passes += 1
    per = spent / passes
    rows_1 = min(wl.M, 4096)                                                  # a slice on one core: 1.9 GB would take 3 s
    t0 = time.perf_counter()
    oracle.addrms(xb[:rows_1], rb[:rows_1], wb, wl.eps, dt, nthreads=1)
    one = (time.perf_counter() - t0) * wl.M / rows_1
    return {"value": nbytes / per * 1e-9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{passes} full passes over {wl.name} ({wl.M}x{wl.N}), rows split over {cores} threads; "
                      f"plus {rows_1} rows on a single thread, scaled to the full shape",
            "ms_per_step": per * 1e3, "tokens_per_s": wl.M / per,
            "single_thread": {"value": nbytes / one * 1e-9, "unit": "GB/s", "cores": 1, "ms_per_step": one * 1e3}}


def run_probe(a, torch, lib, B, W, wl, d, dtype_id):
    keep, nsets, args = make_sets(torch, W, wl, d, dtype_id)
    r = Runner(torch, lib, B, args, torch.cuda.current_stream())
    wall, ev = r.timed(r.probe, a.warmup, a.steps)
    moved = 2 * wl.M * wl.N * (W.x_bytes(wl.dtype) + W.r_bytes(wl.dtype))
    print(json.dumps({"metric": "stream probe (read and write back x and residual, no arithmetic)",
                      "value": round(moved / (wall / a.steps) * 1e-9, 1), "unit": "GB/s", "n_gpus": 1,
                      "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(wall / a.steps * 1e3, 6),
                      "kernel_us": round(ev / a.steps * 1e3, 3), "bytes_per_step": moved,
                      "config": {"workload": wl.name, "rotating_buffer_sets": nsets}}))


def configs_table(B, W, headline_name, headline_entry):
    """All five benchmark configurations through the library's own harness: guided search, then the confirmation
    protocol (2 x (20 warm-up + 100 timed launches), buffers rotated past the last-level cache) for the winner
    and for the default cfg.  Shapes under about 1 MB of traffic are bound by launch latency, not by HBM."""
    shapes = [W.SMOKE, W.PREFILL] + [W.DECODE.with_rows(m) for m in W.DECODE_M] + [W.LARGE_PREFILL] + \
             [W.ODD_WIDTH.with_cols(n) for n in W.ODD_WIDTH_N]
    out = []
    for wl in shapes:
        if wl.name == headline_name and headline_entry is not None:
            out.append(headline_entry)
            continue
        nbytes = B.addrms_algorithmic_bytes(wl.M, wl.N, wl.dtype)
        t0 = time.perf_counter()
        cfg, rep = B.addrms_tune(wl.M, wl.N, wl.dtype, B.make_budget(eps=wl.eps))
        out.append(config_entry(wl, nbytes, cfg, rep, (time.perf_counter() - t0) * 1e3))
    return out


def config_entry(wl, nbytes, cfg, rep, search_ms):
    gbps = nbytes / rep.best_us * 1e-3
    return {"workload": wl.name, "M": wl.M, "N": wl.N, "storage": wl.dtype, "bytes": nbytes,
            "tuned_us": round(rep.best_us, 3), "default_us": round(rep.default_us, 3),
            "speedup": round(rep.default_us / rep.best_us, 4) if rep.best_us > 0 else None,
            "tuned_gbps": round(gbps, 1), "frac": round(gbps / HBM_PEAK_GBPS, 4),
            "tokens_per_s": round(wl.M / (rep.best_us * 1e-6), 1), "cfg": list(cfg.as_tuple()),
            "search_ms": round(search_ms, 1), "n_measured": rep.n_measured, "n_feasible": rep.n_feasible}


def bounded_cpu_passes(fn, t_budget=12.0):
    fn()
    passes, spent = 0, 0.0
    while spent < t_budget and passes < 5000:
        t0 = time.perf_counter()
        fn()
        spent += time.perf_counter() - t0
        passes += 1
    return spent / passes, passes


def timed_loop(torch, launch, nsets, warmup, steps, stream):
    """`launch(i)` enqueues one step on buffer set i.  Returns (wall s, event ms) for `steps` launches."""
    k = 0
    for _ in range(warmup):
        launch(k % nsets); k += 1
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        launch(k % nsets); k += 1
    e1.record(stream)
    torch.cuda.synchronize()
    return time.perf_counter() - t0, e0.elapsed_time(e1)


def run_other_op(a, torch, lib, B, W):
    """silu_and_mul or merge_attn_states: tune, then default and tuned cfg timed over rotated buffers."""
    stream = torch.cuda.current_stream()
    sp = int(stream.cuda_stream)
    budget = B.make_budget(strategy=B.SEARCH_EXHAUSTIVE if a.exhaustive else B.SEARCH_GUIDED, log_path=a.tune_log)
    if a.op == "silumul":
        wl = W.SILU_PREFILL
        rows, width, units = wl.M, wl.d, wl.M
        nbytes = B.silumul_algorithmic_bytes(wl.M, wl.d, wl.dtype)
        tune, feasible, default_of, run = B.silumul_tune, B.silumul_cfg_feasible, B.silumul_default_cfg, lib.silumul_run
        x0 = W.generate_gated(wl)
        nsets = max(2, -(-4 * (LLC_BYTES + L2_TOTAL_BYTES) // nbytes))
        xs = [x0.cuda() for _ in range(nsets)]
        outs = [torch.empty((wl.M, wl.d), dtype=x0.dtype, device="cuda") for _ in range(nsets)]
        dt = B.DTYPE_IDS[wl.dtype]
        argv = [(x.data_ptr(), o.data_ptr(), wl.M, wl.d, dt) for x, o in zip(xs, outs)]
        metric = "silu_and_mul achieved HBM GB/s (% of peak), tuned vs default cfg"
    else:
        n, h, d = max(W.MERGE_SHAPES, key=lambda t: t[0] * t[1] * t[2])
        wl = W.MergeWorkload(f"merge_{n}x{h}x{d}_bf16", n, h, d, "bf16", 21)
        rows, width, units = wl.rows, wl.d, wl.n
        nbytes = B.mergestates_algorithmic_bytes(wl.rows, wl.d, wl.dtype)
        tune, feasible, default_of, run = (B.mergestates_tune, B.mergestates_cfg_feasible, B.mergestates_default_cfg,
                                           lib.mergestates_run)
        t0 = W.generate_merge(wl)
        nsets = max(2, -(-4 * (LLC_BYTES + L2_TOTAL_BYTES) // nbytes))
        sets = [{k: v.cuda() for k, v in t0.items()} for _ in range(nsets)]
        for s_ in sets:
            s_["vo"] = torch.empty_like(s_["va"])
            s_["so"] = torch.empty_like(s_["sa"])
        dt = B.DTYPE_IDS[wl.dtype]
        argv = [(s_["va"].data_ptr(), s_["sa"].data_ptr(), s_["vb"].data_ptr(), s_["sb"].data_ptr(),
                 s_["vo"].data_ptr(), s_["so"].data_ptr(), wl.rows, wl.d, dt) for s_ in sets]
        metric = "merge_attn_states achieved HBM GB/s (% of peak), tuned vs default cfg"

    t_start = time.perf_counter()
    if a.cfg:
        tuned = B.make_cfg(*[int(v) for v in a.cfg.split(",")])
        st, why, _ = feasible(tuned, rows, width, wl.dtype)
        if st != 0:
            print(f"--cfg is not feasible: {why}", file=sys.stderr)
            sys.exit(2)
        rep = B.TuneReport()
    else:
        tuned, rep = tune(rows, width, wl.dtype, budget)
    tune_wall = time.perf_counter() - t_start
    default = default_of(width, wl.dtype)

    def launcher(cfg):
        ref = ctypes.byref(cfg)
        def launch(i):
            if run(*argv[i], ref, sp) != 0:
                raise RuntimeError(B.addrms_last_error())
        return launch

    wall_d, ev_d = timed_loop(torch, launcher(default), nsets, a.warmup, a.steps, stream)
    wall_t, ev_t = timed_loop(torch, launcher(tuned), nsets, a.warmup, a.steps, stream)
    # default and tuned in alternating blocks, one event pair per block, median block of each
    blocks, per_block = 7, max(5, min(a.steps, 200))
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(blocks)] for _ in (0, 1)]
    launchers, k = [launcher(default), launcher(tuned)], 0
    for b_ in range(blocks):
        for i_, launch in enumerate(launchers):
            ev[i_][b_][0].record(stream)
            for _ in range(per_block):
                launch(k % nsets); k += 1
            ev[i_][b_][1].record(stream)
    torch.cuda.synchronize()
    blk_d, blk_t = ([e0.elapsed_time(e1) * 1e3 / per_block for e0, e1 in row] for row in ev)
    med_d, med_t = statistics.median(blk_d), statistics.median(blk_t)
    value = nbytes / (wall_t / a.steps) * 1e-9
    kernel_us = ev_t / a.steps * 1e3
    achieved = nbytes / (kernel_us * 1e-6) * 1e-9
    out = {
        "metric": metric, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(wall_t / a.steps * 1e3, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "rows": rows, "width": width, "storage": wl.dtype, "seed": wl.seed,
                   "cfg": tuned.as_dict(), "rotating_buffer_sets": nsets, "algorithmic_bytes_per_step": nbytes},
        "pct_of_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "tokens_per_s": round(units / (wall_t / a.steps), 1),
        "default_cfg": {"cfg": default.as_dict(), "value": round(nbytes / (wall_d / a.steps) * 1e-9, 1),
                        "ms_per_step": round(wall_d / a.steps * 1e3, 6), "kernel_us": round(ev_d / a.steps * 1e3, 3)},
        "tuned_over_default": round(wall_d / wall_t, 4),
        "interleaved": {"blocks": blocks, "launches_per_block": per_block,
                        "tuned_us_median": round(med_t, 3), "default_us_median": round(med_d, 3),
                        "tuned_over_default": round(med_d / med_t, 4),
                        "tuned_gbps_median": round(nbytes / med_t * 1e-3, 1),
                        "tuned_frac_median": round(nbytes / med_t * 1e-3 / HBM_PEAK_GBPS, 4),
                        "tuned_us_blocks": [round(v, 2) for v in blk_t],
                        "default_us_blocks": [round(v, 2) for v in blk_d]},
        "tune": {"strategy": "given" if a.cfg else "exhaustive" if a.exhaustive else "guided",
                 "wall_ms": round(tune_wall * 1e3, 1), "n_grid": rep.n_grid, "n_feasible": rep.n_feasible,
                 "n_measured": rep.n_measured, "n_failed": rep.n_failed, "best_us": round(rep.best_us, 3),
                 "default_us": round(rep.default_us, 3)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None, "kernel_us": round(kernel_us, 3),
                     "algorithmic_bytes": nbytes},
    }
    out["device"] = device_info(torch)
    if not a.no_cpu_baseline:
        import oracle
        oracle.build()
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))
        if a.op == "silumul":
            xb = W.to_bits(x0)
            per, passes = bounded_cpu_passes(lambda: oracle.silumul(xb, dt, nthreads=cores))
            sample = f"{passes} full passes over {wl.name}, rows split over {cores} threads"
        else:
            cores = 1                                   # this oracle is a plain serial loop
            bits = {k: (W.to_bits(v) if k in ("va", "vb") else v.numpy()) for k, v in t0.items()}
            per, passes = bounded_cpu_passes(lambda: oracle.mergestates(bits["va"], bits["sa"], bits["vb"], bits["sb"], dt))
            sample = f"{passes} full passes over {wl.name} on one thread"
        out["cpu_baseline"] = {"value": nbytes / per * 1e-9, "unit": "GB/s", "cores": cores, "kind": "oracle",
                               "sample": sample, "ms_per_step": per * 1e3}
    print(json.dumps(out))


def main():
    a = parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (rows are independent, so more GPUs "
              "means sharding rows with no communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if a.steps < 1 or a.warmup < 0:
        print("need --steps >= 1 and --warmup >= 0", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2601_12698_amd import binding as B
    from paper_2601_12698_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    lib = B.load()
    if a.op != "addrms":
        if a.probe:
            print("--probe applies to --op addrms only", file=sys.stderr)
            sys.exit(2)
        run_other_op(a, torch, lib, B, W)
        return
    wl = pick_workload(W, a.workload)
    dtype_id = B.DTYPE_IDS[wl.dtype]
    nbytes = B.addrms_algorithmic_bytes(wl.M, wl.N, wl.dtype)
    d = W.generate(wl)

    if a.probe:
        run_probe(a, torch, lib, B, W, wl, d, dtype_id)
        return

    # ---- Level 2 of the tuner: feasible region + search (reported, not timed as steps)
    budget = B.make_budget(strategy=B.SEARCH_EXHAUSTIVE if a.exhaustive else B.SEARCH_GUIDED, eps=wl.eps,
                           log_path=a.tune_log, top_k=7)    # seven confirmed + the default: all re-tested below
    t0 = time.perf_counter()
    if a.cfg:
        tuned = B.make_cfg(*[int(v) for v in a.cfg.split(",")])
        st, why, _ = B.addrms_cfg_feasible(tuned, wl.M, wl.N, wl.dtype)
        if st != 0:
            print(f"--cfg is not feasible: {why}", file=sys.stderr)
            sys.exit(2)
        rep = None
    else:
        tuned, rep = B.addrms_tune(wl.M, wl.N, wl.dtype, budget)
    tune_wall = time.perf_counter() - t0
    default = B.addrms_default_cfg(wl.N, wl.dtype)

    keep, nsets, args = make_sets(torch, W, wl, d, dtype_id)
    stream = torch.cuda.current_stream()
    r = Runner(torch, lib, B, args, stream)

    # The search ranked its Top-K on the library's own synthetic buffers; they are usually within a per cent of each
    # other.  Re-test them once on this workload's buffers (alternating blocks, median block of each) and take the
    # fastest: still part of tuning (Section 3.2's Top-K re-test), done before anything is timed as a step.
    retest = None
    if rep is not None and rep.n_topk > 1:
        cands = [B.make_cfg(*rep.topk[i].as_tuple()) for i in range(rep.n_topk)]
        t0 = time.perf_counter()
        per = r.interleaved([(lambda n, c=c: r.run(c, n)) for c in cands], 5, max(5, min(40, int(4000 / max(rep.best_us, 1.0)))))
        med = [statistics.median(v) for v in per]
        pick = min(range(len(cands)), key=lambda i: med[i])
        retest = {"candidates": [list(c.as_tuple()) for c in cands], "us_median": [round(v, 3) for v in med],
                  "picked": pick, "wall_ms": round((time.perf_counter() - t0) * 1e3, 1)}
        tuned = cands[pick]
        tune_wall += retest["wall_ms"] * 1e-3

    run_default = lambda n: r.run(default, n)
    run_tuned = lambda n: r.run(tuned, n)
    wall_d, ev_d = r.timed(run_default, a.warmup, a.steps)
    wall_t, ev_t = r.timed(run_tuned, a.warmup, a.steps)                   # the K timed steps of the headline
    wall_p, ev_p = r.timed(r.probe, a.warmup, a.steps)
    blocks, per_block = 7, max(5, min(a.steps, 40))
    blk_d, blk_t, blk_p = r.interleaved([run_default, run_tuned, r.probe], blocks, per_block)

    row_best = r.best_row_probe(wl.N * W.x_bytes(wl.dtype))

    ms_step = wall_t / a.steps * 1e3
    value = nbytes / (wall_t / a.steps) * 1e-9
    kernel_us = ev_t / a.steps * 1e3
    achieved = nbytes / (kernel_us * 1e-6) * 1e-9
    probe_bytes = 2 * wl.M * wl.N * (W.x_bytes(wl.dtype) + W.r_bytes(wl.dtype))
    probe_us = ev_p / a.steps * 1e3
    probe_gbps = probe_bytes / (probe_us * 1e-6) * 1e-9
    med_d, med_t, med_p = (statistics.median(v) for v in (blk_d, blk_t, blk_p))
    traffic = measured_traffic(wl.name, tuned.as_tuple())
    out = {
        "metric": METRIC,
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(ms_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "M": wl.M, "N": wl.N, "storage": wl.dtype, "eps": wl.eps, "seed": wl.seed,
                   "cfg": tuned.as_dict(), "rotating_buffer_sets": nsets, "algorithmic_bytes_per_step": nbytes},
        "pct_of_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "tokens_per_s": round(wl.M / (wall_t / a.steps), 1),
        "default_cfg": {"cfg": default.as_dict(), "value": round(nbytes / (wall_d / a.steps) * 1e-9, 1),
                        "ms_per_step": round(wall_d / a.steps * 1e3, 6),
                        "kernel_us": round(ev_d / a.steps * 1e3, 3),
                        "pct_of_peak": round(100.0 * nbytes / (wall_d / a.steps) * 1e-9 / HBM_PEAK_GBPS, 2)},
        "tuned_over_default": round(wall_d / wall_t, 4),
        "interleaved": {"blocks": blocks, "launches_per_block": per_block,
                        "tuned_us_median": round(med_t, 3), "default_us_median": round(med_d, 3),
                        "probe_us_median": round(med_p, 3), "tuned_over_default": round(med_d / med_t, 4),
                        "tuned_gbps_median": round(nbytes / med_t * 1e-3, 1),
                        "tuned_frac_median": round(nbytes / med_t * 1e-3 / HBM_PEAK_GBPS, 4),
                        "tuned_us_blocks": [round(v, 2) for v in blk_t],
                        "default_us_blocks": [round(v, 2) for v in blk_d]},
        "copy_probe": {"what": "library calibration kernel: reads and writes back x and residual over the same buffers, "
                               "no arithmetic, streaming policy, three 256-thread workgroups per CU",
                       "value": round(probe_gbps, 1), "unit": "GB/s", "kernel_us": round(probe_us, 3),
                       "frac_of_peak": round(probe_gbps / HBM_PEAK_GBPS, 4),
                       "operator_frac_of_probe": round(achieved / probe_gbps, 4),
                       "operator_frac_of_probe_interleaved": round((nbytes / med_t) / (probe_bytes / med_p), 4)},
        "row_probe": None if row_best is None else {
            "what": "copy under the operator's constraint: one workgroup holds a whole row of both streams, meets at a "
                    "barrier, then writes it back; no arithmetic; best over workgroup sizes and occupancy caps",
            "value": round(probe_bytes / row_best[0] * 1e-3, 1), "unit": "GB/s", "kernel_us": round(row_best[0], 3),
            "frac_of_peak": round(probe_bytes / row_best[0] * 1e-3 / HBM_PEAK_GBPS, 4),
            "threads_per_row": row_best[1], "wgs_per_cu": row_best[2],
            "operator_over_row_probe": round((nbytes / kernel_us) / (probe_bytes / row_best[0]), 4)},
        "tune": {"strategy": "given" if a.cfg else "exhaustive" if a.exhaustive else "guided", "wall_ms": round(tune_wall * 1e3, 1)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic["bytes"] if traffic else None,
                     "traffic_source": (f"profiles/{os.path.basename(TRAFFIC_FILE)}: FETCH_SIZE + WRITE_SIZE of cfg "
                                        f"{traffic['cfg']}, {traffic['over_algorithmic']:.4f} x algorithmic") if traffic else None,
                     "kernel_us": round(kernel_us, 3), "algorithmic_bytes": nbytes},
    }
    out["tune"]["regret_vs_exhaustive_on_prefill_4096x4096"] = recorded_regret()
    out["tune"]["regret_vs_exhaustive_on_large_prefill_32768x7168"] = recorded_regret("large prefill")
    out["tune"]["regret_vs_exhaustive_on_odd_widths_8192xN"] = {str(n): recorded_regret(f"odd width N={n}") for n in W.ODD_WIDTH_N}
    headline_entry = None
    if retest is not None:
        out["tune"]["retest_on_workload_buffers"] = retest
    if rep is not None:
        out["tune"].update({"n_grid": rep.n_grid, "n_feasible": rep.n_feasible, "n_measured": rep.n_measured,
                            "n_failed": rep.n_failed, "best_found_at": rep.best_found_at,
                            "time_to_best_ms": round(rep.time_to_best_ms, 2), "best_us": round(rep.best_us, 3),
                            "default_us": round(rep.default_us, 3)})
        headline_entry = config_entry(wl, nbytes, rep.best, rep, rep.wall_ms)      # as the library's harness saw it
    del r, keep, args
    torch.cuda.empty_cache()
    if not a.no_configs:
        out["configs"] = configs_table(B, W, wl.name, headline_entry)
    out["device"] = device_info(torch)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(W, wl, d, nbytes)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
