"""Profiling signals for the tuner (Algorithm 1 line 25, CollectSignals; line 9, Suggest).

The paper's testing agent collects performance signals for the configurations a
round produced and the planning agent turns them into suggestions for the next
round.  Hardware counters on this platform are read by ``rocprofv3``, which wraps
a whole process, so collection is out of process:

* ``collect(cfgs, M, N, dtype)`` writes the configurations to a spec file and
  runs ``rocprofv3 --pmc <counters> -- python3 -m paper_2601_12698_amd.signals
  --child <spec>`` once per counter pass (one pass per run: the profiler does
  not split counters over passes and a pass may hold only a few counters of
  each hardware block).  The child launches every configuration a few times
  through the C ABI; the parent reads the per-dispatch counter CSV back and
  averages per configuration.
* ``suggest(record)`` is the deterministic stand-in for the planner: it maps a
  configuration's signals to search hints (``ADDRMS_HINT_*`` bits of the budget)
  with a stated reason each.
* ``tune_with_signals(M, N, dtype)`` is the two-round loop: search, collect
  signals for the Top-K, derive hints, search again with the hints, keep the
  better configuration; everything is appended to a JSON-lines log.  The
  orchestrating process never touches the GPU itself: the searches and the
  profiled launches all run in child processes it starts, so that no process
  that holds GPU state ever has to start another program.

No arithmetic of the operator happens here; kernels run in ``libaddrms.so``.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import shutil
import subprocess
import sys
import tempfile
from typing import Dict, List, Optional, Sequence, Tuple

from . import binding as B

# One list per profiler run.  Derived metrics expand to several hardware counters, so they
# travel alone; FETCH_SIZE uses three L2 counters and WRITE_SIZE two.
DEFAULT_PASSES: Tuple[Tuple[str, ...], ...] = (
    ("FETCH_SIZE",),
    ("WRITE_SIZE",),
    ("TCC_HIT_sum", "TCC_MISS_sum"),
    ("TCC_EA0_WRREQ_STALL_sum", "TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum"),
    ("MemUnitStalled",),
    ("VALUBusy",),
    ("MeanOccupancyPerCU",),
)
LAUNCHES_PER_CFG = 4          # the first launch of each configuration is discarded (cold code, cold TLB)

# FETCH_SIZE and WRITE_SIZE units on this device, from the calibration kernel of known
# traffic (65,536 KiB read registers as 32,779.0; 65,536 KiB written as 65,536.0).
FETCH_UNIT_BYTES = 65536.0 * 1024.0 / 32779.0
WRITE_UNIT_BYTES = 1024.0


def _spec(cfgs: Sequence[B.Cfg], M: int, N: int, dtype: str, eps: float, probes: Sequence[dict] = ()) -> dict:
    return {"M": M, "N": N, "dtype": dtype, "eps": eps, "launches": LAUNCHES_PER_CFG,
            "cfgs": [c.as_dict() for c in cfgs], "probes": list(probes)}


def parse_probes(text: str) -> List[dict]:
    """"copy;rows:256,6" -> the plain calibration copy, then the row-holding copy with 256 threads per row and
    at most six workgroups per CU."""
    out = []
    for t in (text or "").split(";"):
        t = t.strip()
        if not t:
            continue
        if t == "copy":
            out.append({"kind": "copy"})
        elif t.startswith("rows:"):
            threads, wgs = (int(v) for v in t[5:].split(","))
            out.append({"kind": "rows", "threads": threads, "wgs": wgs})
        else:
            raise ValueError(f"unknown probe {t!r}")
    return out


def child_main(spec_path: str) -> int:
    """Runs inside the profiler: launch every cfg of the spec LAUNCHES_PER_CFG times."""
    import torch

    from . import workloads as W
    spec = json.load(open(spec_path))
    M, N, dtype = spec["M"], spec["N"], spec["dtype"]
    wl = W.Workload("signals", M, N, dtype, spec["eps"], 7)
    nsets = 3
    xs = [torch.randn(M, N, device="cuda").to(W.x_torch_dtype(dtype)) for _ in range(nsets)]
    rs = [torch.randn(M, N, device="cuda").to(W.r_torch_dtype(dtype)) for _ in range(nsets)]
    w = (torch.rand(N, device="cuda") + 0.5).to(W.x_torch_dtype(dtype))
    torch.cuda.synchronize()
    k = 0
    for d in spec["cfgs"]:
        cfg = B.make_cfg(**d)
        for _ in range(spec["launches"]):
            B.addrms_run(xs[k % nsets], rs[k % nsets], w, wl.eps, M, N, dtype, cfg)
            k += 1
        torch.cuda.synchronize()
    for pr in spec.get("probes", []):
        for _ in range(spec["launches"]):
            if pr["kind"] == "copy":
                B.addrms_stream_probe(xs[k % nsets], rs[k % nsets], M, N, dtype)
            else:
                B.addrms_row_probe(xs[k % nsets], rs[k % nsets], M, N, dtype, pr["threads"], pr["wgs"])
            k += 1
        torch.cuda.synchronize()
    return 0


def child_probe_main(spec_path: str) -> int:
    """Runs inside the profiler: the library's calibration kernel (known traffic) on the spec's shape."""
    import torch

    from . import workloads as W
    spec = json.load(open(spec_path))
    M, N, dtype = spec["M"], spec["N"], spec["dtype"]
    nsets = 3
    xs = [torch.randn(M, N, device="cuda").to(W.x_torch_dtype(dtype)) for _ in range(nsets)]
    rs = [torch.randn(M, N, device="cuda").to(W.r_torch_dtype(dtype)) for _ in range(nsets)]
    torch.cuda.synchronize()
    for k in range(spec["launches"]):
        B.addrms_stream_probe(xs[k % nsets], rs[k % nsets], M, N, dtype)
    torch.cuda.synchronize()
    return 0


def _read_counter_csv(outdir: str) -> List[dict]:
    rows = []
    for root, _dirs, files in os.walk(outdir):
        for f in files:
            if f.endswith("counter_collection.csv"):
                with open(os.path.join(root, f), newline="") as fh:
                    rows.extend(csv.DictReader(fh))
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    return rows


def collect(cfgs: Sequence[B.Cfg], M: int, N: int, dtype: str, eps: float = 1e-6,
            passes: Sequence[Sequence[str]] = DEFAULT_PASSES, workdir: Optional[str] = None,
            timeout_s: int = 180, probes: Sequence[dict] = ()) -> List[dict]:
    """Counter values per configuration: ``[{cfg, counters: {name: mean}, derived: {...}}, ...]``, followed by one
    record ``{probe, counters, derived}`` per calibration kernel asked for in `probes` (see parse_probes)."""
    rocprof = shutil.which("rocprofv3")
    if rocprof is None:
        raise RuntimeError("rocprofv3 is not on PATH")
    tmp = workdir or tempfile.mkdtemp(prefix="addrms_signals_")
    os.makedirs(tmp, exist_ok=True)
    spec_path = os.path.join(tmp, "spec.json")
    with open(spec_path, "w") as f:
        json.dump(_spec(cfgs, M, N, dtype, eps, probes), f)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ)
    env["PYTHONPATH"] = root + os.pathsep + env.get("PYTHONPATH", "")
    env.setdefault("TMPDIR", "/tmp")
    records = [{"cfg": c.as_dict(), "counters": {}} for c in cfgs] + [{"probe": dict(p), "counters": {}} for p in probes]
    ours = ("addrms_k_", "stream_probe_kernel", "row_probe_kernel")
    for i, names in enumerate(passes):
        outdir = os.path.join(tmp, f"pass{i}")
        cmd = [rocprof, "--pmc", *names, "--output-format", "csv", "-d", outdir, "-o", "sig", "--",
               sys.executable, "-m", "paper_2601_12698_amd.signals", "--child", spec_path]
        r = subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                           timeout=timeout_s)
        if r.returncode != 0:
            raise RuntimeError(f"rocprofv3 pass {names} failed ({r.returncode}):\n{r.stdout[-2000:]}")
        rows = [x for x in _read_counter_csv(outdir) if any(tag in x["Kernel_Name"] for tag in ours)]
        by_counter: Dict[str, List[float]] = {}
        for x in rows:
            by_counter.setdefault(x["Counter_Name"], []).append(float(x["Counter_Value"]))
        for name, vals in by_counter.items():
            if len(vals) != LAUNCHES_PER_CFG * len(records):
                raise RuntimeError(f"{name}: expected {LAUNCHES_PER_CFG * len(records)} dispatches, saw {len(vals)}")
            for j in range(len(records)):
                chunk = vals[j * LAUNCHES_PER_CFG + 1:(j + 1) * LAUNCHES_PER_CFG]
                records[j]["counters"][name] = sum(chunk) / len(chunk)
    from . import workloads as W
    nbytes = W.algorithmic_bytes(M, N, dtype)     # plain formula; the orchestrator does not load the HIP library
    for rec in records:
        c = rec["counters"]
        d = {}
        if "FETCH_SIZE" in c and "WRITE_SIZE" in c:
            d["hbm_read_bytes"] = c["FETCH_SIZE"] * FETCH_UNIT_BYTES
            d["hbm_write_bytes"] = c["WRITE_SIZE"] * WRITE_UNIT_BYTES
            d["traffic_over_algorithmic"] = (d["hbm_read_bytes"] + d["hbm_write_bytes"]) / nbytes
        if "TCC_HIT_sum" in c and "TCC_MISS_sum" in c and c["TCC_HIT_sum"] + c["TCC_MISS_sum"] > 0:
            d["l2_hit_rate"] = c["TCC_HIT_sum"] / (c["TCC_HIT_sum"] + c["TCC_MISS_sum"])
        if "TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum" in c and c.get("TCC_MISS_sum", 0) > 0:
            d["dram_credit_stall_per_l2_miss"] = c["TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum"] / c["TCC_MISS_sum"]
        rec["derived"] = d
    if workdir is None:
        shutil.rmtree(tmp, ignore_errors=True)
    return records


def collect_probe(M: int, N: int, dtype: str, counters: Sequence[str] = ("FETCH_SIZE", "WRITE_SIZE"),
                  workdir: Optional[str] = None, timeout_s: int = 180) -> Dict[str, float]:
    """Mean counter values per launch of the calibration kernel (reads and writes back x and residual of the
    shape, nothing else), one profiler run per counter; the first launch is discarded."""
    rocprof = shutil.which("rocprofv3")
    if rocprof is None:
        raise RuntimeError("rocprofv3 is not on PATH")
    tmp = workdir or tempfile.mkdtemp(prefix="addrms_probe_")
    os.makedirs(tmp, exist_ok=True)
    spec_path = os.path.join(tmp, "probe_spec.json")
    with open(spec_path, "w") as f:
        json.dump({"M": M, "N": N, "dtype": dtype, "launches": LAUNCHES_PER_CFG + 2}, f)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ)
    env["PYTHONPATH"] = root + os.pathsep + env.get("PYTHONPATH", "")
    env.setdefault("TMPDIR", "/tmp")
    out = {}
    for i, name in enumerate(counters):
        outdir = os.path.join(tmp, f"probe_pass{i}")
        cmd = [rocprof, "--pmc", name, "--output-format", "csv", "-d", outdir, "-o", "sig", "--",
               sys.executable, "-m", "paper_2601_12698_amd.signals", "--child-probe", spec_path]
        r = subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                           timeout=timeout_s)
        if r.returncode != 0:
            raise RuntimeError(f"rocprofv3 probe pass {name} failed ({r.returncode}):\n{r.stdout[-2000:]}")
        vals = [float(x["Counter_Value"]) for x in _read_counter_csv(outdir)
                if "stream_probe_kernel" in x["Kernel_Name"] and x["Counter_Name"] == name]
        if len(vals) < 2:
            raise RuntimeError(f"{name}: no dispatches of the calibration kernel in the profiler output")
        out[name] = sum(vals[1:]) / len(vals[1:])
    if workdir is None:
        shutil.rmtree(tmp, ignore_errors=True)
    return out


TRAFFIC_WORKLOADS = ("large_prefill", "prefill", "odd_width_5120", "odd_width_2880", "odd_width_1000")
# further cfgs measured beside the tuned and the default one: the aligned-span form on the shape it was built for
TRAFFIC_EXTRA = {"odd_width_1000": (("aligned_span", (4, 128, 8, 0, 2, 98, 0, 0)),),
                 # the cfgs the search returns on the headline shape from run to run (all within a per cent of each other)
                 "large_prefill": (("plateau_a", (8, 448, 1, 0, 1, 34, 6, 0)), ("plateau_b", (8, 448, 1, 0, 2, 34, 0, 0)),
                                   ("plateau_c", (2, 512, 1, 0, 2, 34, 0, 0)), ("plateau_d", (8, 448, 1, 0, 1, 2, 6, 0)))}


def traffic_report(path: str, names: Sequence[str] = TRAFFIC_WORKLOADS) -> List[dict]:
    """HBM traffic per launch of the tuned and the default configuration of each named benchmark workload:
    search (child process), FETCH_SIZE and WRITE_SIZE of both cfgs (one profiler run per counter), the same
    counters on the calibration kernel of known traffic on the same shape (which gives bytes per counter unit),
    written as a table that bench.py reads its `roofline.traffic` from."""
    from . import workloads as W
    rows, lines = [], []
    for name in names:
        wl = (W.LARGE_PREFILL if name == "large_prefill" else W.PREFILL if name == "prefill"
              else W.ODD_WIDTH.with_cols(int(name[10:])))
        r0 = _run_stage(["--stage-tune", str(wl.M), str(wl.N), wl.dtype, "--eps", repr(wl.eps), "--top-k", "1", "--hints", "0"])
        cfgs = [B.make_cfg(**r0["cfg"]), B.make_cfg(**r0["default_cfg"])]
        extra = TRAFFIC_EXTRA.get(name, ())
        cfgs += [B.make_cfg(*t) for _label, t in extra]
        recs = collect(cfgs, wl.M, wl.N, wl.dtype, wl.eps, passes=(("FETCH_SIZE",), ("WRITE_SIZE",)))
        # The plain copy kernel always runs in its symmetric 16-bit form (one aligned 16-byte piece of each stream per
        # lane, whole cache lines per wave): with an fp32 residual beside 16-bit x its two pieces per lane leave the
        # chip as half-line writes, which the write counter then sees as more than the bytes stored.
        probe = collect_probe(wl.M, wl.N, "bf16")
        stream_bytes = wl.M * wl.N * 4                                               # the probe reads and writes this much
        fetch_unit = stream_bytes / probe["FETCH_SIZE"]
        write_unit = stream_bytes / probe["WRITE_SIZE"]
        alg = W.algorithmic_bytes(wl.M, wl.N, wl.dtype)
        measured = [("tuned", cfgs[0], recs[0], r0["us"]), ("default", cfgs[1], recs[1], r0["default_us"])]
        measured += [(label, cfgs[2 + i], recs[2 + i], float("nan")) for i, (label, _t) in enumerate(extra)]
        for which, cfg, rec, us in measured:
            rd = rec["counters"]["FETCH_SIZE"] * fetch_unit
            wr = rec["counters"]["WRITE_SIZE"] * write_unit
            row = {"workload": wl.name, "which": which, "cfg": cfg.as_tuple(), "read_bytes": rd, "write_bytes": wr,
                   "total_bytes": rd + wr, "algorithmic_bytes": alg, "ratio": (rd + wr) / alg, "us": us,
                   "fetch_units": rec["counters"]["FETCH_SIZE"], "write_units": rec["counters"]["WRITE_SIZE"],
                   "fetch_unit_bytes": fetch_unit, "write_unit_bytes": write_unit}
            rows.append(row)
            lines.append("| %s | %s | %s | %d | %d | %d | %d | %.5f | %.2f | %.1f | %.1f | %.2f | %.2f |" % (
                wl.name, which, ",".join(str(v) for v in cfg.as_tuple()), round(rd), round(wr), round(rd + wr), alg,
                (rd + wr) / alg, us, rec["counters"]["FETCH_SIZE"], rec["counters"]["WRITE_SIZE"], fetch_unit, write_unit))
    with open(path, "w") as f:
        f.write("# HBM traffic per launch of addrms: profiler counters scaled by a kernel of known traffic (MI355X)\n\n"
                "Command (no GPU work happens in the orchestrating process; searches and profiled launches run in child\n"
                "processes, one `rocprofv3 --pmc <counter>` run per counter and per kernel kind):\n\n"
                "    python -m paper_2601_12698_amd.signals --traffic-report profiles/addrms_hbm_traffic.md\n\n"
                "Per workload: guided search, then FETCH_SIZE and WRITE_SIZE (mean of three launches after one discarded,\n"
                "three rotating buffer sets) of the tuned and the default cfg, and of the library's calibration kernel (a plain\n"
                "copy kernel: 16-bit x and residual of the same M x N, read and written back once, 4*M*N bytes each way): that\n"
                "fixes the bytes per counter unit (last two columns; the counters' nominal units are 2 KiB and 1 KiB here).  cfg = vec, threads_per_row, rows_per_wg, reduce, unroll, flags, max_waves_per_simd, walk.\n"
                "Rows other than `tuned` and `default` are further cfgs of interest: `plateau_*` are cfgs the search returns on the\n"
                "headline shape from run to run (all within a per cent of each other), `aligned_span` is the form built for rows\n"
                "that are not whole cache lines.  bench.py takes `roofline.traffic` from the `total bytes` column of the row whose\n"
                "cfg is the one it timed, else of the `tuned` row of its workload.\n\n"
                "| workload | which | cfg | read bytes | written bytes | total bytes | algorithmic bytes | total / algorithmic | us (search) | FETCH_SIZE | WRITE_SIZE | bytes per FETCH unit | bytes per WRITE unit |\n"
                "|---|---|---|---|---|---|---|---|---|---|---|---|---|\n" + "\n".join(lines) + "\n")
    return rows


HBM_PEAK_BYTES_PER_S = 8.0e12


def suggest(record: dict, achieved_frac: Optional[float] = None) -> Tuple[int, List[str]]:
    """Signals of one configuration (plus, if known, the fraction of the HBM roofline
    its measured time corresponds to) -> (hint bits for the next search, reasons)."""
    c, d = record.get("counters", {}), record.get("derived", {})
    hints, why = 0, []
    occ = c.get("MeanOccupancyPerCU")
    valu = c.get("VALUBusy")
    stall_per_miss = d.get("dram_credit_stall_per_l2_miss")
    two_pass = bool(int(record.get("cfg", {}).get("flags", 0)) & B.FLAG_TWO_PASS)
    if d.get("traffic_over_algorithmic", 1.0) > 1.05 and two_pass:
        why.append(f"HBM traffic is {d['traffic_over_algorithmic']:.2f}x the algorithmic bytes, as expected of the two-pass "
                   "form (rows beyond the register cache are read twice): no hint")
    elif d.get("traffic_over_algorithmic", 1.0) > 1.05:
        hints |= B.HINT_FEWER_LARGER_WORKGROUPS
        why.append(f"HBM traffic is {d['traffic_over_algorithmic']:.2f}x the algorithmic bytes: something is re-read; "
                   "prefer shapes that keep a row in one workgroup's registers")
    if valu is not None and valu > 70.0:
        hints |= B.HINT_WIDER_VECTORS
        why.append(f"VALU busy {valu:.0f}%: instruction-bound; wider vectors amortise address and control work")
    saturated = (achieved_frac is not None and achieved_frac >= 0.6 and (valu is None or valu < 60.0)
                 and (occ is None or occ >= 16.0) and (stall_per_miss is None or stall_per_miss > 0.005))
    if saturated:
        hints |= B.HINT_LOWER_OCCUPANCY
        why.append(f"{100 * achieved_frac:.0f}% of the HBM roofline with VALU busy {valu if valu is not None else float('nan'):.0f}%, "
                   f"{occ if occ is not None else float('nan'):.0f} waves per CU resident and "
                   f"{stall_per_miss if stall_per_miss is not None else float('nan'):.3f} DRAM credit stalls per L2 miss: the memory "
                   "system is saturated; fewer requests in flight may raise mixed read/write DRAM efficiency")
    if achieved_frac is not None and achieved_frac < 0.4 and (valu is None or valu < 40.0):
        hints |= B.HINT_HIGHER_OCCUPANCY
        why.append(f"only {100 * achieved_frac:.0f}% of the HBM roofline and VALU busy "
                   f"{valu if valu is not None else float('nan'):.0f}%: latency-bound; more waves or more loads in flight "
                   "per wave should help")
    return hints, why


def _run_stage(args: List[str], timeout_s: int = 600) -> dict:
    """Run one GPU stage of this module in a child process and return its JSON result."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ)
    env["PYTHONPATH"] = root + os.pathsep + env.get("PYTHONPATH", "")
    r = subprocess.run([sys.executable, "-m", "paper_2601_12698_amd.signals", *args], env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=timeout_s)
    if r.returncode != 0:
        raise RuntimeError(f"stage {args} failed ({r.returncode}):\n{r.stderr[-2000:]}")
    return json.loads(r.stdout.strip().splitlines()[-1])


def stage_tune(M: int, N: int, dtype: str, eps: float, hints: int, log_path: Optional[str], top_k: int) -> dict:
    """(child process) One search; prints the winner and the Top-K as JSON."""
    cfg, rep = B.addrms_tune(M, N, dtype, B.make_budget(eps=eps, log_path=log_path, hints=hints))
    return {"cfg": cfg.as_dict(), "default_cfg": rep.default_cfg.as_dict(), "us": rep.best_us, "default_us": rep.default_us,
            "n_measured": rep.n_measured,
            "wall_ms": rep.wall_ms,
            "topk": [{"cfg": rep.topk[i].as_dict(), "us": rep.topk_us[i]} for i in range(min(top_k, rep.n_topk))]}


def stage_table(M: int, N: int, dtype: str, cfg: dict, us: float, path: str) -> dict:
    """(child process) Merge one entry into a table file."""
    if os.path.exists(path):
        B.addrms_table_load(path)
    B.addrms_table_insert(M, N, dtype, B.make_cfg(**cfg), us)
    B.addrms_table_save(path)
    return {"entries": B.addrms_table_size()}


def tune_with_signals(M: int, N: int, dtype: str, eps: float = 1e-6, log_path: Optional[str] = None,
                      top_k: int = 3, table_path: Optional[str] = None) -> dict:
    """Two rounds of Level 2 with counter feedback in between (runs GPU work in child processes)."""
    def log(obj):
        if log_path:
            with open(log_path, "a") as f:
                f.write(json.dumps(obj) + "\n")

    base = ["--stage-tune", str(M), str(N), dtype, "--eps", repr(eps), "--top-k", str(top_k)]
    if log_path:
        base += ["--log", log_path]
    r0 = _run_stage(base + ["--hints", "0"])
    top = [B.make_cfg(**t["cfg"]) for t in r0["topk"]]
    records = collect(top, M, N, dtype, eps)
    for r in records:
        log({"event": "signals", **r})
    from . import workloads as W
    frac = W.algorithmic_bytes(M, N, dtype) / (r0["us"] * 1e-6) / HBM_PEAK_BYTES_PER_S
    hints, why = suggest(records[0], frac)
    log({"event": "suggest", "achieved_frac": frac, "hints": hints, "reasons": why})
    result = {"round0": r0, "signals": records, "hints": hints, "reasons": why, "best": r0["cfg"], "best_us": r0["us"]}
    if hints:
        r1 = _run_stage(base + ["--hints", str(hints)])
        result["round1"] = r1
        if r1["us"] < r0["us"]:
            result["best"], result["best_us"] = r1["cfg"], r1["us"]
    if table_path:
        _run_stage(["--stage-table", str(M), str(N), dtype, "--cfg-json", json.dumps(result["best"]),
                    "--us", repr(result["best_us"]), "--table", table_path])
    log({"event": "rounds_end", "best": result["best"], "best_us": result["best_us"]})
    return result


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--child", default=None, help="(internal) run the launches of a spec file")
    ap.add_argument("--child-probe", default=None, help="(internal) run the calibration kernel of a spec file")
    ap.add_argument("--traffic-report", default=None, metavar="PATH",
                    help="measure HBM traffic of the tuned and default cfgs of the benchmark workloads and write the table")
    ap.add_argument("--counters", nargs=3, metavar=("M", "N", "DTYPE"), default=None,
                    help="collect the default counter passes for the cfgs given with --cfgs and print one JSON record each")
    ap.add_argument("--cfgs", default=None,
                    help="semicolon-separated cfgs for --counters: vec,threads_per_row,rows_per_wg,reduce,unroll,flags,cap,walk")
    ap.add_argument("--probes", default=None,
                    help="calibration kernels to count beside the cfgs of --counters: 'copy' and/or 'rows:THREADS,WGS_PER_CU', "
                         "semicolon-separated")
    ap.add_argument("--stage-tune", nargs=3, metavar=("M", "N", "DTYPE"), default=None,
                    help="(internal) run one search in this process and print its result as JSON")
    ap.add_argument("--stage-table", nargs=3, metavar=("M", "N", "DTYPE"), default=None,
                    help="(internal) merge --cfg-json/--us into --table")
    ap.add_argument("--cfg-json", default=None)
    ap.add_argument("--us", type=float, default=0.0)
    ap.add_argument("--shape", nargs=3, metavar=("M", "N", "DTYPE"), help="tune this shape with counter feedback")
    ap.add_argument("--eps", type=float, default=1e-6)
    ap.add_argument("--hints", type=int, default=0)
    ap.add_argument("--top-k", type=int, default=3)
    ap.add_argument("--log", default=None)
    ap.add_argument("--table", default=None, help="merge the winner into this table file")
    a = ap.parse_args(argv)
    if a.child:
        return child_main(a.child)
    if a.child_probe:
        return child_probe_main(a.child_probe)
    if a.counters:
        cfgs = [B.make_cfg(*[int(v) for v in t.split(",")]) for t in (a.cfgs or "").split(";") if t.strip()]
        if not cfgs:
            ap.error("--counters needs --cfgs")
        m, n, dt = a.counters
        for j, rec in enumerate(collect(cfgs, int(m), int(n), dt, a.eps, probes=parse_probes(a.probes))):
            what = {"cfg": list(cfgs[j].as_tuple())} if j < len(cfgs) else {"probe": rec["probe"]}
            print(json.dumps({**what, "counters": {k: round(v, 3) for k, v in rec["counters"].items()},
                              "derived": {k: round(v, 5) for k, v in rec["derived"].items()}}))
        return 0
    if a.traffic_report:
        for row in traffic_report(a.traffic_report):
            print(json.dumps(row))
        return 0
    if a.stage_tune:
        m, n, dt = a.stage_tune
        print(json.dumps(stage_tune(int(m), int(n), dt, a.eps, a.hints, a.log, a.top_k)))
        return 0
    if a.stage_table:
        m, n, dt = a.stage_table
        print(json.dumps(stage_table(int(m), int(n), dt, json.loads(a.cfg_json), a.us, a.table)))
        return 0
    if a.shape:
        res = tune_with_signals(int(a.shape[0]), int(a.shape[1]), a.shape[2], eps=a.eps, log_path=a.log,
                                top_k=a.top_k, table_path=a.table)
        print(json.dumps(res, indent=1))
        return 0
    ap.print_help()
    return 2


if __name__ == "__main__":
    sys.exit(main())
