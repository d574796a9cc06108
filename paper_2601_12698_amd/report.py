"""Tuned-versus-default report over the benchmark configurations (needs an MI355X).

    python -m paper_2601_12698_amd.report [--exhaustive-prefill] [--table PATH]

For every configuration it runs the library's guided search (the paper's Level 2:
feasible region, search, Top-K re-test), then prints one markdown row with the
four forms the measurement plan asks for: absolute GB/s and tokens/s, fraction
of the 8 TB/s HBM roofline, default versus tuned configuration, and what the
search cost (wall time, candidates timed).  The calibration kernel (same traffic,
no arithmetic) is timed beside each shape as the attainable ceiling.  The
specialised table built on the way can be saved with --table.

All compute runs in libaddrms.so; this module only loops over shapes and formats text.
"""
from __future__ import annotations

import argparse
import sys
import time

import torch

from . import binding as B
from . import workloads as W

HBM_PEAK_GBPS = 8000.0
# (m, n) shape lists of the paper's evaluation (Section 4, Kernels): plain shape tuples
PAPER_MN_16BIT = [(16, 4096), (32, 5120), (32, 8192), (16, 12288), (64, 8192)]
PAPER_MN_FP32 = [(128, 4096), (256, 4096), (1024, 4096), (2048, 8192), (128, 11008), (256, 13824), (512, 14336),
                 (1024, 8192)]


def shapes():
    yield W.SMOKE
    yield W.PREFILL
    for m in W.DECODE_M:
        yield W.DECODE.with_rows(m)
    yield W.LARGE_PREFILL
    for n in W.ODD_WIDTH_N:
        yield W.ODD_WIDTH.with_cols(n)


class _Shape:
    def __init__(self, M, N, dtype):
        self.M, self.N, self.dtype = M, N, dtype


def probes_us(wl, reps=50):
    """Mean times of the two calibration kernels over rotated buffers: the plain copy (0 if the shape does not meet
    its 16-byte granularity) and the best row-holding copy over workgroup sizes and occupancy caps, as
    (us, threads per row, workgroups per CU) or None where a row is not whole 16-byte pieces or is too long.
    Buffers are carved from one pool the way the tuner's harness and bench.py lay theirs out: 64 KiB-aligned, the
    residual skewed by 4 KiB against x."""
    xb, rb = W.x_bytes(wl.dtype), W.r_bytes(wl.dtype)
    if (wl.M * wl.N * xb) % 16:
        return 0.0, None
    nx, nr = wl.M * wl.N * xb, wl.M * wl.N * rb
    align, skew = 1 << 16, 4096

    def up(v):
        return (v + align - 1) // align * align

    stride = up(nx) + up(nr) + 2 * align
    nsets = int(max(2, min(32, -(-4 * (288 << 20) // (nx + nr)))))
    pool = torch.zeros(stride * nsets + align, dtype=torch.uint8, device="cuda")
    base = (-pool.data_ptr()) % align
    xt, rt = W.x_torch_dtype(wl.dtype), W.r_torch_dtype(wl.dtype)
    xs = [pool[base + i * stride: base + i * stride + nx].view(xt) for i in range(nsets)]
    rs = [pool[base + i * stride + up(nx) + skew: base + i * stride + up(nx) + skew + nr].view(rt)
          for i in range(nsets)]

    def timed(launch, warm, n):
        for i in range(warm):
            launch(xs[i % nsets], rs[i % nsets])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            launch(xs[i % nsets], rs[i % nsets])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n

    plain = timed(lambda x, r: B.addrms_stream_probe(x, r, wl.M, wl.N, wl.dtype), 10, reps)
    best = None
    if (wl.N * xb) % 16 == 0:
        pieces = wl.N * xb // 16
        for t in sorted({min(1024, -(-(-(-pieces // c)) // 64) * 64) for c in (1, 2, 3, 4, 6, 8, 12, 16)}):
            chunks = -(-pieces // t)
            if chunks > 16 or (chunks - 1) * t >= pieces:
                continue
            for wgs in (1, 2, 3, 4, 6, 8, 12, 16):
                if wgs * t > 2048:
                    continue
                us = timed(lambda x, r: B.addrms_row_probe(x, r, wl.M, wl.N, wl.dtype, t, wgs), 3, max(6, reps // 4))
                if best is None or us < best[0]:
                    best = (us, t, wgs)
        if best is not None:
            best = (timed(lambda x, r: B.addrms_row_probe(x, r, wl.M, wl.N, wl.dtype, best[1], best[2]), 5, reps),
                    best[1], best[2])
    return plain, best


def _row_cell(best, moved):
    return "-" if best is None else f"{moved / best[0] * 1e-3:.0f} ({best[1]} x {best[2]})"


def _eager_and_graph_us(issue, chain, laps):
    """Per-launch time of the `chain` launches that issue() makes: issued one by one from the host, and replayed
    from a captured HIP graph."""
    def timed(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(laps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (laps * chain)

    eager = timed(issue)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        issue()
    torch.cuda.synchronize()
    return eager, timed(g.replay)


def graph_vs_eager_us(wl, cfg, chain=64, laps=20, nsets=8):
    """Per-launch time of `chain` back-to-back launches (rotating over `nsets` buffer pairs):
    issued one by one from the host, and replayed from a captured HIP graph."""
    dev = torch.device("cuda")
    d = W.generate(wl)
    w = d["w"].to(dev)
    xs = [d["x"].to(dev) for _ in range(nsets)]
    rs = [d["r"].to(dev) for _ in range(nsets)]

    def issue():
        for i in range(chain):
            B.addrms_run(xs[i % nsets], rs[i % nsets], w, wl.eps, wl.M, wl.N, wl.dtype, cfg)

    return _eager_and_graph_us(issue, chain, laps)


def launch_floor_us(chain=64, laps=20):
    """What a launch costs when the kernel has next to nothing to do: the calibration copy on 16 bytes of each
    stream (one workgroup, one active lane), chained and timed like the decode shapes."""
    x = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    r = torch.zeros(8, dtype=torch.bfloat16, device="cuda")

    def issue():
        for _ in range(chain):
            B.addrms_stream_probe(x, r, 1, 8, "bf16")

    return _eager_and_graph_us(issue, chain, laps)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--exhaustive-prefill", action="store_true",
                    help="also run the exhaustive search on the prefill shape and report the guided search's regret")
    ap.add_argument("--exhaustive-large", action="store_true",
                    help="the same on the large prefill shape (33,000 cfgs at about 50 ms each: half an hour)")
    ap.add_argument("--exhaustive-odd", action="store_true",
                    help="the same on the three odd-width mixed-precision shapes (a quarter of an hour)")
    ap.add_argument("--exhaustive-decode", action="store_true",
                    help="the same on the nine decode shapes (launch-bound: their times move by a few per cent by themselves)")
    ap.add_argument("--exhaustive-others", action="store_true",
                    help="the same for silu_and_mul (4096 x 11008) and merge_attn_states (768 x 32 x 256), bf16")
    ap.add_argument("--exhaustive-log", default=None,
                    help="log of the exhaustive searches; a later run with the same file takes what it holds and measures the rest")
    ap.add_argument("--exhaustive-wall-ms", type=float, default=0.0,
                    help="time limit of one exhaustive search (0: none); with a log, several limited runs add up to a whole one")
    ap.add_argument("--table", default=None, help="save the specialised table here")
    ap.add_argument("--silumul", action="store_true",
                    help="also tune silu_and_mul (the second kernel behind the same tuner) on three shapes")
    ap.add_argument("--mergestates", action="store_true",
                    help="also tune merge_attn_states (third kernel) on the (n, h, d) shapes of the paper's evaluation")
    ap.add_argument("--paper-shapes", action="store_true",
                    help="also select one general cfg over the (m, n) shape lists the paper evaluates on "
                         "(Section 4: five fp16/bf16 shapes, eight fp32 shapes) and print general vs specialised")
    ap.add_argument("--long-rows", action="store_true",
                    help="also tune rows beyond the register row cache (cache continued in LDS, hybrid or two-pass form)")
    ap.add_argument("--graph-decode", action="store_true",
                    help="decode shapes: per-launch time of a chain of launches issued eagerly vs replayed from a HIP graph")
    ap.add_argument("--row-scan", action="store_true",
                    help="time against the number of rows for N = 1000, 1024 and 5120 (fp16 x, fp32 residual) and N = 4096 (bf16): "
                         "separates the fixed cost of a launch from the per-row rate, and rows that are whole cache lines from "
                         "rows that are not")
    ap.add_argument("--width-scan", action="store_true",
                    help="tuned rate against the row length at constant traffic (1.9 GB, bf16): what holding longer rows costs")
    ap.add_argument("--only", action="store_true", help="skip the main table; print only the sections asked for")
    ap.add_argument("--audit-large", action="store_true",
                    help="the audit on the large prefill shape instead (several minutes)")
    ap.add_argument("--audit", action="store_true",
                    help="time what the deriver's efficiency rules prune beside what they retain (three shapes)")
    a = ap.parse_args(argv)
    if not torch.cuda.is_available():
        print("needs a GPU", file=sys.stderr)
        return 2
    B.addrms_table_clear()
    if not a.only:
        print("| workload | M x N | default us | tuned us | speedup | tuned GB/s | % of 8 TB/s | tokens/s | copy GB/s | "
              "row-holding copy GB/s (threads x workgroups per CU) | "
              "tuned cfg (vec, threads/row, rows/wg, reduce, unroll, flags, cap, walk) | feasible | timed | search ms |")
        print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    for wl in ([] if a.only else shapes()):
        nbytes = B.addrms_algorithmic_bytes(wl.M, wl.N, wl.dtype)
        t0 = time.perf_counter()
        cfg, rep = B.addrms_tune(wl.M, wl.N, wl.dtype, B.make_budget(eps=wl.eps))
        wall = (time.perf_counter() - t0) * 1e3
        p, rowp = probes_us(wl)
        moved = 2 * wl.M * wl.N * (W.x_bytes(wl.dtype) + W.r_bytes(wl.dtype))
        gbps = nbytes / rep.best_us * 1e-3
        print(f"| {wl.name} | {wl.M} x {wl.N} | {rep.default_us:.2f} | {rep.best_us:.2f} | "
              f"{rep.default_us / rep.best_us:.3f} | {gbps:.0f} | {100 * gbps / HBM_PEAK_GBPS:.1f} | "
              f"{wl.M / rep.best_us * 1e6:.3g} | {(moved / p * 1e-3) if p else float('nan'):.0f} | {_row_cell(rowp, moved)} | "
              f"{cfg.as_tuple()} | {rep.n_feasible} | {rep.n_measured} | {wall:.0f} |", flush=True)
    regret_shapes = [(a.exhaustive_prefill, W.PREFILL, "prefill"), (a.exhaustive_large, W.LARGE_PREFILL, "large prefill")]
    regret_shapes += [(a.exhaustive_odd, W.ODD_WIDTH.with_cols(n), f"odd width N={n}") for n in W.ODD_WIDTH_N]
    regret_shapes += [(a.exhaustive_decode, W.DECODE.with_rows(m), f"decode M={m}") for m in W.DECODE_M]
    for asked, wl, label in regret_shapes:
        if not asked:
            continue
        g, grep = B.addrms_tune(wl.M, wl.N, wl.dtype, B.make_budget(eps=wl.eps))
        e, erep = B.addrms_tune(wl.M, wl.N, wl.dtype, B.make_budget(eps=wl.eps, strategy=B.SEARCH_EXHAUSTIVE,
                                                                    log_path=a.exhaustive_log, max_wall_ms=a.exhaustive_wall_ms))
        if erep.n_measured + erep.n_failed + erep.n_resumed < erep.n_feasible:
            print(f"\n{label}: the exhaustive search stopped at its time limit after {erep.n_measured + erep.n_resumed} of "
                  f"{erep.n_feasible} cfgs ({erep.n_resumed} of them taken from the log); run again with the same log to go on",
                  flush=True)
            continue
        tgs, tes = [], []
        for _ in range(5):                      # alternating, so that drift after the long search hits both alike
            tgs.append(B.addrms_measure(g, wl.M, wl.N, wl.dtype))
            tes.append(B.addrms_measure(e, wl.M, wl.N, wl.dtype))
        tg, te = sorted(tgs)[2], sorted(tes)[2]
        print(f"\n{label}: guided {g.as_tuple()} after {grep.n_measured} cfgs / {grep.wall_ms:.0f} ms; "
              f"exhaustive {e.as_tuple()} after {erep.n_measured} cfgs / {erep.wall_ms:.0f} ms"
              f"{f' (and {erep.n_resumed} taken from the log of earlier runs)' if erep.n_resumed else ''}.  "
              f"Confirmed inside their own searches (2 x (20 + 100) launches): {grep.best_us:.2f} us against {erep.best_us:.2f} us, "
              f"regret {grep.best_us / erep.best_us:.4f}; measured afterwards in alternation on newly allocated buffers "
              f"(median of 5 each): {tg:.2f} us against {te:.2f} us, regret {tg / te:.4f}", flush=True)
    if a.exhaustive_others:
        # the two further operators: the same search code, so the same question
        for label, tune, measure, dims, dt in (
                ("silu_and_mul 4096 x 11008", B.silumul_tune, B.silumul_measure, (W.SILU_PREFILL.M, W.SILU_PREFILL.d), W.SILU_PREFILL.dtype),
                ("merge_attn_states 768 x 32 x 256", B.mergestates_tune, B.mergestates_measure, (768 * 32, 256), "bf16")):
            g, grep = tune(*dims, dt, B.make_budget())
            e, erep = tune(*dims, dt, B.make_budget(strategy=B.SEARCH_EXHAUSTIVE))
            tgs, tes = [], []
            for _ in range(5):
                tgs.append(measure(g, *dims, dt))
                tes.append(measure(e, *dims, dt))
            tg, te = sorted(tgs)[2], sorted(tes)[2]
            print(f"\n{label} bf16: guided {g.as_tuple()} after {grep.n_measured} cfgs / {grep.wall_ms:.0f} ms; "
                  f"exhaustive {e.as_tuple()} after {erep.n_measured} cfgs / {erep.wall_ms:.0f} ms.  Confirmed inside their own "
                  f"searches: {grep.best_us:.2f} us against {erep.best_us:.2f} us, regret {grep.best_us / erep.best_us:.4f}; "
                  f"measured afterwards in alternation (median of 5 each): {tg:.2f} us against {te:.2f} us, regret "
                  f"{tg / te:.4f}", flush=True)
    if a.silumul:
        print("\nsilu_and_mul (out[i,j] = silu(x[i,j]) * x[i,d+j]), tuned vs default:\n")
        print("| workload | M x d | default us | tuned us | speedup | tuned GB/s | % of 8 TB/s | tuned cfg | feasible | timed | search ms |")
        print("|---|---|---|---|---|---|---|---|---|---|---|")
        # the last shape is eight times the prefill one (2.2 GB per launch): what the kernel streams at once the
        # fixed cost of a launch no longer shows
        big = W.GatedWorkload("silu_32768x11008_bf16", 32768, 11008, "bf16", 14)
        for wl in (W.SILU_PREFILL, W.SILU_DECODE, W.SILU_FP16, big):
            nbytes = B.silumul_algorithmic_bytes(wl.M, wl.d, wl.dtype)
            t0 = time.perf_counter()
            cfg, rep = B.silumul_tune(wl.M, wl.d, wl.dtype, B.make_budget())
            wall = (time.perf_counter() - t0) * 1e3
            gbps = nbytes / rep.best_us * 1e-3
            print(f"| {wl.name} | {wl.M} x {wl.d} | {rep.default_us:.2f} | {rep.best_us:.2f} | "
                  f"{rep.default_us / rep.best_us:.3f} | {gbps:.0f} | {100 * gbps / HBM_PEAK_GBPS:.1f} | {cfg.as_tuple()} | "
                  f"{rep.n_feasible} | {rep.n_measured} | {wall:.0f} |", flush=True)
    if a.mergestates:
        print("\nmerge_attn_states (log-sum-exp merge of two partial attention states), tuned vs default:\n")
        print("| n x h x d | dtype | default us | tuned us | speedup | tuned GB/s | tuned cfg | feasible | timed | search ms |")
        print("|---|---|---|---|---|---|---|---|---|---|")
        for dtype in ("bf16", "fp16"):
            for n, h, d in W.MERGE_SHAPES:
                rows = n * h
                nbytes = B.mergestates_algorithmic_bytes(rows, d, dtype)
                t0 = time.perf_counter()
                cfg, rep = B.mergestates_tune(rows, d, dtype, B.make_budget())
                wall = (time.perf_counter() - t0) * 1e3
                print(f"| {n} x {h} x {d} | {dtype} | {rep.default_us:.2f} | {rep.best_us:.2f} | "
                      f"{rep.default_us / rep.best_us:.3f} | {nbytes / rep.best_us * 1e-3:.0f} | {cfg.as_tuple()} | "
                      f"{rep.n_feasible} | {rep.n_measured} | {wall:.0f} |", flush=True)
    if a.paper_shapes:
        # the paper's (m, n) lists, and the decode sweep of the benchmark configurations read the same way: one cfg for
        # all nine M against one cfg per M (Section 4, the finding that no single configuration suits every shape)
        decode = [(m, W.DECODE.N) for m in W.DECODE_M]
        for dtype, shape_list, what in (("bf16", PAPER_MN_16BIT, ""), ("fp16", PAPER_MN_16BIT, ""), ("fp32", PAPER_MN_FP32, ""),
                                        (W.DECODE.dtype, decode, "decode sweep, ")):
            g, rep = B.addrms_select_general(shape_list, dtype, B.make_budget(eps=W.DECODE.eps if what else 0.0))
            print(f"\n{what}{dtype}: general cfg {g.as_tuple()}: geomean speedup over default x{rep.geomean_speedup_general:.3f} "
                  f"(arithmetic mean x{rep.mean_speedup_general:.3f}); specialised table x{rep.geomean_speedup_specialized:.3f}; "
                  f"{rep.n_pool} universally feasible candidates timed; {rep.wall_ms:.0f} ms\n")
            print("| m x n | default us | general us | specialised us | general speedup | specialised speedup | specialised cfg |")
            print("|---|---|---|---|---|---|---|")
            for i, (m, n) in enumerate(shape_list):
                print(f"| {m} x {n} | {rep.default_us[i]:.2f} | {rep.general_us[i]:.2f} | {rep.specialized_us[i]:.2f} | "
                      f"{rep.default_us[i] / rep.general_us[i]:.3f} | {rep.default_us[i] / rep.specialized_us[i]:.3f} | "
                      f"{rep.specialized[i].as_tuple()} |", flush=True)
    if a.long_rows:
        print("\nRows beyond the register row cache (flags 16: cache continued in LDS, one pass; flags 8: two passes; flags 24: "
              "hybrid, only what fits neither registers nor LDS is read twice), tuned vs default:\n")
        print("| M x N | dtype | default us | tuned us | speedup | tuned GB/s (algorithmic) | % of 8 TB/s | copy GB/s | "
              "row-holding copy GB/s (threads x workgroups per CU) | tuned cfg | feasible | timed | search ms |")
        print("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
        for M, N, dtype in ((4096, 40960, "bf16"), (2048, 65536, "bf16"), (1024, 131072, "bf16"),
                            (2048, 49152, "fp16_res32"), (512, 262144, "fp32")):
            nbytes = B.addrms_algorithmic_bytes(M, N, dtype)
            t0 = time.perf_counter()
            cfg, rep = B.addrms_tune(M, N, dtype, B.make_budget())
            wall = (time.perf_counter() - t0) * 1e3
            gbps = nbytes / rep.best_us * 1e-3
            p, rowp = probes_us(_Shape(M, N, dtype), reps=24)
            moved = 2 * M * N * (W.x_bytes(dtype) + W.r_bytes(dtype))
            print(f"| {M} x {N} | {dtype} | {rep.default_us:.1f} | {rep.best_us:.1f} | {rep.default_us / rep.best_us:.3f} | "
                  f"{gbps:.0f} | {100 * gbps / HBM_PEAK_GBPS:.1f} | {moved / p * 1e-3:.0f} | {_row_cell(rowp, moved)} | {cfg.as_tuple()} | {rep.n_feasible} | {rep.n_measured} | "
                  f"{wall:.0f} |", flush=True)
    if a.width_scan:
        total, dt = 32768 * 7168, "bf16"
        print("\nTuned rate against the row length at constant traffic (M x N = 32768 x 7168 elements, bf16):\n")
        print("| M x N | default us | tuned us | % of 8 TB/s | copy % | row-holding copy % (threads x workgroups per CU) | tuned cfg |")
        print("|---|---|---|---|---|---|---|")
        for N in (512, 1024, 2048, 3584, 4096, 7168, 8192, 14336, 16384, 28672, 32768):
            M = total // N
            nbytes = B.addrms_algorithmic_bytes(M, N, dt)
            cfg, rep = B.addrms_tune(M, N, dt, B.make_budget())
            p, rowp = probes_us(_Shape(M, N, dt), reps=24)
            moved = 2 * M * N * (W.x_bytes(dt) + W.r_bytes(dt))
            row_cell = "-" if rowp is None else f"{moved / rowp[0] * 1e-3 / HBM_PEAK_GBPS * 100:.1f} ({rowp[1]} x {rowp[2]})"
            print(f"| {M} x {N} | {rep.default_us:.1f} | {rep.best_us:.1f} | "
                  f"{nbytes / rep.best_us * 1e-3 / HBM_PEAK_GBPS * 100:.1f} | {moved / p * 1e-3 / HBM_PEAK_GBPS * 100:.1f} | "
                  f"{row_cell} | {cfg.as_tuple()} |", flush=True)
    if a.row_scan:
        print("\nTime against the number of rows (tuned per shape): t = t0 + M * slope by least squares; t0 is what a launch "
              "costs before any row streams, bytes per row / slope the rate the rows stream at:\n")
        print("| N | storage | M | tuned us | GB/s | % of 8 TB/s | tuned cfg |")
        print("|---|---|---|---|---|---|---|")
        for N, dt, ms in ((1000, "fp16_res32", (8192, 16384, 32768, 65536)), (1024, "fp16_res32", (8192, 16384, 32768, 65536)),
                          (4096, "bf16", (4096, 8192, 16384, 32768)), (5120, "fp16_res32", (8192, 16384, 32768, 65536))):
            pts = []
            for M in ms:
                nbytes = B.addrms_algorithmic_bytes(M, N, dt)
                cfg, rep = B.addrms_tune(M, N, dt, B.make_budget())
                pts.append((M, rep.best_us))
                print(f"| {N} | {dt} | {M} | {rep.best_us:.2f} | {nbytes / rep.best_us * 1e-3:.0f} | "
                      f"{nbytes / rep.best_us * 1e-3 / HBM_PEAK_GBPS * 100:.1f} | {cfg.as_tuple()} |", flush=True)
            n = len(pts)
            sx, sy = sum(p[0] for p in pts), sum(p[1] for p in pts)
            sxx, sxy = sum(p[0] * p[0] for p in pts), sum(p[0] * p[1] for p in pts)
            slope = (n * sxy - sx * sy) / (n * sxx - sx * sx)
            t0 = (sy - slope * sx) / n
            row_bytes = 2 * N * (W.x_bytes(dt) + W.r_bytes(dt))
            print(f"| {N} | {dt} | fit | t0 = {t0:.2f} us | {row_bytes / slope * 1e-3:.0f} GB/s asymptotic | "
                  f"{row_bytes / slope * 1e-3 / HBM_PEAK_GBPS * 100:.1f} | slope {slope * 1e3:.3f} ns per row |", flush=True)
    if a.graph_decode:
        print("\nDecode shapes, chain of 64 launches, tuned cfg: microseconds per launch issued eagerly vs from a HIP graph:\n")
        print("| M x N | cfg | eager us | graph us |")
        print("|---|---|---|---|")
        for m in W.DECODE_M:
            wl = W.DECODE.with_rows(m)
            cfg = B.addrms_table_lookup(wl.M, wl.N, wl.dtype) or B.addrms_default_cfg(wl.N, wl.dtype)
            eager, graph = graph_vs_eager_us(wl, cfg)
            print(f"| {wl.M} x {wl.N} | {cfg.as_tuple()} | {eager:.2f} | {graph:.2f} |", flush=True)
        eager, graph = launch_floor_us()
        print(f"| launch floor | (copy kernel on 16 bytes of each stream) | {eager:.2f} | {graph:.2f} |", flush=True)
    if a.audit or a.audit_large:
        print("\nAudit of the efficiency rules (every cfg gated and timed, 3 + 15 launches):\n")
        print("| M x N | dtype | retained | best us | decile us | median us | rule | pruned | failed gate | best us | "
              "median us | in top decile | beating best | s |")
        print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
        shapes_audited = [(2048, 1000, "fp16_res32", 0), (4096, 4096, "bf16", 0), (1024, 11008, "fp32", 0)]
        if a.audit_large:       # the retained region in full (33,000 cfgs), 300 sampled cfgs of each pruned class
            shapes_audited = [(W.LARGE_PREFILL.M, W.LARGE_PREFILL.N, W.LARGE_PREFILL.dtype, 300)]
        for M, N, dtype, cap in shapes_audited:
            rep = B.addrms_audit_rules(M, N, dtype, B.make_budget(max_candidates=cap))
            for r in rep.rules:
                if r.n_pruned:
                    print(f"| {M} x {N} | {dtype} | {rep.n_retained} | {rep.retained_best_us:.2f} | "
                          f"{rep.retained_decile_us:.2f} | {rep.retained_median_us:.2f} | {r.rule.decode()} | {r.n_pruned} | "
                          f"{r.n_failed} | {r.best_us:.2f} | {r.median_us:.2f} | {r.n_in_top_decile} | {r.n_beating_best} | "
                          f"{rep.wall_ms / 1e3:.1f} |", flush=True)
    if a.paper_shapes:
        def general_table(title, select, shapes, dtype, label):
            g, rep = select(shapes, dtype, B.make_budget())
            print(f"\n{title} {dtype}: general cfg {g.as_tuple()}: geomean speedup over default x{rep.geomean_speedup_general:.3f}; "
                  f"specialised table x{rep.geomean_speedup_specialized:.3f}; {rep.n_pool} universally feasible candidates "
                  f"timed; {rep.wall_ms:.0f} ms\n")
            print(f"| {label} | default us | general us | specialised us | general speedup | specialised speedup | specialised cfg |")
            print("|---|---|---|---|---|---|---|")
            for i, sh in enumerate(shapes):
                print(f"| {sh[0]} x {sh[1]} | {rep.default_us[i]:.2f} | {rep.general_us[i]:.2f} | {rep.specialized_us[i]:.2f} | "
                      f"{rep.default_us[i] / rep.general_us[i]:.3f} | {rep.default_us[i] / rep.specialized_us[i]:.3f} | "
                      f"{rep.specialized[i].as_tuple()} |", flush=True)

        merge_shapes = [(n * h, d) for n, h, d in W.MERGE_SHAPES]
        for dtype in ("bf16", "fp16"):
            general_table("merge_attn_states on the (n, h, d) shapes of Section 4 (rows = n*h),", B.mergestates_select_general,
                          merge_shapes, dtype, "rows x d")
        general_table("silu_and_mul on the fp32 (m, n) shapes of Section 4 (d = n),", B.silumul_select_general,
                      PAPER_MN_FP32, "fp32", "m x d")
        general_table("silu_and_mul on the 16-bit (m, n) shapes of Section 4 (d = n),", B.silumul_select_general,
                      PAPER_MN_16BIT, "bf16", "m x d")
    if a.table:
        B.addrms_table_save(a.table)
    return 0


if __name__ == "__main__":
    sys.exit(main())
