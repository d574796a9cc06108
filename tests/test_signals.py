"""Host-side logic of the profiling-signal loop (no GPU, no profiler): parsing of the
per-dispatch counter table and the rules that turn signals into search hints."""
import os

import pytest

from paper_2601_12698_amd import binding as B
from paper_2601_12698_amd import signals as S

HEADER = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id",'
          '"Kernel_Name","Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count",'
          '"Counter_Name","Counter_Value","Start_Timestamp","End_Timestamp"\n')


def _row(i, kernel, name, value):
    return f'{i},{i},"Agent 1",1,1,1,1024,1,"{kernel}",256,0,0,32,0,16,"{name}",{value},0,1\n'


def test_counter_csv_is_read_in_dispatch_order(tmp_path):
    d = tmp_path / "pass0" / "host"
    os.makedirs(d)
    with open(d / "123_counter_collection.csv", "w") as f:
        f.write(HEADER)
        f.write(_row(3, "addrms_k_d0_v8_c1_u1_n1", "FETCH_SIZE", 30.0))
        f.write(_row(1, "fill_kernel", "FETCH_SIZE", 1.0))
        f.write(_row(2, "addrms_k_d0_v8_c1_u1_n1", "FETCH_SIZE", 20.0))
    rows = S._read_counter_csv(str(tmp_path / "pass0"))
    assert [int(r["Dispatch_Id"]) for r in rows] == [1, 2, 3]
    assert [r["Kernel_Name"] for r in rows][0] == "fill_kernel"


def test_suggest_rules():
    sat = {"counters": {"VALUBusy": 36.0, "MeanOccupancyPerCU": 24.0},
           "derived": {"traffic_over_algorithmic": 1.0, "dram_credit_stall_per_l2_miss": 0.015}}
    hints, why = S.suggest(sat, achieved_frac=0.78)
    assert hints == B.HINT_LOWER_OCCUPANCY and "saturated" in why[0]
    # the same signals far from the roofline are read as latency-bound, not saturated
    hints, why = S.suggest(sat, achieved_frac=0.25)
    assert hints == B.HINT_HIGHER_OCCUPANCY and "latency-bound" in why[0]
    waste = {"counters": {"VALUBusy": 20.0}, "derived": {"traffic_over_algorithmic": 1.4}}
    hints, why = S.suggest(waste, achieved_frac=0.5)
    assert hints & B.HINT_FEWER_LARGER_WORKGROUPS and "re-read" in why[0]
    alu = {"counters": {"VALUBusy": 85.0, "MeanOccupancyPerCU": 30.0}, "derived": {}}
    hints, why = S.suggest(alu, achieved_frac=0.7)
    assert hints == B.HINT_WIDER_VECTORS
    assert S.suggest({"counters": {}, "derived": {}}, None) == (0, [])


def test_spec_round_trip():
    cfgs = [B.make_cfg(8, 512, 1, flags=2, max_waves_per_simd=6), B.make_cfg(4, 128, 2, unroll=2)]
    spec = S._spec(cfgs, 64, 4096, "bf16", 1e-6)
    back = [B.make_cfg(**d) for d in spec["cfgs"]]
    assert [c.as_tuple() for c in back] == [c.as_tuple() for c in cfgs]
    assert spec["launches"] == S.LAUNCHES_PER_CFG >= 2


def test_hints_reach_the_search():
    """A lower-occupancy hint adds the capped sweep mode (visible in the log phases)."""
    import json
    import tempfile
    import math

    def measure(c, w, r):
        us = 20.0 * (1.0 + 0.02 * abs((c.max_waves_per_simd or 8) - 3)) * (0.9 if c.flags & 2 else 1.0)
        return us * (1.0 + 0.1 * abs(math.log2(c.threads_per_row / 512.0))) * (1.0 + 0.1 * abs(math.log2(c.vec / 8.0)))
    with tempfile.TemporaryDirectory() as d:
        p0, p1 = os.path.join(d, "a.jsonl"), os.path.join(d, "b.jsonl")
        B.addrms_tune_with_backend(4096, 4096, "bf16", B.make_budget(log_path=p0), measure)
        g, rep = B.addrms_tune_with_backend(4096, 4096, "bf16",
                                            B.make_budget(log_path=p1, hints=B.HINT_LOWER_OCCUPANCY), measure)
        ph0 = {json.loads(l).get("phase") for l in open(p0)}
        ph1 = {json.loads(l).get("phase") for l in open(p1)}
    assert "sweep_capped" not in ph0 and "sweep_capped" in ph1
    assert 0 < g.max_waves_per_simd <= 4


def test_two_pass_re_reads_are_not_taken_for_waste():
    rec = {"cfg": {"vec": 8, "threads_per_row": 1024, "rows_per_wg": 1, "reduce": 0, "unroll": 2, "flags": 10,
                   "max_waves_per_simd": 0},
           "counters": {"VALUBusy": 22.0, "MeanOccupancyPerCU": 12.0},
           "derived": {"traffic_over_algorithmic": 1.45}}
    hints, why = S.suggest(rec, achieved_frac=0.6)
    assert hints == 0 and any("two-pass" in w for w in why)
    rec["cfg"]["flags"] = 2
    hints, why = S.suggest(rec, achieved_frac=0.6)
    assert hints & B.HINT_FEWER_LARGER_WORKGROUPS


def test_probe_list_of_the_counters_command():
    assert S.parse_probes(None) == [] and S.parse_probes(" ; ") == []
    assert S.parse_probes("copy;rows:256,6") == [{"kind": "copy"}, {"kind": "rows", "threads": 256, "wgs": 6}]
    with pytest.raises(ValueError):
        S.parse_probes("columns:3")
    spec = S._spec([], 8, 4096, "bf16", 1e-6, S.parse_probes("rows:448,3"))
    assert spec["probes"] == [{"kind": "rows", "threads": 448, "wgs": 3}] and spec["cfgs"] == []


def test_report_and_bench_say_that_they_need_a_gpu(capsys):
    """Neither measures anything without a device, and neither pretends to: no CPU fallback."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2601_12698_amd import report
    assert report.main(["--only", "--width-scan", "--exhaustive-large", "--exhaustive-log", "x.jsonl"]) == 2
    assert "needs a GPU" in capsys.readouterr().err
    import bench
    assert bench.recorded_regret("large prefill")["exhaustive_cfgs"] > 0      # parses the committed profile
    assert bench.recorded_regret()["guided_cfgs"] > 0
    assert bench.measured_traffic("large_prefill_32768x7168_bf16_outliers")["over_algorithmic"] < 1.01
