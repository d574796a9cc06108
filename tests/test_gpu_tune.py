"""The tuner on the device (needs an MI355X): deriver model against the device's
own resource report, guided search against exhaustive search, the correctness
gate, the table, and the measurement harness."""
import json

import numpy as np
import pytest
import torch

from paper_2601_12698_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def clean_table():
    B.addrms_table_clear()
    yield
    B.addrms_table_clear()


@pytest.mark.parametrize("M,N,dtype", [(4096, 4096, "bf16"), (8192, 1000, "fp16_res32"), (512, 14336, "fp32"),
                                       (64, 8192, "bf16"), (64, 49152, "bf16"), (16, 131072, "bf16")])
def test_deriver_model_matches_device(M, N, dtype):
    """Registers, LDS, workgroup bound and resident workgroups per CU predicted by
    the host-side deriver equal what the HIP runtime reports for the loaded kernels."""
    cfgs, _ = B.addrms_enumerate_feasible(M, N, dtype)
    if N == 131072:      # this row brings in the long-row instances compiled for at most 512 threads
        assert any(B.addrms_cfg_feasible(c, M, N, dtype)[2].max_threads == 512 for c in cfgs[::5])
    for c in cfgs[::5]:
        st, _, model = B.addrms_cfg_feasible(c, M, N, dtype)
        dev = B.addrms_device_resources(c, M, N, dtype)
        assert st == 0
        assert model.vgprs + model.agprs == dev.vgprs, c
        assert dev.scratch_bytes == 0, c
        assert model.lds_bytes == dev.lds_bytes, c
        assert model.max_threads == dev.max_threads, c
        assert model.wgs_per_cu == dev.wgs_per_cu, (c, model.as_dict(), dev.as_dict())


def test_guided_close_to_exhaustive_on_prefill(tmp_path):
    M, N, dt = 4096, 4096, "bf16"
    log = str(tmp_path / "guided.jsonl")
    g, grep = B.addrms_tune(M, N, dt, B.make_budget(log_path=log))
    e, erep = B.addrms_tune(M, N, dt, B.make_budget(strategy=B.SEARCH_EXHAUSTIVE, warmup=5, reps=30))
    assert grep.n_failed == 0 and erep.n_failed == 0            # every candidate passed the gate
    assert erep.n_measured == erep.n_feasible
    assert grep.n_measured <= 0.1 * grep.n_feasible
    # re-measure both winners back to back with the confirmation protocol
    tg = min(B.addrms_measure(g, M, N, dt) for _ in range(3))
    te = min(B.addrms_measure(e, M, N, dt) for _ in range(3))
    td = min(B.addrms_measure(B.addrms_default_cfg(N, dt), M, N, dt) for _ in range(3))
    print(f"guided {g} {tg:.2f} us ({grep.n_measured} cfgs, {grep.wall_ms:.0f} ms); exhaustive {e} {te:.2f} us "
          f"({erep.n_measured} cfgs, {erep.wall_ms:.0f} ms); default {td:.2f} us", flush=True)
    # regret of the guided search: by the times both searches confirmed for their winners (same protocol, each in
    # its own harness) or by the re-measurement above.  The re-measurement alone is not a fair judge on this shape:
    # on buffers allocated after earlier ones were freed, persistent-grid cfgs with one workgroup per CU run up to
    # 6 % slower than on a harness's first allocation, and not all of them by the same amount.
    print(f"confirmed in the searches: guided {grep.best_us:.2f} us, exhaustive {erep.best_us:.2f} us", flush=True)
    assert min(tg / te, grep.best_us / erep.best_us) <= 1.05
    assert tg <= td * 1.01                                       # tuned is not slower than the default
    lines = [json.loads(l) for l in open(log)]
    assert lines[0]["event"] == "begin" and lines[-1]["event"] == "end"
    # the winner went into the table and is what a cfg-less run resolves to
    assert B.addrms_table_lookup(M, N, dt).as_tuple() == e.as_tuple()


def test_gate_passes_every_feasible_candidate():
    """The gate compares each candidate with the default configuration's output; with identical
    arithmetic in every instance nothing may be rejected.  (That the gate does reject what differs is
    shown in test_gpu_gate.py and, for the search's handling of rejections, on the fake backend.)"""
    c, rep = B.addrms_tune(37, 1000, "fp16", B.make_budget(strategy=B.SEARCH_EXHAUSTIVE, warmup=1, reps=3))
    assert rep.n_failed == 0 and rep.n_measured == rep.n_feasible > 100


def test_tune_small_budget_and_errors():
    c, rep = B.addrms_tune(16, 4096, "bf16", B.make_budget(max_candidates=6, warmup=2, reps=10))
    assert rep.n_measured <= 6 and B.addrms_cfg_feasible(c, 16, 4096, "bf16")[0] == 0
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_tune(16, 1 << 30, "bf16")
    assert e.value.status == B.ERR_UNSUPPORTED_SHAPE
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_tune(0, 4096, "bf16")
    assert e.value.status == B.ERR_INVALID_ARG


def test_second_tune_on_the_device_resumes_from_the_log(tmp_path):
    """The log of a device search serves a later one: nothing is gated or screened again, only the Top-K
    confirmation runs, and the winner is confirmed at about the same time."""
    M, N, dt = 64, 8192, "bf16"
    log = str(tmp_path / "tune.jsonl")
    first, rep1 = B.addrms_tune(M, N, dt, B.make_budget(log_path=log))
    assert rep1.n_resumed == 0 and rep1.n_measured > 50 and rep1.n_failed == 0
    B.addrms_table_clear()
    second, rep2 = B.addrms_tune(M, N, dt, B.make_budget(log_path=log))
    assert rep2.n_measured == 0 and rep2.n_resumed == rep1.n_measured
    assert rep2.wall_ms < rep1.wall_ms                      # (setting up the harness and the confirmation remain)
    # same screening times, so the same Top-K; which of them confirms fastest may differ between two runs
    assert second.as_tuple() in {rep1.topk[i].as_tuple() for i in range(rep1.n_topk)} | {rep1.default_cfg.as_tuple()}
    assert rep2.best_us == pytest.approx(rep1.best_us, rel=0.1)
    assert B.addrms_table_lookup(M, N, dt).as_tuple() == second.as_tuple()
    print(f"first {first} {rep1.best_us:.2f} us in {rep1.wall_ms:.0f} ms; resumed {second} {rep2.best_us:.2f} us in "
          f"{rep2.wall_ms:.0f} ms", flush=True)


def test_tune_rows_beyond_the_register_cache():
    """The search runs unchanged over the long-row forms: every candidate passes the gate, the winner is one of
    them, is not slower than the default and is what a cfg-less run resolves to."""
    long_forms = B.FLAG_TWO_PASS | B.FLAG_LDS_CACHE
    for M, N, dt in ((256, 40960, "bf16"), (128, 131072, "bf16")):
        c, rep = B.addrms_tune(M, N, dt, B.make_budget(warmup=5, reps=30))
        assert c.flags & long_forms and rep.n_failed == 0 and 20 < rep.n_measured < 0.1 * rep.n_feasible
        assert rep.default_cfg.flags & long_forms and rep.best_us <= rep.default_us * 1.02
        assert B.addrms_table_lookup(M, N, dt).as_tuple() == c.as_tuple()
        nbytes = B.addrms_algorithmic_bytes(M, N, dt)
        print(f"long rows {M}x{N}: {c} {rep.best_us:.2f} us = {nbytes / rep.best_us * 1e-3:.0f} GB/s; default "
              f"{rep.default_cfg} {rep.default_us:.2f} us", flush=True)


def test_measure_and_stream_probe():
    M, N, dt = 4096, 4096, "bf16"
    d = B.addrms_default_cfg(N, dt)
    cold = B.addrms_measure(d, M, N, dt, rotate=True)
    warm = B.addrms_measure(d, M, N, dt, rotate=False)
    nbytes = B.addrms_algorithmic_bytes(M, N, dt)
    assert 10.0 < warm <= cold * 1.05 < 200.0
    assert nbytes / cold * 1e-3 > 2000.0                         # GB/s: far above anything cache-less code would miss
    x = torch.randn(M, N, device="cuda").to(torch.bfloat16)
    r = torch.randn(M, N, device="cuda").to(torch.bfloat16)
    x0, r0 = x.clone(), r.clone()
    B.addrms_stream_probe(x, r, M, N, dt)
    torch.cuda.synchronize()
    assert torch.equal(x.view(torch.int16), ~x0.view(torch.int16)) and torch.equal(r.view(torch.int16), ~r0.view(torch.int16))


PAPER_MN_16BIT = [(16, 4096), (32, 5120), (32, 8192), (16, 12288), (64, 8192)]
PAPER_MN_FP32 = [(128, 4096), (256, 4096), (1024, 4096), (2048, 8192), (128, 11008), (256, 13824), (512, 14336),
                 (1024, 8192)]


@pytest.mark.parametrize("shapes,dtype", [(PAPER_MN_16BIT, "bf16"), (PAPER_MN_FP32, "fp32")])
def test_select_general_on_paper_shape_lists(shapes, dtype):
    """One general cfg over the (m, n) shape lists the paper evaluates on (Section 4,
    Kernels), and the specialised table built on the way (Algorithm 1 lines 22-23)."""
    budget = B.make_budget(max_candidates=60, warmup=5, reps=30, coarse_reps=8)
    g, rep = B.addrms_select_general(shapes, dtype, budget)
    print(f"{dtype}: general {g} geomean x{rep.geomean_speedup_general:.3f} (mean x{rep.mean_speedup_general:.3f}), "
          f"specialised x{rep.geomean_speedup_specialized:.3f}, pool {rep.n_pool}, {rep.wall_ms:.0f} ms", flush=True)
    for i, (M, N) in enumerate(shapes):
        assert B.addrms_cfg_feasible(g, M, N, dtype)[0] == 0
        assert rep.default_us[i] > 0 and rep.general_us[i] > 0 and rep.specialized_us[i] > 0
        # what a cfg-less run resolves to is what the report calls specialised (also where the general cfg replaced
        # a shape's own winner because it measured faster there)
        assert B.addrms_table_lookup(M, N, dtype).as_tuple() == rep.specialized[i].as_tuple()
    assert rep.geomean_speedup_specialized >= rep.geomean_speedup_general - 1e-9
    assert rep.geomean_speedup_general > 0.97        # the defaults are in the pool when they fit every shape


def test_rounds_on_device(tmp_path):
    """Level-1 rounds on the device: every family passes validation (all instances share
    one arithmetic), the score never gets worse, streaming is the structural gain."""
    log = str(tmp_path / "rounds.jsonl")
    shapes = [(4096, 4096), (2048, 8192)]
    g, rep = B.addrms_tune_rounds(shapes, "bf16", B.make_budget(log_path=log, warmup=5, reps=30))
    print(json.dumps(rep.as_dict()["rounds"]), flush=True)
    assert rep.n_rounds == B.MAX_ROUNDS == 5 and all(rep.rounds[i].passed for i in range(5))
    assert rep.rounds[4].families & B.FAMILY_STORE_PHASE
    scores = [rep.rounds[i].score for i in range(5)]
    assert scores[1] < scores[0] - 0.03            # the non-temporal policy is worth well over 3 %
    assert min(scores) == scores[rep.best_round]
    assert rep.rounds[0].general.flags == 0 and rep.rounds[0].general.max_waves_per_simd == 0
    for M, N in shapes:
        assert B.addrms_table_lookup(M, N, "bf16") is not None


def test_hw_limits_match_the_device():
    """The deriver's r(h) against what the runtime reports for the card."""
    L = B.addrms_get_hw_limits()
    p = torch.cuda.get_device_properties(0)
    assert "gfx950" in p.gcnArchName
    assert L.compute_units == p.multi_processor_count
    assert L.wave_size == p.warp_size
    assert L.max_threads_per_wg == getattr(p, "max_threads_per_block", 1024)
    assert L.max_waves_per_simd * L.simds_per_cu * L.wave_size == p.max_threads_per_multi_processor
    assert p.total_memory > 200 * (1 << 30)                       # 288 GB HBM3E part
    assert L.lds_bytes_per_cu == 160 * 1024
    l2 = getattr(p, "L2_cache_size", None)
    if l2:
        assert l2 == L.l2_bytes_per_xcd


def test_measure_stats():
    M, N, dt = 4096, 4096, "bf16"
    d = B.addrms_default_cfg(N, dt)
    s = B.addrms_measure_stats(d, M, N, dt, warmup=10, reps=60)
    print(s.as_dict(), flush=True)
    assert s.reps == 60 and s.buffer_sets >= 9
    assert 0 < s.min_us <= s.median_us <= s.max_us
    assert s.min_us <= s.per_launch_mean_us <= s.max_us
    # an event pair around each launch can only add to what back-to-back launches cost on average
    assert s.per_launch_mean_us >= 0.9 * s.mean_us
    assert 10.0 < s.mean_us < 100.0
