"""Parity of the HIP path with the CPU oracle, through the C ABI (needs an MI355X).

Bar: residual output bit-exact; normalised output within 1 unit in the last
place of its storage format AND within 2e-2 absolute.  Because both sides
form the sum of squares in fp64 and round rstd to fp32 once, the outputs are
expected to be identical; the few-ulp allowance only covers the (about 1e-7
per row) chance that the two fp64 summation orders straddle an fp32 rounding
boundary of rstd.
"""
import math

import numpy as np
import pytest
import torch

from gpu_util import DeviceCase, compare, oracle_outputs
from paper_2601_12698_amd import binding as B
from paper_2601_12698_amd import workloads as W

pytestmark = pytest.mark.gpu


def _wl(M, N, dtype, seed, eps=1e-6, **kw):
    return W.Workload(f"t_{M}x{N}_{dtype}", M, N, dtype, eps, seed, **kw)


def test_smoke_shape_default_cfg(oracle):
    wl = W.SMOKE
    d = W.generate(wl)
    case = DeviceCase(d, wl)
    y, res = case.run(None)
    y_ref, res_ref = oracle_outputs(oracle, d, wl)
    st = compare(y, res, y_ref, res_ref, wl.dtype, wl.name)
    assert st["n_diff"] == 0


# Small shapes that still span several chunks, ragged row tails (N not a
# multiple of vec*threads) and a ragged last workgroup (M not a multiple of
# rows_per_wg).
SMALL = [
    ("bf16", 37, 4096, 0), ("bf16", 5, 8192, 1), ("bf16", 70, 7168, 2),
    ("fp16", 19, 1000, 3), ("fp16_res32", 21, 2880, 4), ("fp16_res32", 9, 5120, 5),
    ("fp16_res32", 33, 1000, 6), ("fp32", 13, 1536, 7), ("fp32", 3, 11008, 8), ("bf16", 130, 512, 9),
]


@pytest.mark.parametrize("dtype,M,N,seed", SMALL)
def test_every_feasible_cfg_matches_oracle(oracle, dtype, M, N, seed):
    wl = _wl(M, N, dtype, seed, x_std=1.3, r_std=0.9)
    d = W.generate(wl)
    case = DeviceCase(d, wl)
    y_ref, res_ref = oracle_outputs(oracle, d, wl)
    cfgs, grid = B.addrms_enumerate_feasible(M, N, dtype)
    assert len(cfgs) > 50
    print(f"{wl.name}: {len(cfgs)} feasible of {grid}", flush=True)
    total_diff = 0
    # occupancy-capped variants run the same kernel with more LDS: cover every uncapped cfg, a third of the capped
    cfgs = [c for i, c in enumerate(cfgs) if c.max_waves_per_simd == 0 or i % 3 == 0]
    for c in cfgs:
        y, res = case.run(c)
        st = compare(y, res, y_ref, res_ref, dtype, f"{wl.name} {c}")
        total_diff += st["n_diff"]
    # identical everywhere is the expectation, across all configurations
    assert total_diff == 0


def test_results_do_not_depend_on_cfg_and_are_repeatable(oracle):
    wl = _wl(257, 4096, "bf16", 21)
    d = W.generate(wl)
    case = DeviceCase(d, wl)
    cfgs, _ = B.addrms_enumerate_feasible(wl.M, wl.N, wl.dtype)
    y0, r0 = case.run(cfgs[0])
    for c in cfgs[:: max(1, len(cfgs) // 40)]:
        for _ in range(2):
            y, r = case.run(c)
            assert np.array_equal(y, y0) and np.array_equal(r, r0), str(c)


@pytest.mark.parametrize("N", [8, 24, 1001, 333, 2050])
def test_narrow_and_odd_widths(oracle, N):
    """Widths that force narrow vectors (odd N needs vec=1) and rows shorter than a wave."""
    for dtype in ("bf16", "fp16_res32"):
        wl = _wl(11, N, dtype, 30 + N)
        d = W.generate(wl)
        case = DeviceCase(d, wl)
        y_ref, res_ref = oracle_outputs(oracle, d, wl)
        cfgs, _ = B.addrms_enumerate_feasible(wl.M, N, dtype)
        assert cfgs, f"no feasible cfg for N={N}"
        for c in [None] + cfgs[::7]:
            y, res = case.run(c)
            assert compare(y, res, y_ref, res_ref, dtype, f"N={N} {c}")["n_diff"] == 0


@pytest.mark.parametrize("dtype,M,N", [("bf16", 3, 32768), ("fp32", 2, 32768), ("fp16", 3, 32766),
                                       ("bf16", 2, 16383), ("fp16_res32", 5, 28672)])
def test_widest_rows_the_template_covers(oracle, dtype, M, N):
    """The register row cache bounds N: even N up to 32768, odd N up to 16384.  Every
    feasible cfg at the bound is checked (there are few), the default included."""
    wl = _wl(M, N, dtype, 900 + N % 97)
    d = W.generate(wl)
    case = DeviceCase(d, wl)
    y_ref, res_ref = oracle_outputs(oracle, d, wl)
    cfgs, _ = B.addrms_enumerate_feasible(M, N, dtype)
    assert cfgs
    print(f"{wl.name}: {len(cfgs)} feasible", flush=True)
    for c in [None] + cfgs[:: max(1, len(cfgs) // 60)]:
        y, res = case.run(c)
        assert compare(y, res, y_ref, res_ref, dtype, f"{wl.name} {c}")["n_diff"] == 0


def test_rows_beyond_the_template_are_refused_before_launch():
    """Rows longer than 2^28 elements have no configuration: the call fails before anything is launched."""
    N, dtype = (1 << 28) + 8, "bf16"
    x = torch.full((N * 2,), 0x3C, dtype=torch.uint8, device="cuda")
    r = torch.full((N * 2,), 0x3C, dtype=torch.uint8, device="cuda")
    w = torch.zeros(N * 2, dtype=torch.uint8, device="cuda")
    st = B.load().addrms_run(x.data_ptr(), r.data_ptr(), w.data_ptr(), 1e-6, 1, N, B._dtype_id(dtype), None, None)
    assert st == B.ERR_UNSUPPORTED_SHAPE, B.addrms_last_error()
    torch.cuda.synchronize()
    assert bool((x == 0x3C).all()) and bool((r == 0x3C).all())


@pytest.mark.parametrize("dtype,M,N", [("bf16", 5, 32770), ("bf16", 3, 65536), ("fp16", 4, 40001), ("fp16_res32", 3, 49152),
                                       ("fp32", 2, 100000), ("bf16", 37, 36864), ("fp32", 1, 1 << 20), ("bf16", 7, 20001),
                                       ("fp32", 6, 32767), ("bf16", 3, 73720), ("bf16", 5, 131072), ("fp16_res32", 3, 99992),
                                       ("fp16", 2, 262146)])
def test_long_row_forms_beyond_the_register_cache(oracle, dtype, M, N):
    """Rows that no plain single-pass configuration holds run with the row cache continued in LDS (one pass)
    while 160 KB suffice; beyond that in the hybrid form (registers and LDS hold what they can, the rest of the row
    is read twice) or the plain two-pass form (read, sum, read again, write).  Same arithmetic, same bar:
    bit-identical to the oracle over a spread of the configurations of each form."""
    long_forms = B.FLAG_TWO_PASS | B.FLAG_LDS_CACHE
    wl = _wl(M, N, dtype, 1200 + N % 89)
    d = W.generate(wl)
    case = DeviceCase(d, wl)
    y_ref, res_ref = oracle_outputs(oracle, d, wl)
    dflt = B.addrms_default_cfg(N, dtype)
    assert dflt.flags & long_forms
    cfgs, _ = B.addrms_enumerate_feasible(M, N, dtype)
    assert cfgs and all(c.flags & long_forms for c in cfgs)
    by_form = {f: [c for c in cfgs if c.flags & long_forms == f] for f in (B.FLAG_TWO_PASS, B.FLAG_LDS_CACHE, long_forms)}
    print(f"{wl.name}: two-pass {len(by_form[B.FLAG_TWO_PASS])}, lds-cache {len(by_form[B.FLAG_LDS_CACHE])}, hybrid "
          f"{len(by_form[long_forms])} feasible, default {dflt.as_tuple()}", flush=True)
    if N > 80000:
        assert by_form[long_forms] and dflt.flags & long_forms == long_forms
    picks = [None]
    for lst in by_form.values():
        picks += lst[:: max(1, len(lst) // 50)]
    # the instances with the larger register cache (workgroups of at most 512 threads) are configurations like any other;
    # make sure a spread of them is among the picks wherever the deriver offers them
    big = [c for c in cfgs if c.threads_per_row * c.rows_per_wg <= 512 and c.flags & B.FLAG_LDS_CACHE
           and B.addrms_cfg_feasible(c, M, N, dtype)[2].max_threads == 512]
    picks += big[:: max(1, len(big) // 30)]
    if dtype != "fp32" and N % 4 == 0 and N >= 98304:
        assert big
    print(f"   {len(big)} of them on the 144-value instances; {len(picks)} cfgs run", flush=True)
    for c in picks:
        y, res = case.run(c)
        assert compare(y, res, y_ref, res_ref, dtype, f"{wl.name} {c}")["n_diff"] == 0


def test_degenerate_rows(oracle):
    """Zero rows, signed zeros, rounding ties, subnormal sums, large magnitudes."""
    N = 1024
    wl = _wl(8, N, "bf16", 40)
    d = W.generate(wl)
    x = d["x"].clone()
    r = d["r"].clone()
    x[0].zero_(); r[0].zero_()                                   # zero row: rstd = 1/sqrt(eps)
    x[1] = -0.0; r[1] = 0.0                                      # (-0) + (+0) = +0
    x[2] = -0.0; r[2] = -0.0                                     # stays -0
    x[3] = 1.0; r[3] = 2.0 ** -8                                 # exact tie in bf16: rounds to even
    x[4] = 1.0; r[4] = 3 * 2.0 ** -8                             # tie the other way
    x[5] = 2.0 ** -120; r[5] = 2.0 ** -127                       # subnormal fp32 partial sums
    x[6] = 1e18; r[6] = -3e17                                    # large finite values (h^2 ~ 1e36)
    x[7, ::2] = 0.0                                              # half zeros
    d2 = {"x": x.contiguous(), "r": r.contiguous(), "w": d["w"]}
    case = DeviceCase(d2, wl)
    y_ref, res_ref = oracle_outputs(oracle, d2, wl)
    cfgs, _ = B.addrms_enumerate_feasible(wl.M, N, "bf16")
    for c in [None] + cfgs[::11]:
        y, res = case.run(c)
        assert compare(y, res, y_ref, res_ref, "bf16", f"degenerate {c}")["n_diff"] == 0
    assert np.all(res_ref[0] == 0) and np.all(y_ref[0] == 0)


def test_fp16_ties_and_subnormal_outputs(oracle):
    N = 512
    wl = _wl(4, N, "fp16", 41, eps=1e-6)
    d = W.generate(wl)
    x = d["x"].clone(); r = d["r"].clone()
    x[0] = 1.0; r[0] = 2.0 ** -11                                # tie in fp16
    x[1] = 2.0 ** -14; r[1] = 2.0 ** -24                         # sums near the fp16 subnormal boundary
    x[2, :] = 0.0; x[2, 0] = 6e-5; r[2] = 0.0                    # y has fp16-subnormal entries? (others 0)
    d2 = {"x": x.contiguous(), "r": r.contiguous(), "w": d["w"]}
    case = DeviceCase(d2, wl)
    y_ref, res_ref = oracle_outputs(oracle, d2, wl)
    cfgs, _ = B.addrms_enumerate_feasible(wl.M, N, "fp16")
    for c in [None] + cfgs[::13]:
        y, res = case.run(c)
        assert compare(y, res, y_ref, res_ref, "fp16", f"fp16 edge {c}")["n_diff"] == 0


def test_rstd_probe_matches_oracle(oracle):
    rng = np.random.default_rng(50)
    for N, eps in ((4096, 1e-6), (7168, 1e-6), (1000, 1e-5), (8192, 1e-5)):
        ss = np.concatenate([np.exp(rng.uniform(-30, 40, 200000)), rng.uniform(0.5, 2.0, 100000) * N,
                             np.array([0.0, 1e-300, 1e300])])
        ss_d = torch.from_numpy(ss).cuda()
        out = torch.empty(ss.size, dtype=torch.float32, device="cuda")
        B.addrms_rstd_probe(ss_d, N, eps, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        want = np.array([oracle.rstd_canonical(float(v), N, eps) for v in ss[:5000]], dtype=np.float32)
        assert np.array_equal(got[:5000], want)
        # vectorised check of the rest with numpy fp64 (same formula, correctly rounded ops)
        want_all = (1.0 / np.sqrt(ss / N + np.float64(np.float32(eps)))).astype(np.float32)
        assert np.array_equal(got, want_all)


def test_m_zero_is_noop_and_m_one_works(oracle):
    wl = _wl(1, 8192, "bf16", 60, eps=1e-5, x_std=2.0, r_std=2.0)
    d = W.generate(wl)
    case = DeviceCase(d, wl)
    y_ref, res_ref = oracle_outputs(oracle, d, wl)
    cfgs, _ = B.addrms_enumerate_feasible(1, 8192, "bf16")
    for c in [None] + cfgs[::5]:
        y, res = case.run(c)
        assert compare(y, res, y_ref, res_ref, "bf16", f"M=1 {c}")["n_diff"] == 0
    x = case.x0.clone(); r = case.r0.clone()
    B.load().addrms_run(x.data_ptr(), r.data_ptr(), case.w.data_ptr(), 1e-5, 0, 8192, B.BF16, None, None)
    torch.cuda.synchronize()
    assert torch.equal(x, case.x0) and torch.equal(r, case.r0)


def test_argument_errors_launch_nothing():
    wl = _wl(4, 4096, "bf16", 61)
    d = W.generate(wl)
    case = DeviceCase(d, wl)
    case.x.copy_(case.x0); case.r.copy_(case.r0)
    lib = B.load()
    xp, rp, wp = case.x.data_ptr(), case.r.data_ptr(), case.w.data_ptr()
    bad = B.make_cfg(8, 1024, 1)                                  # half the lanes idle: pruned
    assert lib.addrms_run(xp, rp, wp, 1e-6, 4, 4096, B.BF16, bad, None) == B.ERR_INFEASIBLE_CFG
    assert "lane slots" in B.addrms_last_error()
    ok = B.make_cfg(8, 256, 1, unroll=2)
    assert lib.addrms_run(xp + 2, rp, wp, 1e-6, 4, 4096, B.BF16, ok, None) == B.ERR_MISALIGNED
    assert lib.addrms_run(xp, rp + 4, wp, 1e-6, 4, 4096, B.BF16, ok, None) == B.ERR_MISALIGNED
    assert lib.addrms_run(None, rp, wp, 1e-6, 4, 4096, B.BF16, ok, None) == B.ERR_INVALID_ARG
    assert lib.addrms_run(xp, rp, wp, 1e-6, 4, 0, B.BF16, ok, None) == B.ERR_INVALID_ARG
    assert lib.addrms_run(xp, rp, wp, 1e-6, -1, 4096, B.BF16, ok, None) == B.ERR_INVALID_ARG
    assert lib.addrms_run(xp, rp, wp, 1e-6, 4, 4096, 9, ok, None) == B.ERR_UNSUPPORTED_DTYPE
    assert lib.addrms_run(xp, rp, wp, 1e-6, 4, 4100, B.BF16, ok, None) == B.ERR_INFEASIBLE_CFG   # 8 does not divide 4100
    torch.cuda.synchronize()
    assert torch.equal(case.x, case.x0) and torch.equal(case.r, case.r0)


def test_runs_on_a_side_stream(oracle):
    wl = _wl(64, 4096, "bf16", 62)
    d = W.generate(wl)
    case = DeviceCase(d, wl)
    y_ref, res_ref = oracle_outputs(oracle, d, wl)
    s = torch.cuda.Stream()
    case.x.copy_(case.x0); case.r.copy_(case.r0)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        B.addrms_run(case.x, case.r, case.w, wl.eps, wl.M, wl.N, wl.dtype, None, stream=s)
    s.synchronize()
    st = compare(W.to_bits(case.x), W.to_bits(case.r), y_ref, res_ref, "bf16", "side stream")
    assert st["n_diff"] == 0, st


def _run_raw(x, r, w, eps, dtype, cfg=None):
    M, N = x.shape
    xd, rd, wd = x.cuda(), r.cuda(), w.cuda()
    B.addrms_run(xd, rd, wd, eps, M, N, dtype, cfg)
    torch.cuda.synchronize()
    return W.to_bits(xd), W.to_bits(rd)


def test_exact_invariants_hold_on_the_device():
    """Properties that hold at any size, checked on the device output itself: row
    permutation, negation, power-of-two scaling (with eps scaled by 4^k)."""
    wl = _wl(3000, 4096, "bf16", 70)
    d = W.generate(wl)
    x, r, w = d["x"], d["r"], d["w"]
    eps = 2.0 ** -20
    y0, r0 = _run_raw(x, r, w, eps, "bf16")
    perm = torch.randperm(wl.M, generator=torch.Generator().manual_seed(1))
    y1, r1 = _run_raw(x[perm].contiguous(), r[perm].contiguous(), w, eps, "bf16", B.make_cfg(8, 512, 2, flags=2))
    assert np.array_equal(y1, y0[perm.numpy()]) and np.array_equal(r1, r0[perm.numpy()])
    # negation flips every sign, except where x + r cancels exactly: a + (-a) is +0 either way
    nz = (r0 & 0x7fff) != 0
    assert (~nz).sum() < 0.01 * nz.size
    y2, r2 = _run_raw(-x, -r, w, eps, "bf16")
    assert np.array_equal((y2 ^ np.uint16(0x8000))[nz], y0[nz]) and np.array_equal((r2 ^ np.uint16(0x8000))[nz], r0[nz])
    assert np.all(r2[~nz] == 0) and np.all(r0[~nz] == 0) and np.all((y2[~nz] & 0x7fff) == 0)
    # scale by 2^k: y unchanged, residual scaled (zeros excluded: 0 * 2^k keeps its pattern)
    k = 5
    y3, r3 = _run_raw(x * 2.0 ** k, r * 2.0 ** k, w, eps * 4.0 ** k, "bf16")
    assert np.array_equal(y3, y0)
    assert np.array_equal(r3[nz], (r0 + np.uint16(k << 7))[nz])


def test_run_is_reentrant_across_host_threads(oracle):
    """Four host threads, each with its own stream, shape, storage format and cfg, call
    addrms_run (and the error path) concurrently; every result must match the oracle."""
    import threading

    jobs = [(_wl(257, 4096, "bf16", 81), None), (_wl(64, 8192, "fp16", 82), B.make_cfg(8, 512, 2, flags=2)),
            (_wl(500, 1000, "fp16_res32", 83), B.make_cfg(4, 128, 2, unroll=2)), (_wl(33, 5120, "fp32", 84), None)]
    prepared = []
    for wl, cfg in jobs:
        d = W.generate(wl)
        prepared.append((wl, cfg, DeviceCase(d, wl), oracle_outputs(oracle, d, wl), torch.cuda.Stream()))
    torch.cuda.synchronize()
    errors = []

    def worker(wl, cfg, case, stream):
        try:
            lib = B.load()
            for _ in range(50):
                with torch.cuda.stream(stream):
                    case.x.copy_(case.x0, non_blocking=True)
                    case.r.copy_(case.r0, non_blocking=True)
                    B.addrms_run(case.x, case.r, case.w, wl.eps, wl.M, wl.N, wl.dtype, cfg, stream=stream)
                # an argument error on this thread must not disturb the others (thread-local message)
                st = lib.addrms_run(None, None, None, 1e-6, 1, wl.N, B.DTYPE_IDS[wl.dtype], None, None)
                if st != B.ERR_INVALID_ARG or "NULL" not in B.addrms_last_error():
                    errors.append(f"{wl.name}: error path returned {st}: {B.addrms_last_error()}")
            stream.synchronize()
        except Exception as e:                      # noqa: BLE001 - reported below
            errors.append(f"{wl.name}: {e!r}")

    threads = [threading.Thread(target=worker, args=(wl, cfg, case, s)) for wl, cfg, case, _, s in prepared]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for wl, cfg, case, (y_ref, res_ref), _ in prepared:
        st = compare(W.to_bits(case.x), W.to_bits(case.r), y_ref, res_ref, wl.dtype, f"threaded {wl.name}")
        assert st["n_diff"] == 0


def test_random_shapes_and_cfgs(oracle):
    """Seeded random sweep: row lengths of every parity class (odd, 2, 4, 8 mod 16, ...), row counts that
    leave ragged last workgroups, all four storage formats; per shape the default and six random feasible cfgs."""
    rng = np.random.default_rng(20260112)
    n_cases = 0
    for k in range(48):
        dtype = W.DTYPES[k % 4]
        N = int(rng.choice([rng.integers(8, 200), rng.integers(200, 3000), 8 * rng.integers(64, 1200),
                            rng.integers(3000, 12000)]))
        M = int(rng.integers(1, 70))
        try:
            B.addrms_default_cfg(N, dtype)
        except B.AddrmsError:
            continue
        cfgs, _ = B.addrms_enumerate_feasible(M, N, dtype)
        assert cfgs, (M, N, dtype)
        wl = _wl(M, N, dtype, 1000 + k, x_std=float(rng.choice([0.01, 1.0, 30.0])), r_std=float(rng.choice([0.5, 2.0])))
        d = W.generate(wl)
        case = DeviceCase(d, wl)
        y_ref, res_ref = oracle_outputs(oracle, d, wl)
        picks = [None] + [cfgs[int(i)] for i in rng.integers(0, len(cfgs), 6)]
        for c in picks:
            y, res = case.run(c)
            assert compare(y, res, y_ref, res_ref, dtype, f"{wl.name} {c}")["n_diff"] == 0
            n_cases += 1
    assert n_cases > 250


@pytest.mark.parametrize("dtype,N,off", [("bf16", 1001, 1), ("bf16", 1002, 2), ("fp16", 2052, 4), ("fp16_res32", 1004, 4),
                                         ("fp32", 1001, 1), ("fp32", 1002, 2)])
def test_bases_aligned_only_to_the_vector(oracle, dtype, N, off):
    """Tensors that start `off` elements into an allocation: the base is aligned to the widest vector that
    divides N (which is what the cfg needs) and to nothing more."""
    M = 9
    wl = _wl(M, N, dtype, 1300 + N)
    d = W.generate(wl)
    y_ref, res_ref = oracle_outputs(oracle, d, wl)
    dev = torch.device("cuda:0")

    def shifted(t):
        big = torch.zeros(t.numel() + 64, dtype=t.dtype, device=dev)
        view = big[off:off + t.numel()]
        view.copy_(t.reshape(-1).to(dev))
        return big, view

    keep_x, x = shifted(d["x"])
    keep_r, r = shifted(d["r"])
    keep_w, w = shifted(d["w"])
    vec = B.addrms_default_cfg(N, dtype).vec
    assert x.data_ptr() % (vec * W.x_bytes(dtype)) == 0 and x.data_ptr() % (2 * vec * W.x_bytes(dtype)) != 0
    cfgs, _ = B.addrms_enumerate_feasible(M, N, dtype)
    for c in [None] + [c for c in cfgs if c.vec <= vec][::23]:
        x.copy_(d["x"].reshape(-1).to(dev))
        r.copy_(d["r"].reshape(-1).to(dev))
        B.addrms_run(x, r, w, wl.eps, M, N, dtype, c)
        torch.cuda.synchronize()
        got_y, got_r = W.to_bits(x.view(M, N)), W.to_bits(r.view(M, N))
        assert compare(got_y, got_r, y_ref, res_ref, dtype, f"{wl.name} off={off} {c}")["n_diff"] == 0
    # nothing outside the views was touched
    assert float(keep_x[:off].abs().sum()) == 0 and float(keep_x[off + M * N:].abs().sum()) == 0
    assert float(keep_r[:off].abs().sum()) == 0 and float(keep_r[off + M * N:].abs().sum()) == 0


@pytest.mark.parametrize("dtype,M,N", [("bf16", 1_000_003, 40), ("fp16_res32", 300_001, 24), ("fp32", 500_009, 12)])
def test_a_million_short_rows(oracle, dtype, M, N):
    """Rows shorter than a wave, a prime number of them: sub-wave row shapes, many row blocks, ragged last block."""
    wl = _wl(M, N, dtype, 1400 + N)
    d = W.generate(wl)
    case = DeviceCase(d, wl)
    y_ref, res_ref = oracle_outputs(oracle, d, wl)
    cfgs, _ = B.addrms_enumerate_feasible(M, N, dtype)
    assert cfgs
    for c in [None] + cfgs[:: max(1, len(cfgs) // 12)]:
        y, res = case.run(c)
        assert compare(y, res, y_ref, res_ref, dtype, f"{wl.name} {c}")["n_diff"] == 0
