"""Feasible-region deriver (host logic, no GPU): rules, reasons, counts, the
occupancy model against the compiler's own figure, and the default cfg."""
import re

import pytest

from paper_2601_12698_amd import binding as B


def feas(cfg, M, N, dtype):
    st, why, res = B.addrms_cfg_feasible(cfg, M, N, dtype)
    return st, why, res


def test_known_feasible_and_resources():
    c = B.make_cfg(8, 256, 1, unroll=2)
    st, why, res = feas(c, 4096, 4096, "bf16")
    assert st == 0 and why == ""
    assert res.chunks_per_thread == 2 and res.scratch_bytes == 0
    assert res.waves_per_wg == 4 and res.max_threads == 1024
    assert 16 <= res.vgprs <= 128 and res.lds_bytes == 16 * 8
    assert 1 <= res.waves_per_simd <= 8


KNOWN_INFEASIBLE = [
    (B.make_cfg(3, 256, 1), 4096, 4096, "bf16", "vector width"),
    (B.make_cfg(8, 100, 1), 4096, 4096, "bf16", "threads_per_row"),
    (B.make_cfg(8, 256, 3), 4096, 4096, "bf16", "rows_per_wg"),
    (B.make_cfg(8, 256, 1, reduce=2), 4096, 4096, "bf16", "reduce"),
    (B.make_cfg(8, 256, 1, unroll=3), 4096, 4096, "bf16", "unroll"),
    (B.make_cfg(8, 256, 1, flags=128), 4096, 4096, "bf16", "flags"),
    (B.make_cfg(4, 128, 4, unroll=2, flags=64), 8192, 1000, "fp16_res32", "not whole 128-byte cache lines"),
    (B.make_cfg(4, 256, 4, flags=64), 8192, 1024, "fp16_res32", "whole cache lines already"),
    (B.make_cfg(8, 128, 8, flags=64), 8192, 1000, "fp16_res32", "16-byte pieces"),
    (B.make_cfg(4, 128, 8, reduce=1, unroll=2, flags=64), 8192, 1000, "fp16_res32", "its own segmented reduction"),
    (B.make_cfg(4, 128, 8, unroll=2, flags=64 | 4), 65536, 1000, "fp16_res32", "ordinary grid"),
    (B.make_cfg(4, 32, 16, unroll=2, flags=64), 8192, 1000, "fp16_res32", "exists for 1, 2 and 4"),
    (B.make_cfg(8, 256, 1, unroll=2, flags=8 | 32), 4096, 65536, "bf16", "deferred residual store exists for the register-cached form only"),
    (B.make_cfg(8, 1024, 1, unroll=2, flags=16 | 32), 4096, 40960, "bf16", "deferred residual store exists for the register-cached form only"),
    (B.make_cfg(8, 256, 1, unroll=2, walk=4), 32768, 4096, "bf16", "walk=4 sizes a persistent grid"),
    (B.make_cfg(8, 256, 1, unroll=2, flags=4, walk=3), 32768, 4096, "bf16", "walk=3"),
    (B.make_cfg(8, 256, 1, unroll=2, flags=4, walk=16), 8192, 4096, "bf16", "persistent grid is the ordinary grid"),
    (B.make_cfg(8, 256, 1, unroll=2, flags=4), 1024, 4096, "bf16", "persistent grid is the ordinary grid"),
    (B.make_cfg(8, 256, 1), 4096, 4100, "bf16", "does not divide"),
    (B.make_cfg(8, 256, 1), 4096, 4096, "fp32", "wider than"),
    (B.make_cfg(8, 512, 4), 4096, 4096, "bf16", "exceeds the 1024-thread limit"),
    (B.make_cfg(8, 8, 1), 4096, 64, "bf16", "whole number"),
    (B.make_cfg(8, 32, 2), 4096, 4096, "bf16", "row cache"),
    (B.make_cfg(4, 64, 1), 4096, 2304, "bf16", "no compiled instance"),      # 9 chunks
    (B.make_cfg(8, 1024, 1), 4096, 4096, "bf16", "lane slots"),
    (B.make_cfg(8, 512, 1, unroll=2), 4096, 4096, "bf16", "unroll=2 exceeds"),
    (B.make_cfg(8, 256, 4, unroll=2), 2, 4096, "bf16", "exceeds the 2 rows"),
    (B.make_cfg(8, 256, 1, unroll=2, flags=1), 8, 4096, "bf16", "identity mapping"),
    (B.make_cfg(8, 64, 16, unroll=2), 4096, 4096, "bf16", "at most 256 threads"),
    (B.make_cfg(8, 256, 1, unroll=2, max_waves_per_simd=8), 4096, 4096, "bf16", "max_waves_per_simd"),
    (B.make_cfg(8, 576, 1, max_waves_per_simd=6), 4096, 4096, "bf16", "both leave"),   # 9-wave groups: caps 5 and 6 both leave 2
    (B.make_cfg(8, 576, 1, max_waves_per_simd=2), 4096, 4096, "bf16", "less than one"),
    (B.make_cfg(8, 576, 1, max_waves_per_simd=7), 4096, 4096, "bf16", "changes nothing"),
]


@pytest.mark.parametrize("cfg,M,N,dtype,needle", KNOWN_INFEASIBLE)
def test_known_infeasible_with_rationale(cfg, M, N, dtype, needle):
    st, why, _ = feas(cfg, M, N, dtype)
    assert st == B.ERR_INFEASIBLE_CFG
    assert needle in why, why
    assert B.addrms_last_error() == why


def test_bad_shape_and_dtype_codes():
    c = B.make_cfg(8, 256, 1)
    assert feas(c, 4, 0, "bf16")[0] == B.ERR_INVALID_ARG
    assert feas(c, -1, 8, "bf16")[0] == B.ERR_INVALID_ARG
    assert feas(c, 4, 4096, 5)[0] == B.ERR_UNSUPPORTED_DTYPE


@pytest.mark.parametrize("M,N,dtype", [(4096, 4096, "bf16"), (1, 8192, "bf16"), (32768, 7168, "bf16"),
                                       (8192, 1000, "fp16_res32"), (8192, 2880, "fp16_res32"), (128, 11008, "fp32")])
def test_enumeration_is_exactly_the_feasible_subset(M, N, dtype):
    cfgs, grid = B.addrms_enumerate_feasible(M, N, dtype)
    # vec, threads/row, rows/wg, reduce, unroll, cap; 7 flag bits, and for the half of them with a persistent grid
    # two more walk lengths
    assert grid == (4 * 19 * 5 * 2 * 4 * 8) * (128 + 64 * 2)
    assert not any(c.flags & (B.FLAG_TWO_PASS | B.FLAG_LDS_CACHE) for c in cfgs)   # these rows fit the register cache
    assert 0 < len(cfgs) < grid
    seen = set()
    for c in cfgs:
        assert feas(c, M, N, dtype)[0] == 0
        assert c.as_tuple() not in seen
        seen.add(c.as_tuple())
        per_pass = c.vec * c.threads_per_row
        cpt = -(-N // per_pass)
        assert N % c.vec == 0 and c.vec * cpt <= 64 and c.unroll <= cpt
        assert (c.threads_per_row * c.rows_per_wg) % 64 == 0 and c.threads_per_row * c.rows_per_wg <= 1024
        assert N / (per_pass * cpt) > 0.5
    # deterministic order
    again, _ = B.addrms_enumerate_feasible(M, N, dtype)
    assert [c.as_tuple() for c in again] == [c.as_tuple() for c in cfgs]


def test_enumeration_counts_are_stable():
    """Region sizes for the benchmark shapes.  Exact counts move with the compiler's
    register allocation (it decides which occupancy caps bind), so only the scale is pinned."""
    got = {k: len(B.addrms_enumerate_feasible(*k)[0]) for k in
           [(4096, 4096, "bf16"), (16, 4096, "bf16"), (256, 8192, "bf16"), (32768, 7168, "bf16")]}
    assert 10000 < got[(4096, 4096, "bf16")] < 60000
    assert got[(16, 4096, "bf16")] < got[(4096, 4096, "bf16")]      # fewer rows: fewer row packings, no XCD map
    assert all(v > 100 for v in got.values())


def test_occupancy_model_matches_compiler_report():
    """waves/SIMD by registers = min(8, 512 // ceil8(vgprs + agprs)) must equal the
    occupancy the compiler printed for the same instance when the library was built."""
    import os
    build = os.path.join(os.path.dirname(B.LIB_PATH), "_build")
    if not os.path.isdir(build):
        pytest.skip("build directory with the compiler's resource report is not present")
    from paper_2601_12698_amd.build import parse_remarks
    reports = {}
    for f in os.listdir(build):
        if f.endswith(".remarks"):
            reports.update(parse_remarks(open(os.path.join(build, f)).read()))
    assert len(reports) >= 1000
    checked = spilled = 0
    for name, r in reports.items():
        m = re.match(r"addrms_k_d(\d)_v(\d)_c(\d+)_u(\d)_n(\d)$", name)
        if not m:
            continue
        regs = -(-max(1, r["vgprs"] + r["agprs"]) // 8) * 8
        assert min(8, 512 // regs) == r["occupancy"], (name, r)
        checked += 1
        if r["scratch"]:
            # an instance that spills is pruned by the deriver whenever a cfg selects it
            dt, vec, cpt, unr, nt = (int(g) for g in m.groups())
            dtype = ["bf16", "fp16", "fp16_res32", "fp32"][dt]
            if cpt == 0:       # two-pass instance: selected by the flag, for a row beyond the register cache
                c = B.make_cfg(vec, 1024, 1, unroll=unr, flags=B.FLAG_TWO_PASS | (B.FLAG_NONTEMPORAL if nt else 0))
                st, why, _ = feas(c, 4096, vec * 1024 * 40, dtype)
            elif cpt >= 400:   # 144-value long-row instance (<= 512 threads): a spilling one is never selected; the
                               # 48-value instance of the same (vec, unroll, policy) stands in, if there is one and it
                               # does not spill
                fit = (160 * 1024 - 128) // (512 * vec * 4)
                c = B.make_cfg(vec, 512, 1, unroll=unr, flags=B.FLAG_LDS_CACHE | B.FLAG_TWO_PASS | (B.FLAG_NONTEMPORAL if nt else 0))
                st, why, res = feas(c, 4096, vec * 512 * (cpt - 400 + fit + 1), dtype)
                assert (st == 0 and res.max_threads == 1024) or \
                       (st == B.ERR_INFEASIBLE_CFG and ("spills" in why or "no compiled instance" in why)), (name, why)
                spilled += 1
                continue
            elif cpt >= 300:   # hybrid instance: registers full (cpt - 300 chunks), LDS full, one more chunk read twice
                fit = (160 * 1024 - 128) // (1024 * vec * 4)
                c = B.make_cfg(vec, 1024, 1, unroll=unr, flags=B.FLAG_LDS_CACHE | B.FLAG_TWO_PASS | (B.FLAG_NONTEMPORAL if nt else 0))
                st, why, _ = feas(c, 4096, vec * 1024 * (cpt - 300 + fit + 1), dtype)
            elif cpt >= 200:   # aligned-span instance
                c = B.make_cfg(vec, 128, 8, unroll=unr, flags=B.FLAG_ALIGNED_SPAN | (B.FLAG_NONTEMPORAL if nt else 0))
                st, why, _ = feas(c, 4096, 1000 if (cpt - 200) * vec * 128 >= 1000 else vec * 125 * (cpt - 200), dtype)
            else:
                c = B.make_cfg(vec, 64, 1, unroll=unr, flags=B.FLAG_NONTEMPORAL if nt else 0)
                st, why, _ = feas(c, 4096, vec * 64 * cpt, dtype)
            assert st == B.ERR_INFEASIBLE_CFG and "spills" in why, (name, why)
            spilled += 1
    # (most of the spilling instances are hybrid long-row ones: 48 cached values at some load depths do not fit 128 registers)
    assert checked >= 1000 and spilled < 0.06 * checked
    # and the library's table carries the same numbers
    c = B.make_cfg(8, 64, 1, unroll=2)
    st, _, res = feas(c, 4096, 4096, "bf16")
    assert st == 0
    rr = reports["addrms_k_d0_v8_c8_u2_n0"]
    assert (res.vgprs, res.agprs) == (rr["vgprs"], rr["agprs"])
    assert res.waves_per_simd_regs == rr["occupancy"]


def test_occupancy_cap_is_modelled():
    """max_waves_per_simd lowers the resident workgroups per CU by LDS padding."""
    base = B.make_cfg(8, 256, 1, unroll=2)
    st, _, r0 = feas(base, 4096, 4096, "bf16")
    assert st == 0 and r0.wgs_per_cu >= 6 and r0.lds_bytes == 128      # 4-wave groups: one per wave-per-SIMD step
    assert r0.wgs_per_cu == r0.waves_per_simd_regs
    for cap, wgs in ((5, 5), (4, 4), (3, 3), (2, 2)):
        c = B.make_cfg(8, 256, 1, unroll=2, max_waves_per_simd=cap)
        st, why, r = feas(c, 4096, 4096, "bf16")
        assert st == 0, why
        assert r.wgs_per_cu == wgs and r.waves_per_simd == wgs
        # the padding admits exactly `wgs` workgroups in 160 KB
        assert wgs * r.lds_bytes <= 160 * 1024 < (wgs + 1) * r.lds_bytes
    st, why, _ = feas(B.make_cfg(8, 256, 1, unroll=2, max_waves_per_simd=1), 4096, 4096, "bf16")
    assert st == B.ERR_INFEASIBLE_CFG and "too few loads in flight" in why


def test_default_cfg():
    for N, dtype in [(4096, "bf16"), (8192, "bf16"), (7168, "bf16"), (5120, "fp16_res32"), (2880, "fp16_res32"),
                     (1000, "fp16_res32"), (4096, "fp32"), (11008, "fp32"), (14336, "fp32"), (1001, "bf16"), (8, "bf16")]:
        d = B.addrms_default_cfg(N, dtype)
        for M in (1, 16, 4096):
            assert feas(d, M, N, dtype)[0] == 0, (N, dtype, M, d)
        assert d.reduce == B.REDUCE_WAVE and d.flags == 0 and d.max_waves_per_simd == 0
    d = B.addrms_default_cfg(4096, "bf16")
    assert d.as_tuple() == (8, 256, 1, 0, 2, 0, 0, 0)
    assert B.load().addrms_default_cfg(1 << 30, B.BF16, B.Cfg()) == B.ERR_UNSUPPORTED_SHAPE
    assert "row cache" in B.addrms_last_error()


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp16_res32", "fp32"])
def test_row_length_bound_of_the_register_cache(dtype):
    """1024 threads x 32 cached values, at most 16 accesses per thread: even N up to 32768 and odd N up to
    16384 run in the plain single-pass form; beyond that the row cache continues in LDS while 160 KB hold
    the rest; then the hybrid form (registers and LDS hold what they can, the rest is read twice) and the plain
    two-pass form take over up to 2^28 elements; beyond that nothing is feasible."""
    long_forms = B.FLAG_TWO_PASS | B.FLAG_LDS_CACHE
    for N in (32768, 32766, 32764, 16383, 16381):
        c = B.addrms_default_cfg(N, dtype)
        assert not c.flags & long_forms
        assert N % c.vec == 0 and c.threads_per_row * c.vec * 16 >= N
        st, why, res = B.addrms_cfg_feasible(c, 4, N, dtype)
        assert st == 0, why
        assert res.chunks_per_thread * c.vec <= 64 and res.scratch_bytes == 0
        two = B.make_cfg(c.vec, 1024, 1, unroll=2, flags=B.FLAG_TWO_PASS)
        st, why, _ = B.addrms_cfg_feasible(two, 4, N, dtype)
        assert st == B.ERR_INFEASIBLE_CFG and "reading every row twice" in why
        st, why, _ = B.addrms_cfg_feasible(B.make_cfg(c.vec, 256, 1, unroll=2, flags=B.FLAG_LDS_CACHE), 4, N, dtype)
        assert st == B.ERR_INFEASIBLE_CFG and ("detour through LDS" in why or "nothing to park" in why), why
    for N in (16385, 24577, 32767):                 # odd rows past 16 one-element chunks: still all in registers
        c = B.addrms_default_cfg(N, dtype)
        assert c.flags == B.FLAG_LDS_CACHE and c.vec == 1 and c.threads_per_row == 1024
        st, why, res = B.addrms_cfg_feasible(c, 4, N, dtype)
        assert st == 0 and 17 <= res.chunks_per_thread <= 32 and res.lds_bytes <= 128, why      # nothing parked
    for N in (32770, 40960, 65536):
        c = B.addrms_default_cfg(N, dtype)          # somewhat beyond the registers: one pass, the rest parked in LDS
        assert c.flags == B.FLAG_LDS_CACHE and N % c.vec == 0 and c.threads_per_row == 1024 and c.rows_per_wg == 1
        st, why, res = B.addrms_cfg_feasible(c, 4, N, dtype)
        assert st == 0, why
        parked = max(0, res.chunks_per_thread - 48 // c.vec)      # 48 values per thread stay in registers
        assert parked >= (1 if N > 49152 else 0) and res.lds_bytes >= parked * 1024 * c.vec * 4 and res.lds_bytes <= 160 * 1024
        assert res.scratch_bytes == 0
    for N in (32767 * 4 + 1, 1 << 20, 1 << 28):
        c = B.addrms_default_cfg(N, dtype)          # too long for LDS as well: what does not fit the chip is read twice
        assert c.flags == long_forms and N % c.vec == 0 and c.threads_per_row == 1024 and c.rows_per_wg == 1
        st, why, res = B.addrms_cfg_feasible(c, 4, N, dtype)
        assert st == 0, why
        assert res.chunks_per_thread == -(-N // (c.vec * c.threads_per_row)) and res.scratch_bytes == 0
        assert 100 * 1024 < res.lds_bytes <= 160 * 1024          # the LDS part is as large as a CU allows
        two = B.make_cfg(c.vec, 1024, 1, unroll=2, flags=B.FLAG_TWO_PASS)
        assert B.addrms_cfg_feasible(two, 4, N, dtype)[0] == 0     # the plain two-pass form stays available
        st, why, _ = B.addrms_cfg_feasible(B.make_cfg(c.vec, 1024, 1, unroll=2, flags=B.FLAG_LDS_CACHE), 4, N, dtype)
        assert st == B.ERR_INFEASIBLE_CFG and "bytes of LDS" in why, why
    for N in (65536, 100001):
        cfgs, _ = B.addrms_enumerate_feasible(4, N, dtype)
        assert cfgs and all(c.flags & long_forms and not c.flags & B.FLAG_PERSISTENT for c in cfgs)
        assert any(c.flags & B.FLAG_TWO_PASS for c in cfgs)
        one = B.make_cfg(cfgs[0].vec, 1024, 1)
        st, why, _ = B.addrms_cfg_feasible(one, 4, N, dtype)
        assert st == B.ERR_INFEASIBLE_CFG and ("row cache" in why or "compiled for workgroups" in why), why
    st, why, _ = B.addrms_cfg_feasible(B.make_cfg(8 if dtype != "fp32" else 4, 1024, 1, flags=B.FLAG_TWO_PASS | B.FLAG_LDS_CACHE),
                                       4, 65536, dtype)
    assert st == B.ERR_INFEASIBLE_CFG and "nothing has to be read twice" in why
    # a workgroup addresses rows_per_wg * N elements with 32-bit byte offsets
    st, why, _ = B.addrms_cfg_feasible(B.make_cfg(1, 64, 2, flags=B.FLAG_TWO_PASS), 4, (1 << 28) - 1, dtype)
    assert st == B.ERR_INFEASIBLE_CFG and "32-bit offsets" in why
    for N in ((1 << 28) + 8, 1 << 30):
        with pytest.raises(B.AddrmsError) as e:
            B.addrms_default_cfg(N, dtype)
        assert e.value.status == B.ERR_UNSUPPORTED_SHAPE
        assert B.addrms_enumerate_feasible(4, N, dtype)[0] == []      # the feasible region is empty, not an error


def test_deferred_store_and_walk_are_part_of_the_region():
    """The deferred residual store doubles the register-cached part of the region (another instance, same launch
    shapes); the walk length multiplies only persistent cfgs, and only while the longer grid is still shorter than
    the list of row blocks."""
    M, N, dt = 32768, 7168, "bf16"
    cfgs, _ = B.addrms_enumerate_feasible(M, N, dt)
    plain = [c for c in cfgs if not c.flags & B.FLAG_DEFER_STORE]
    deferred = [c for c in cfgs if c.flags & B.FLAG_DEFER_STORE]
    assert deferred and 0.9 * len(plain) <= len(deferred) <= len(plain)      # a few differ where register counts move a cap
    assert all(c.walk in (0, 4, 16) for c in cfgs)
    assert all(c.flags & B.FLAG_PERSISTENT for c in cfgs if c.walk)
    assert {c.walk for c in cfgs if c.flags & B.FLAG_PERSISTENT} == {0, 4, 16}
    # the instance is another one: resources are reported for it
    base = B.make_cfg(8, 448, 1, unroll=1, flags=B.FLAG_NONTEMPORAL)
    d = B.make_cfg(8, 448, 1, unroll=1, flags=B.FLAG_NONTEMPORAL | B.FLAG_DEFER_STORE)
    (s0, _, r0), (s1, _, r1) = feas(base, M, N, dt), feas(d, M, N, dt)
    assert s0 == 0 and s1 == 0 and r0.chunks_per_thread == r1.chunks_per_thread == 2
    # on a small problem a 16-fold grid covers every row block: pruned as the ordinary grid
    small, _ = B.addrms_enumerate_feasible(4096, 4096, dt)
    assert sum(1 for c in small if c.walk == 16) < sum(1 for c in small if c.walk == 4) < sum(1 for c in small if c.flags & B.FLAG_PERSISTENT and c.walk == 0)
    # the two further operators have no residual stream and therefore no such flag
    assert B.silumul_cfg_feasible(B.make_cfg(8, 704, 1, flags=B.FLAG_DEFER_STORE), 4096, 11008, "bf16")[0] == B.ERR_INFEASIBLE_CFG


def test_aligned_span_form_is_offered_only_where_rows_are_not_whole_lines():
    """N = 1000: rows of 2000 and 4000 bytes; eight of them are whole 128-byte lines.  The span cfgs are
    those whose rows_per_wg makes the span line-aligned, with 16-byte residual pieces."""
    for dt, vec in (("fp16_res32", 4), ("bf16", 8), ("fp32", 4)):
        cfgs, _ = B.addrms_enumerate_feasible(8192, 1000, dt)
        span = [c for c in cfgs if c.flags & B.FLAG_ALIGNED_SPAN]
        assert span and all(c.vec == vec and c.reduce == 0 and not c.flags & B.FLAG_PERSISTENT for c in span)
        xb = 4 if dt == "fp32" else 2
        assert all((c.rows_per_wg * 1000 * xb) % 128 == 0 for c in span)
        assert {c.flags & B.FLAG_DEFER_STORE for c in span} == {0, B.FLAG_DEFER_STORE}
    for n in (4096, 7168, 5120, 2880, 1024):                 # whole lines already: nothing to offer
        cfgs, _ = B.addrms_enumerate_feasible(8192, n, "fp16_res32")
        assert not any(c.flags & B.FLAG_ALIGNED_SPAN for c in cfgs)
    c = B.make_cfg(4, 128, 8, unroll=2, flags=B.FLAG_ALIGNED_SPAN | B.FLAG_NONTEMPORAL)
    st, _, res = feas(c, 8192, 1000, "fp16_res32")
    assert st == 0 and res.chunks_per_thread == 2 and res.lds_bytes == 1024 * 2 * 8 + 32


def test_long_rows_in_small_workgroups_take_the_instance_with_the_larger_register_cache():
    """Workgroups of at most 512 threads leave each lane 256 registers: where the 48-value instance cannot keep
    the whole row on the chip, the long-row forms use the instance that keeps 144 values per thread."""
    lds, two = B.FLAG_LDS_CACHE, B.FLAG_TWO_PASS
    # 131072 bf16 over 512 threads of 8: 32 chunks per thread; 48-value instance: 6 + 9 in LDS; 144-value: 18 + 9
    st, why, res = feas(B.make_cfg(8, 512, 1, unroll=2, flags=lds | two | B.FLAG_NONTEMPORAL), 1024, 131072, "bf16")
    assert st == 0 and res.max_threads == 512 and res.vgprs + res.agprs > 200, (why, res.as_dict())
    # the same row over 1024 threads stays with the 48-value instance
    st, why, res = feas(B.make_cfg(8, 1024, 1, unroll=2, flags=lds | two | B.FLAG_NONTEMPORAL), 1024, 131072, "bf16")
    assert st == 0 and res.max_threads == 1024 and res.vgprs + res.agprs <= 128
    # 98304 elements over 512 threads: 24 chunks = 18 in registers + 6 in LDS: one pass where there was none
    st, why, res = feas(B.make_cfg(8, 512, 1, unroll=2, flags=lds), 1024, 98304, "bf16")
    assert st == 0 and res.max_threads == 512, why
    st, why, _ = feas(B.make_cfg(8, 512, 1, unroll=2, flags=lds | two), 1024, 98304, "bf16")
    assert st == B.ERR_INFEASIBLE_CFG and "nothing has to be read twice" in why
    # a row the 48-value instance holds on the chip at 512 threads keeps that instance (two workgroups fit a CU)
    st, why, res = feas(B.make_cfg(8, 512, 1, unroll=2, flags=lds), 1024, 49152, "bf16")
    assert st == 0 and res.max_threads == 1024 and res.vgprs + res.agprs <= 128
    # fp32: every 144-value instance spills, so the 48-value one stands in
    st, why, res = feas(B.make_cfg(4, 512, 1, unroll=2, flags=lds | two), 512, 262144, "fp32")
    assert st == 0 and res.max_threads == 1024, why
