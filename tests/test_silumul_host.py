"""silu_and_mul through the same deriver and search (host logic, no GPU)."""
import math

import pytest

from paper_2601_12698_amd import binding as B


def test_bytes_and_dtypes():
    assert B.silumul_algorithmic_bytes(4096, 11008, "bf16") == 4096 * 11008 * 6
    assert B.silumul_algorithmic_bytes(16, 1000, "fp32") == 16 * 1000 * 12
    assert B.load().silumul_algorithmic_bytes(16, 1000, B.FP16_RES32) == B.ERR_UNSUPPORTED_DTYPE
    assert B.load().silumul_algorithmic_bytes(16, 0, B.BF16) == B.ERR_INVALID_ARG


def test_default_and_feasibility_rules():
    for d, dt in [(11008, "bf16"), (14336, "bf16"), (13824, "fp16"), (28672, "bf16"), (1000, "fp16"), (4096, "fp32"),
                  (1001, "bf16")]:
        c = B.silumul_default_cfg(d, dt)
        assert c.reduce == 0 and c.flags == 0
        for M in (1, 64, 4096):
            assert B.silumul_cfg_feasible(c, M, d, dt)[0] == 0, (d, dt, M, c)
    st, why, _ = B.silumul_cfg_feasible(B.make_cfg(8, 256, 1, reduce=1), 64, 4096, "bf16")
    assert st == B.ERR_INFEASIBLE_CFG and "no reduction" in why
    st, why, _ = B.silumul_cfg_feasible(B.make_cfg(8, 256, 1), 64, 4100, "bf16")
    assert st == B.ERR_INFEASIBLE_CFG and "does not divide" in why
    st, why, _ = B.silumul_cfg_feasible(B.make_cfg(8, 64, 1), 64, 8192, "bf16")      # 16 chunks: no instance here
    assert st == B.ERR_INFEASIBLE_CFG
    assert B.silumul_cfg_feasible(B.make_cfg(8, 256, 1), 64, 4096, B.FP16_RES32)[0] == B.ERR_UNSUPPORTED_DTYPE
    # no LDS is needed without a reduction, persistent or not
    st, _, res = B.silumul_cfg_feasible(B.make_cfg(8, 512, 1, flags=B.FLAG_PERSISTENT | B.FLAG_NONTEMPORAL), 8192, 4096, "bf16")
    assert st == 0 and res.lds_bytes == 0


def test_enumeration_has_no_reduction_variants():
    cfgs, grid = B.silumul_enumerate_feasible(4096, 11008, "bf16")
    assert grid == (4 * 19 * 5 * 2 * 4 * 8) * (128 + 64 * 2) and len(cfgs) > 500
    assert all(c.reduce == 0 for c in cfgs)
    for c in cfgs[::37]:
        assert B.silumul_cfg_feasible(c, 4096, 11008, "bf16")[0] == 0
        # the same cfg need not be feasible for the other operator and vice versa; the spaces are separate
    a, _ = B.addrms_enumerate_feasible(4096, 11008, "bf16")
    assert {c.as_tuple() for c in cfgs} != {c.as_tuple() for c in a}


def test_search_runs_over_this_operator_space():
    seen = []

    def measure(c, w, r):
        seen.append(c.as_tuple())
        return 30.0 * (1 + 0.2 * abs(math.log2(c.threads_per_row / 512))) * (0.9 if c.flags & 2 else 1.0) \
            * (1 + 0.1 * abs(math.log2(c.vec / 8)))
    g, rep = B.silumul_tune_with_backend(4096, 11008, "bf16", B.make_budget(), measure, lambda c: True)
    assert all(t[3] == 0 for t in seen)
    assert B.silumul_cfg_feasible(g, 4096, 11008, "bf16")[0] == 0
    assert g.flags & B.FLAG_NONTEMPORAL and g.vec == 8
    assert rep.best_us < rep.default_us


def test_tables_are_per_operator(tmp_path):
    B.addrms_table_clear()
    c = B.make_cfg(8, 512, 1, flags=2)
    B.addrms_table_insert(4096, 4096, "bf16", c, 1.0)
    assert B.silumul_table_lookup(4096, 4096, "bf16") is None        # the add+RMSNorm entry is not visible here
    assert B.addrms_table_lookup(4096, 4096, "bf16").as_tuple() == c.as_tuple()
    p = str(tmp_path / "t.txt")
    B.addrms_table_save(p)
    assert open(p).read().splitlines()[4].startswith("0 0 4096 4096 ")
    B.addrms_table_clear()
