"""The audit of the deriver's efficiency rules, driven by synthetic cost functions (no GPU).

The audit switches the judgement rules off (lane utilisation, occupancy floor, spilling
instances, long-row forms and the aligned span where the plain form would do), times
retained and pruned configurations alike and says whether
anything pruned beats the best retained one.  Here the "timings" are functions chosen
so that the right answer is known.
"""
import ctypes

import pytest

from paper_2601_12698_amd import binding as B

M, N, DT = 2048, 1000, "fp16_res32"


def _util(c):
    per_pass = c.vec * c.threads_per_row
    need = -(-N // per_pass)
    return N / (per_pass * need)


def _honest_cost(c, _w, _r):
    """Idle lanes cost time and so does reading a row twice; nothing pruned can win."""
    t = 10.0 / _util(c) + 0.01 * c.rows_per_wg + (0.5 if c.reduce else 0.0)
    return t * (1.5 if c.flags & B.FLAG_TWO_PASS else 1.1 if c.flags & B.FLAG_LDS_CACHE else 1.0)


def test_struct_sizes():
    assert ctypes.sizeof(B.AuditRule) == 96
    assert ctypes.sizeof(B.AuditReport) == 88 + B.AUDIT_RULES * 96 and B.AUDIT_RULES == 6


def test_classes_partition_the_relaxed_grid():
    seen = []
    rep = B.addrms_audit_rules_with_backend(M, N, DT, B.make_budget(), lambda c, w, r: (seen.append(c.as_tuple()), _honest_cost(c, w, r))[1])
    strict, _ = B.addrms_enumerate_feasible(M, N, DT)
    assert rep.n_retained == len(strict) == rep.n_retained_measured
    names = [r.rule.decode() for r in rep.rules]
    assert names == ["lane_utilisation", "occupancy_floor", "scratch", "two_pass_needless", "lds_cache_needless",
                     "span_needless"]
    lane = rep.rules[0]
    assert lane.n_pruned > 0 and lane.n_measured == lane.n_pruned
    assert len(seen) == len(set(seen)) == rep.n_retained + sum(r.n_measured for r in rep.rules)
    # every cfg the audit timed beyond the strict region is refused by the strict check, for the rule it was filed under
    strict_set = {c.as_tuple() for c in strict}
    extra = [t for t in seen if t not in strict_set]
    assert len(extra) == sum(r.n_pruned for r in rep.rules)
    words = {"lane_utilisation": "lane slots", "occupancy_floor": "wave per SIMD", "scratch": "spills",
             "two_pass_needless": "reading every row twice", "lds_cache_needless": "detour through LDS",
             "span_needless": "whole cache lines already"}
    n_lane = 0
    for t in extra[::17]:
        st, why, _ = B.addrms_cfg_feasible(B.make_cfg(*t), M, N, DT)
        assert st == B.ERR_INFEASIBLE_CFG and any(w in why for w in words.values()), why
        n_lane += "lane slots" in why
    assert n_lane > 0


def test_sound_rules_report_nothing_beating_the_best():
    rep = B.addrms_audit_rules_with_backend(M, N, DT, B.make_budget(), _honest_cost)
    assert not rep.truncated
    for r in rep.rules:
        assert r.n_beating_best == 0
        if r.rule == b"lane_utilisation":
            assert r.n_measured and r.best_us >= 2 * 10.0 > rep.retained_best_us      # util <= 1/2 costs at least double
            assert r.n_in_top_decile == 0 and r.median_us >= r.best_us
    assert rep.retained_best_us <= rep.retained_decile_us <= rep.retained_median_us


def test_an_unsound_rule_is_caught():
    """If a pruned configuration were in fact the fastest, the audit names it."""
    rep0 = B.addrms_audit_rules_with_backend(M, N, DT, B.make_budget(), _honest_cost)
    target = rep0.rules[0].best.as_tuple()                  # some cfg only the lane rule prunes

    def cost(c, w, r):
        return 1.0 if c.as_tuple() == target else _honest_cost(c, w, r)

    rep = B.addrms_audit_rules_with_backend(M, N, DT, B.make_budget(), cost)
    lane = rep.rules[0]
    assert lane.n_beating_best == 1 and lane.n_in_top_decile >= 1
    assert lane.best.as_tuple() == target and lane.best_us == 1.0
    assert rep.retained_best.as_tuple() != target


def test_gate_failures_and_measure_failures_are_counted_not_ranked():
    def validate(c):
        return c.rows_per_wg != 2

    def cost(c, w, r):
        if c.unroll == 1 and c.rows_per_wg == 1:
            return None
        return _honest_cost(c, w, r)

    rep = B.addrms_audit_rules_with_backend(M, N, DT, B.make_budget(), cost, validate)
    strict, _ = B.addrms_enumerate_feasible(M, N, DT)
    bad = sum(1 for c in strict if c.rows_per_wg == 2 or (c.unroll == 1 and c.rows_per_wg == 1))
    assert rep.n_retained_failed == bad and rep.n_retained_measured == len(strict) - bad
    assert rep.retained_best.rows_per_wg != 2
    assert rep.rules[0].n_failed > 0 and rep.rules[0].n_failed + rep.rules[0].n_measured == rep.rules[0].n_pruned


def test_budget_caps_each_class_and_wall_time_truncates():
    rep = B.addrms_audit_rules_with_backend(M, N, DT, B.make_budget(max_candidates=50), _honest_cost)
    assert rep.n_retained_measured == rep.n_retained          # the yardstick is always measured in full
    for r in rep.rules:
        assert r.n_measured <= 50
        if r.n_pruned > 100:
            assert r.n_measured >= 25
    import time

    def slow(c, w, r):
        time.sleep(0.002)
        return _honest_cost(c, w, r)

    rep = B.addrms_audit_rules_with_backend(M, N, DT, B.make_budget(max_wall_ms=400.0), slow)
    assert rep.truncated and rep.n_retained_measured < rep.n_retained


def test_bad_arguments():
    with pytest.raises(B.AddrmsError):
        B.addrms_audit_rules_with_backend(0, N, DT, None, _honest_cost)
    with pytest.raises(B.AddrmsError):
        B.addrms_audit_rules_with_backend(M, N, 9, None, _honest_cost)
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_audit_rules_with_backend(4, (1 << 28) + 8, "bf16", None, _honest_cost)
    assert e.value.status == B.ERR_UNSUPPORTED_SHAPE
