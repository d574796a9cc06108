"""Audit of the deriver's efficiency rules on the device (needs an MI355X).

The plain definition of the feasible region is "try everything": here every
configuration that only a judgement rule keeps out (lane utilisation, occupancy
floor, spilling instance, a long-row form where the registers would do) is run through the same gate and screening protocol as
the retained ones.  Two things must hold: the pruned configurations are still
*correct* (the rules are about speed, never about validity), and none of them
beats the best retained configuration beyond timing noise (the rules are sound).
"""
import pytest

from paper_2601_12698_amd import binding as B

pytestmark = pytest.mark.gpu

NOISE = 0.95     # 3 + 15 launches of a few microseconds each: allow 5 %


@pytest.mark.parametrize("M,N,dtype,expect", [
    (2048, 1000, "fp16_res32", ("lane_utilisation", "occupancy_floor")),
    (4096, 4096, "bf16", ("lane_utilisation", "occupancy_floor", "span_needless")),
    (1024, 11008, "fp32", ("scratch", "span_needless")),
])
def test_pruned_cfgs_are_correct_and_never_win(M, N, dtype, expect):
    # the retained region is always timed in full; each pruned class is sampled down to at most 4000 cfgs
    rep = B.addrms_audit_rules(M, N, dtype, B.make_budget(max_candidates=4000))
    d = rep.as_dict()
    print({k: v for k, v in d.items() if k != "rules"}, flush=True)
    assert not rep.truncated and rep.n_retained_failed == 0 and rep.n_retained_measured == rep.n_retained
    for r in rep.rules:
        print(r.as_dict(), flush=True)
        assert r.n_failed == 0, "a cfg pruned for efficiency must still compute the right result"
        assert r.n_measured == r.n_pruned or r.n_measured >= 2000
        if r.rule.decode() in expect:
            assert r.n_pruned > 0
        if r.n_measured:
            assert r.best_us >= NOISE * rep.retained_best_us, (r.as_dict(), rep.retained_best_us)
