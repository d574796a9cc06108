"""The outer loop with a fixed strategy list (Level 1 of Algorithm 1 in deterministic
form) against synthetic cost functions: families are added round by round, a family
that fails validation is rolled back, the incumbent is the best-scoring round."""
import json
import math

import pytest

from paper_2601_12698_amd import binding as B

DT = "bf16"
SHAPES = [(4096, 4096), (8192, 8192)]


def cost(M, N):
    def f(c):
        us = 10.0 + M * N * 1e-6
        us *= 1.0 + 0.2 * abs(math.log2(c.threads_per_row / 512.0)) + 0.2 * abs(math.log2(c.vec / 8.0))
        us *= 0.85 if c.flags & B.FLAG_NONTEMPORAL else 1.0                 # streaming pays
        us *= 0.97 if c.max_waves_per_simd in (4, 5, 6) else 1.0             # a cap pays a little
        us *= 1.04 if c.flags & B.FLAG_PERSISTENT else 1.0                   # the persistent grid does not
        us *= 1.01 if c.flags & B.FLAG_XCD_CONTIG else 1.0
        us *= 0.97 if c.flags & B.FLAG_DEFER_STORE else 1.0                  # one read phase, one write phase
        us *= 1.05 if c.reduce else 1.0
        return us
    return f


def backend(validate=lambda c: True):
    def make(M, N):
        fn = cost(M, N)
        return (lambda c, w, r: fn(c)), validate
    return make


def test_rounds_add_families_and_keep_the_best(tmp_path):
    log = str(tmp_path / "rounds.jsonl")
    g, rep = B.addrms_tune_rounds_with_backend(SHAPES, DT, B.make_budget(log_path=log), backend())
    assert rep.n_rounds == 5
    fam = [rep.rounds[i].families for i in range(5)]
    three = B.FAMILY_STREAMING | B.FAMILY_OCCUPANCY_CAP | B.FAMILY_GRID_MAPPING
    assert fam == [0, B.FAMILY_STREAMING, B.FAMILY_STREAMING | B.FAMILY_OCCUPANCY_CAP, three, three | B.FAMILY_STORE_PHASE]
    assert all(rep.rounds[i].passed for i in range(5))
    # round 0 may only use the base template
    r0 = rep.rounds[0].general
    assert r0.flags == 0 and r0.max_waves_per_simd == 0
    assert rep.rounds[1].general.flags == B.FLAG_NONTEMPORAL
    scores = [rep.rounds[i].score for i in range(5)]
    assert scores[1] < scores[0] - 0.1                  # streaming is a structural gain
    assert scores[2] <= scores[1] + 1e-9                # more families never hurt the specialised table
    assert scores[4] < scores[3] - 0.01                 # so is the deferred store in this landscape
    assert rep.best_round == min(range(5), key=lambda i: scores[i])
    assert -rep.rounds[rep.best_round].score == pytest.approx(rep.best.geomean_speedup_specialized)
    assert not (g.flags & B.FLAG_PERSISTENT) and g.flags & B.FLAG_NONTEMPORAL
    lines = [json.loads(l) for l in open(log)]
    rounds = [l for l in lines if l["event"] == "round"]
    assert [l["round"] for l in rounds] == [0, 1, 2, 3, 4] and rounds[-1]["incumbent"] == rep.best_round


def test_a_family_that_fails_validation_is_rolled_back():
    broken = lambda c: not (c.flags & B.FLAG_NONTEMPORAL)      # the streaming variants give wrong output
    g, rep = B.addrms_tune_rounds_with_backend(SHAPES, DT, B.make_budget(), backend(broken))
    assert rep.rounds[1].passed == 0
    assert rep.rounds[1].families == 0                          # rolled back to the base template
    assert rep.rounds[1].score == rep.rounds[0].score
    for i in range(rep.n_rounds):
        assert not (rep.rounds[i].families & B.FAMILY_STREAMING)
        assert not (rep.rounds[i].general.flags & B.FLAG_NONTEMPORAL)
    assert not (g.flags & B.FLAG_NONTEMPORAL)
    assert rep.rounds[2].families == B.FAMILY_OCCUPANCY_CAP     # later families still get their round


def test_family_mask_restricts_a_single_search():
    rec = []
    fn = cost(4096, 4096)
    B.addrms_tune_with_backend(4096, 4096, DT, B.make_budget(family_mask=B.FAMILY_BASE_ONLY),
                               lambda c, w, r: (rec.append(c.as_tuple()), fn(c))[1])
    assert rec and all(t[5] == 0 and t[6] == 0 for t in rec)
    rec.clear()
    B.addrms_tune_with_backend(4096, 4096, DT, B.make_budget(family_mask=B.FAMILY_STREAMING),
                               lambda c, w, r: (rec.append(c.as_tuple()), fn(c))[1])
    assert any(t[5] == B.FLAG_NONTEMPORAL for t in rec) and all(t[5] in (0, 2) and t[6] == 0 for t in rec)
