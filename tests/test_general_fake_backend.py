"""SelectGeneral (one configuration for a set of shapes) against synthetic per-shape
cost functions with a known answer (host logic only)."""
import math

import pytest

from paper_2601_12698_amd import binding as B

DT = "bf16"
SHAPES = [(16, 4096), (32, 5120), (32, 8192), (16, 12288), (64, 8192)]   # (m, n) pairs of the kind the paper lists


def shape_cost(M, N):
    """Each shape prefers a row width proportional to its N (one chunk of 8 per thread),
    so no single threads_per_row suits all of them."""
    want = N / 8.0

    def cost(c):
        us = 3.0 + N * M * 1e-5
        us *= 1.0 + 0.25 * abs(math.log2(c.threads_per_row / want))
        us *= 1.0 + 0.2 * abs(math.log2(c.vec / 8.0))
        us *= 1.05 if c.reduce else 1.0
        us *= 0.9 if c.flags & B.FLAG_NONTEMPORAL else 1.0
        us *= 1.0 + 0.02 * c.rows_per_wg + 0.01 * abs(math.log2(c.unroll))
        us *= 1.0 + 0.01 * c.max_waves_per_simd
        return us
    return cost


def make_backend(M, N):
    fn = shape_cost(M, N)
    return (lambda c, w, r: fn(c)), (lambda c: True)


def brute_force_general():
    sets = []
    for M, N in SHAPES:
        cfgs, _ = B.addrms_enumerate_feasible(M, N, DT)
        sets.append({c.as_tuple(): c for c in cfgs})
    common = set(sets[0])
    for s in sets[1:]:
        common &= set(s)
    defaults = [B.addrms_default_cfg(N, DT) for _, N in SHAPES]

    def score(t):
        c = sets[0][t]
        return math.exp(sum(math.log(shape_cost(M, N)(d) / shape_cost(M, N)(c))
                            for (M, N), d in zip(SHAPES, defaults)) / len(SHAPES))
    best = max(common, key=score)
    return sets[0][best], score(best), len(common)


def test_general_cfg_is_feasible_everywhere_and_near_optimal():
    g, rep = B.addrms_select_general_with_backend(SHAPES, DT, B.make_budget(), make_backend)
    for M, N in SHAPES:
        assert B.addrms_cfg_feasible(g, M, N, DT)[0] == 0
    best, best_score, ncommon = brute_force_general()
    assert ncommon > 10
    assert rep.n_shapes == len(SHAPES) and rep.n_pool >= 3
    # the report's aggregate is the geometric mean of default/general per shape
    ratios = [rep.default_us[i] / rep.general_us[i] for i in range(rep.n_shapes)]
    assert rep.geomean_speedup_general == pytest.approx(math.exp(sum(map(math.log, ratios)) / len(ratios)))
    assert rep.mean_speedup_general == pytest.approx(sum(ratios) / len(ratios))
    # a general cfg is a compromise: never better than specialising, and close to the best compromise
    assert rep.geomean_speedup_specialized >= rep.geomean_speedup_general - 1e-12
    assert rep.geomean_speedup_general >= 0.95 * best_score
    assert rep.geomean_speedup_general > 1.0
    for i, (M, N) in enumerate(SHAPES):
        assert rep.general_us[i] == pytest.approx(shape_cost(M, N)(g))
        assert rep.specialized_us[i] <= rep.general_us[i] + 1e-12
        assert B.addrms_cfg_feasible(rep.specialized[i], M, N, DT)[0] == 0


def test_general_single_shape_equals_specialised():
    g, rep = B.addrms_select_general_with_backend([(4096, 4096)], DT, B.make_budget(), make_backend)
    assert rep.geomean_speedup_general == pytest.approx(rep.geomean_speedup_specialized)
    assert rep.specialized[0].as_tuple() == g.as_tuple()


def test_general_argument_errors():
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_select_general_with_backend([], DT, None, make_backend)
    assert e.value.status == B.ERR_INVALID_ARG
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_select_general_with_backend([(4, 4096)] * 17, DT, None, make_backend)
    assert e.value.status == B.ERR_INVALID_ARG
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_select_general_with_backend([(0, 4096)], DT, None, make_backend)
    assert e.value.status == B.ERR_INVALID_ARG
    # N = 1001 needs vec 1, N = 4096 x 16 rows cannot use vec 1 rows that long? both feasible sets exist but share nothing
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_select_general_with_backend([(64, 8), (64, 16384)], DT, B.make_budget(max_candidates=20), make_backend)
    assert e.value.status == B.ERR_NO_RESULT
