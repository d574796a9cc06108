"""Pins for the merge_attn_states oracle (CPU only)."""
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest

from exact import bits_to_fraction, round_to_format

BF16, FP16 = 0, 1
FMT = {BF16: "bf16", FP16: "f16"}


def _enc(oracle, a, dt):
    a = np.asarray(a, dtype=np.float32)
    return oracle.f32_to_bf16_array(a) if dt == BF16 else oracle.f32_to_f16_array(a)


def _dec(oracle, b, dt):
    return (oracle.bf16_to_f32_array(b) if dt == BF16 else oracle.f16_to_f32_array(b)).astype(np.float64)


def _case(oracle, rows, d, dt, seed, s_scale=3.0):
    rng = np.random.default_rng(seed)
    va = _enc(oracle, rng.standard_normal((rows, d)), dt)
    vb = _enc(oracle, rng.standard_normal((rows, d)), dt)
    sa = (rng.standard_normal(rows) * s_scale).astype(np.float32)
    sb = (rng.standard_normal(rows) * s_scale).astype(np.float32)
    return va, sa, vb, sb


@pytest.mark.parametrize("dt", [BF16, FP16])
def test_equal_scores_give_the_average(oracle, dt):
    va, sa, vb, _ = _case(oracle, 6, 64, dt, 0)
    vout, sout, v64 = oracle.mergestates(va, sa, vb, sa.copy(), dt, want_f64=True)
    assert np.array_equal(v64, (_dec(oracle, va, dt) + _dec(oracle, vb, dt)) / 2)
    assert np.allclose(sout, sa.astype(np.float64) + np.log(2.0), rtol=1e-7)


@pytest.mark.parametrize("dt", [BF16, FP16])
def test_dominant_part_passes_through(oracle, dt):
    """exp(-80) < 2^-53 * anything here: the weaker part vanishes in fp64."""
    va, sa, vb, _ = _case(oracle, 4, 32, dt, 1)
    sb = (sa - 80.0).astype(np.float32)
    vout, sout = oracle.mergestates(va, sa, vb, sb, dt)
    assert np.array_equal(vout, va) and np.array_equal(sout, sa)
    vout, sout = oracle.mergestates(vb, sb, va, sa, dt)
    assert np.array_equal(vout, va) and np.array_equal(sout, sa)


@pytest.mark.parametrize("dt", [BF16, FP16])
def test_swapping_the_parts_changes_nothing(oracle, dt):
    va, sa, vb, sb = _case(oracle, 9, 128, dt, 2)
    a = oracle.mergestates(va, sa, vb, sb, dt)
    b = oracle.mergestates(vb, sb, va, sa, dt)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_common_shift_of_scores(oracle):
    """Scores shifted by a power of two that keeps them exact: v_out identical, s_out shifted."""
    va, sa, vb, sb = _case(oracle, 7, 64, BF16, 3)
    sa = np.round(sa * 8) / 8
    sb = np.round(sb * 8) / 8
    sa, sb = sa.astype(np.float32), sb.astype(np.float32)
    v0, s0, r0 = oracle.mergestates(va, sa, vb, sb, BF16, want_f64=True)
    v1, s1, r1 = oracle.mergestates(va, sa + 16, vb, sb + 16, BF16, want_f64=True)
    assert np.array_equal(r0, r1) and np.array_equal(v0, v1)
    assert np.allclose(s1.astype(np.float64), s0.astype(np.float64) + 16, rtol=0, atol=2e-6)


def test_s_out_is_logaddexp(oracle):
    va, sa, vb, sb = _case(oracle, 500, 8, BF16, 4, s_scale=10.0)
    _, sout = oracle.mergestates(va, sa, vb, sb, BF16)
    want = np.logaddexp(sa.astype(np.float64), sb.astype(np.float64)).astype(np.float32)
    assert np.abs(sout.view(np.int32).astype(np.int64) - want.view(np.int32)).max() <= 1


@pytest.mark.parametrize("dt", [BF16, FP16])
def test_output_lies_between_the_inputs(oracle, dt):
    va, sa, vb, sb = _case(oracle, 20, 96, dt, 5)
    vout, _ = oracle.mergestates(va, sa, vb, sb, dt)
    a, b, o = _dec(oracle, va, dt), _dec(oracle, vb, dt), _dec(oracle, vout, dt)
    assert np.all(o >= np.minimum(a, b)) and np.all(o <= np.maximum(a, b))


@pytest.mark.parametrize("dt", [BF16, FP16])
def test_against_50_digit_decimal(oracle, dt):
    getcontext().prec = 50
    va, sa, vb, sb = _case(oracle, 3, 40, dt, 6)
    vout, sout = oracle.mergestates(va, sa, vb, sb, dt)
    A, Bv = _dec(oracle, va, dt), _dec(oracle, vb, dt)
    for i in range(3):
        a, b = Decimal(float(sa[i])), Decimal(float(sb[i]))
        m = max(a, b)
        ea, eb = (a - m).exp(), (b - m).exp()
        s_real = m + (ea + eb).ln()
        kind, sval = round_to_format(Fraction(s_real), "f32")
        assert Fraction(float(sout[i])) == sval
        for j in range(40):
            real = (ea * Decimal(float(A[i, j])) + eb * Decimal(float(Bv[i, j]))) / (ea + eb)
            kind, val = round_to_format(Fraction(real), FMT[dt])
            assert bits_to_fraction(int(vout[i, j]), FMT[dt]) == val, (i, j)


def test_rows_are_independent_and_indexed_correctly(oracle):
    """Row i of the outputs depends on row i of every input only: permuting rows permutes outputs,
    and a score pair that selects part a on even rows and part b on odd rows copies exactly those."""
    rows, d = 12, 16
    va, sa, vb, sb = _case(oracle, rows, d, BF16, 7)
    sa = np.where(np.arange(rows) % 2 == 0, 50.0, -50.0).astype(np.float32)
    sb = -sa
    vout, sout = oracle.mergestates(va, sa, vb, sb, BF16)
    assert np.array_equal(vout[0::2], va[0::2]) and np.array_equal(vout[1::2], vb[1::2])
    assert np.all(sout == 50.0)
    va, sa, vb, sb = _case(oracle, rows, d, BF16, 8)
    perm = np.random.default_rng(9).permutation(rows)
    a = oracle.mergestates(va, sa, vb, sb, BF16)
    b = oracle.mergestates(va[perm].copy(), sa[perm].copy(), vb[perm].copy(), sb[perm].copy(), BF16)
    assert np.array_equal(b[0], a[0][perm]) and np.array_equal(b[1], a[1][perm])


def test_huge_score_gap_is_stable(oracle):
    """Shifting by the maximum keeps every exponent <= 0; a gap of 1000 must not overflow."""
    va, sa, vb, _ = _case(oracle, 4, 16, BF16, 10)
    sa = np.full(4, 500.0, dtype=np.float32)
    sb = np.full(4, -500.0, dtype=np.float32)
    vout, sout = oracle.mergestates(va, sa, vb, sb, BF16)
    assert np.array_equal(vout, va) and np.all(sout == 500.0)
    vout, sout = oracle.mergestates(va, sb, vb, sa, BF16)
    assert np.array_equal(vout, vb) and np.all(sout == 500.0)


def test_no_double_rounding_through_fp32(oracle):
    """Values that round to fp32 exactly onto a bf16 tie while lying strictly on one side of it."""
    rng = np.random.default_rng(11)
    rows, d = 1 << 13, 128
    va = _enc(oracle, rng.standard_normal((rows, d)), BF16)
    vb = _enc(oracle, rng.standard_normal((rows, d)), BF16)
    sa = rng.standard_normal(rows).astype(np.float32)
    sb = rng.standard_normal(rows).astype(np.float32)
    vout, _, real = oracle.mergestates(va, sa, vb, sb, BF16, want_f64=True)
    f32 = real.astype(np.float32)
    on_tie = ((f32.view(np.uint32) & 0xffff) == 0x8000) & (f32.astype(np.float64) != real)
    idx = np.argwhere(on_tie)
    assert len(idx) >= 4
    differs = 0
    for i, j in idx.tolist():
        kind, val = round_to_format(Fraction(float(real[i, j])), "bf16")
        assert bits_to_fraction(int(vout[i, j]), "bf16") == val
        differs += int(oracle.f32_to_bf16(float(f32[i, j])) != int(vout[i, j]))
    assert differs >= 1
