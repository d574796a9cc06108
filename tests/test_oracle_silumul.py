"""Pins for the silu_and_mul oracle (CPU only)."""
import math
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch

from exact import bits_to_fraction, fraction_to_bits, round_to_format
from ulp import ulp_distance

BF16, FP16, FP32 = 0, 1, 3
FMT = {BF16: "bf16", FP16: "f16"}


def _enc(oracle, a, dt):
    a = np.asarray(a, dtype=np.float32)
    if dt == FP32:
        return a
    return oracle.f32_to_bf16_array(a) if dt == BF16 else oracle.f32_to_f16_array(a)


def _dec(oracle, b, dt):
    if dt == FP32:
        return b.astype(np.float64)
    return (oracle.bf16_to_f32_array(b) if dt == BF16 else oracle.f16_to_f32_array(b)).astype(np.float64)


def _rows(oracle, gate, up, dt):
    return np.ascontiguousarray(np.concatenate([_enc(oracle, gate, dt), _enc(oracle, up, dt)], axis=1))


def test_antisymmetry_identity(oracle):
    """silu(g) - silu(-g) = g, because sigmoid(g) + sigmoid(-g) = 1."""
    rng = np.random.default_rng(0)
    g = (rng.standard_normal((4, 300)) * 4).astype(np.float32)
    one = np.ones_like(g)
    a = oracle.silumul_f64(_rows(oracle, g, one, FP32), FP32)
    b = oracle.silumul_f64(_rows(oracle, -g, one, FP32), FP32)
    assert np.allclose(a - b, g.astype(np.float64), rtol=1e-14, atol=1e-300)


@pytest.mark.parametrize("dt", [BF16, FP16, FP32])
def test_zeros_in_either_half(oracle, dt):
    rng = np.random.default_rng(1)
    v = rng.standard_normal((3, 64)).astype(np.float32)
    z = np.zeros_like(v)
    out = oracle.silumul(_rows(oracle, z, v, dt), dt)
    assert np.all(_dec(oracle, out, dt) == 0)
    out = oracle.silumul(_rows(oracle, v, z, dt), dt)
    assert np.all(_dec(oracle, out, dt) == 0)


@pytest.mark.parametrize("dt", [BF16, FP16])
def test_large_gate_passes_up_through_and_layout(oracle, dt):
    """For g >= 40, exp(-g) < 2^-53 so silu(g) = g exactly in fp64; with position-coded up
    values the output pins which element of the row pairs with which (gate half first)."""
    M, d = 5, 24
    gate = np.full((M, d), 64.0, dtype=np.float32)
    code = np.array([[(i * 7 + j) % 13 - 6 for j in range(d)] for i in range(M)], dtype=np.float32)
    out = oracle.silumul(_rows(oracle, gate, code, dt), dt)
    assert np.array_equal(_dec(oracle, out, dt), 64.0 * code)
    # swapping the halves must change the answer (silu(code) * 64 is something else)
    out2 = oracle.silumul(_rows(oracle, code, gate, dt), dt)
    assert not np.array_equal(out, out2)
    neg = oracle.silumul(_rows(oracle, np.full((1, 8), -60.0, np.float32), np.ones((1, 8), np.float32), dt), dt)
    assert np.all(np.abs(_dec(oracle, neg, dt)) < 1e-20)


@pytest.mark.parametrize("dt", [BF16, FP16])
def test_against_50_digit_decimal(oracle, dt):
    """The real value from 50-digit decimal arithmetic, rounded nearest-even with exact
    rationals, equals the oracle's bits (single rounding of the real result)."""
    getcontext().prec = 50
    rng = np.random.default_rng(2)
    g = (rng.standard_normal((2, 150)) * 3).astype(np.float32)
    u = (rng.standard_normal((2, 150)) * 2).astype(np.float32)
    x = _rows(oracle, g, u, dt)
    out = oracle.silumul(x, dt)
    gd, ud = _dec(oracle, x[:, :150], dt), _dec(oracle, x[:, 150:], dt)
    for i in range(2):
        for j in range(150):
            G, U = Decimal(float(gd[i, j])), Decimal(float(ud[i, j]))
            real = G / (1 + (-G).exp()) * U
            kind, val = round_to_format(Fraction(real), FMT[dt])
            assert kind == "fin"
            got = bits_to_fraction(int(out[i, j]), FMT[dt])
            assert got == val, (i, j, float(real))


def test_fp32_output_is_the_rounded_fp64_value(oracle):
    rng = np.random.default_rng(3)
    g = (rng.standard_normal((3, 200)) * 3).astype(np.float32)
    u = rng.standard_normal((3, 200)).astype(np.float32)
    x = _rows(oracle, g, u, FP32)
    out = oracle.silumul(x, FP32)
    want = (g.astype(np.float64) / (1.0 + np.exp(-g.astype(np.float64))) * u.astype(np.float64)).astype(np.float32)
    assert ulp_distance(out, want).max() <= 1            # numpy's exp may differ in the last fp64 bit
    assert (out != want).mean() < 1e-3


@pytest.mark.parametrize("dt,tdt", [(BF16, torch.bfloat16), (FP16, torch.float16)])
def test_against_torch_cpu(oracle, dt, tdt):
    g = torch.Generator().manual_seed(4)
    x = (torch.randn(16, 2 * 256, generator=g) * 2).to(tdt)
    xb = x.view(torch.int16).numpy().view(np.uint16)
    out = oracle.silumul(xb, dt)
    ref = (torch.nn.functional.silu(x[:, :256].double()) * x[:, 256:].double())
    want = ref.float().to(tdt).view(torch.int16).numpy().view(np.uint16)   # fp64 -> fp32 -> 16 bit: may double-round
    dist = ulp_distance(out, want)
    assert dist.max() <= 1 and (dist > 0).mean() < 1e-3


def test_exact_products_with_saturated_gate(oracle):
    """g = 64 makes silu(g) = g exactly, so the outputs are exact products of format values."""
    up = np.array([[1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1.0, 2.0]], np.float32)
    x = _rows(oracle, np.full((1, 4), 64.0, np.float32), up, FP16)
    out = oracle.silumul(x, FP16)
    assert np.array_equal(_dec(oracle, out, FP16), np.array([[64.25, 64.75, 64.0, 128.0]]))


def test_single_rounding_of_the_real_value(oracle):
    """The 16-bit result is the nearest format value to the fp64 product, ties to even, with no
    detour through fp32: checked with exact rationals on the oracle's own fp64 values."""
    rng = np.random.default_rng(8)
    g = (rng.standard_normal((1, 400)) * 3).astype(np.float32)
    u = (rng.standard_normal((1, 400)) * 3).astype(np.float32)
    for dt in (BF16, FP16):
        x = _rows(oracle, g, u, dt)
        real = oracle.silumul_f64(x, dt)
        out = oracle.silumul(x, dt)
        for j in range(400):
            kind, val = round_to_format(Fraction(float(real[0, j])), FMT[dt])
            assert kind == "fin" and bits_to_fraction(int(out[0, j]), FMT[dt]) == val


def test_no_double_rounding_through_fp32(oracle):
    """Cases where the fp64 value rounds to fp32 exactly onto a bf16 tie: going through fp32
    would then round to even, while the real value lies strictly on one side.  The oracle must
    follow the real value."""
    rng = np.random.default_rng(9)
    n = 1 << 21
    g = (rng.standard_normal(n) * 2).astype(np.float32)
    u = (rng.standard_normal(n) * 2).astype(np.float32)
    x = np.ascontiguousarray(np.concatenate([_enc(oracle, g.reshape(1, -1), BF16), _enc(oracle, u.reshape(1, -1), BF16)], axis=1))
    real = oracle.silumul_f64(x, BF16)[0]
    f32 = real.astype(np.float32)
    on_tie = ((f32.view(np.uint32) & 0xffff) == 0x8000) & (f32.astype(np.float64) != real)
    idx = np.nonzero(on_tie)[0]
    assert idx.size >= 5, "sample too small to contain crafted cases"
    out = oracle.silumul(x, BF16)[0]
    differs = 0
    for j in idx.tolist():
        kind, val = round_to_format(Fraction(float(real[j])), "bf16")
        assert bits_to_fraction(int(out[j]), "bf16") == val
        via_f32 = oracle.f32_to_bf16(float(f32[j]))
        differs += int(via_f32 != int(out[j]))
    assert differs >= 1          # the detour through fp32 really would have given another answer somewhere


def test_row_permutation_and_threads(oracle):
    g = torch.Generator().manual_seed(5)
    x = (torch.randn(33, 2 * 128, generator=g)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    a = oracle.silumul(x, BF16, nthreads=1)
    perm = np.random.default_rng(6).permutation(33)
    b = oracle.silumul(np.ascontiguousarray(x[perm]), BF16, nthreads=4)
    assert np.array_equal(b, a[perm])


def test_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.silumul(np.zeros((2, 5), dtype=np.uint16), BF16)
    with pytest.raises(RuntimeError):
        oracle.silumul(np.zeros((2, 4), dtype=np.uint16), 2)         # the mixed format does not exist for this operator
