"""Pins for the oracle's four storage-format routines (CPU only).

Each routine is checked against (a) exact rational rounding written with
Python integers/Fractions, and (b) an independent library conversion: numpy
for binary16, torch CPU for bfloat16.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from exact import bits_to_fraction, fraction_to_bits, round_to_format

ALL16 = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)


def _finite16(fmt):
    if fmt == "f16":
        return ALL16[(ALL16 & 0x7c00) != 0x7c00]
    return ALL16[(ALL16 & 0x7f80) != 0x7f80]


def test_f16_decode_all_patterns(oracle):
    got = oracle.f16_to_f32_array(ALL16)
    want = ALL16.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_bf16_decode_all_patterns(oracle):
    got = oracle.bf16_to_f32_array(ALL16)
    want = torch.from_numpy(ALL16.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_decode_exact_rational(oracle, fmt):
    pats = _finite16(fmt)[::37]
    dec = oracle.f16_to_f32_array(pats) if fmt == "f16" else oracle.bf16_to_f32_array(pats)
    for b, f in zip(pats.tolist(), dec.tolist()):
        assert Fraction(f) == bits_to_fraction(b, fmt)


def _tie_neighbourhood(fmt, oracle):
    """fp32 values at, just below and just above every midpoint between
    adjacent finite values of the format, plus the values themselves."""
    pats = _finite16(fmt)
    pos = pats[(pats & 0x8000) == 0]
    dec = (oracle.f16_to_f32_array(pos) if fmt == "f16" else oracle.bf16_to_f32_array(pos)).astype(np.float64)
    dec = np.sort(dec)
    mid = ((dec[:-1] + dec[1:]) / 2).astype(np.float32)   # exact: one extra bit fits fp32
    pieces = [dec.astype(np.float32), mid,
              np.nextafter(mid, np.float32(-np.inf)), np.nextafter(mid, np.float32(np.inf))]
    top = np.float32(dec[-1])
    if fmt == "f16":   # overflow threshold 65520 and its neighbours
        pieces.append(np.array([65519.996, 65520.0, 65520.004, 65536.0, 1e6, 3.0e38], dtype=np.float32))
    else:
        pieces.append(np.array([top, np.nextafter(top, np.float32(np.inf)), 3.4e38], dtype=np.float32))
    v = np.concatenate(pieces)
    return np.concatenate([v, -v])


def test_f16_encode_vs_numpy(oracle):
    rng = np.random.default_rng(0)
    rand_bits = rng.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    vals = np.concatenate([_tie_neighbourhood("f16", oracle), rand_bits.view(np.float32),
                           (rng.standard_normal(1_000_000) * 3).astype(np.float32),
                           (rng.standard_normal(200_000) * 1e-6).astype(np.float32)])
    vals = vals[~np.isnan(vals)]
    got = oracle.f32_to_f16_array(vals)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)


def test_bf16_encode_vs_torch(oracle):
    rng = np.random.default_rng(1)
    rand_bits = rng.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    vals = np.concatenate([_tie_neighbourhood("bf16", oracle), rand_bits.view(np.float32),
                           (rng.standard_normal(1_000_000) * 3).astype(np.float32)])
    vals = vals[~np.isnan(vals)]
    got = oracle.f32_to_bf16_array(vals)
    want = torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_encode_exact_rational(oracle, fmt):
    """RNE decided with rationals, on tie neighbourhoods and random values."""
    rng = np.random.default_rng(2)
    ties = _tie_neighbourhood(fmt, oracle)
    vals = np.concatenate([ties[rng.integers(0, ties.size, 3000)],
                           (rng.standard_normal(1500) * 2).astype(np.float32),
                           (rng.standard_normal(500) * 1e-5).astype(np.float32),
                           np.array([0.0, -0.0, 65504.0, 65520.0, -65520.0, 2.0 ** -24, 2.0 ** -25,
                                     np.nextafter(np.float32(2.0 ** -25), np.float32(1)),
                                     2.0 ** -14, 2.0 ** -126, 2.0 ** -133, 2.0 ** -134, 1e-45],
                                    dtype=np.float32)])
    enc = oracle.f32_to_f16_array(vals) if fmt == "f16" else oracle.f32_to_bf16_array(vals)
    inf_bits = 0x7c00 if fmt == "f16" else 0x7f80
    for f, b in zip(vals.tolist(), enc.tolist()):
        kind, val = round_to_format(Fraction(f), fmt)
        neg = np.signbit(np.float32(f))
        if kind == "inf":
            assert b == (inf_bits | (0x8000 if neg else 0)), (f, hex(b))
        else:
            assert b == fraction_to_bits(val, fmt, negative_zero=bool(neg) and val == 0) \
                or (val == 0 and b == (0x8000 if neg else 0)), (f, hex(b))


def test_specials(oracle):
    assert oracle.f32_to_f16(float("inf")) == 0x7c00
    assert oracle.f32_to_f16(float("-inf")) == 0xfc00
    assert oracle.f32_to_bf16(float("inf")) == 0x7f80
    assert oracle.f32_to_bf16(float("-inf")) == 0xff80
    assert (oracle.f32_to_f16(float("nan")) & 0x7c00) == 0x7c00 and (oracle.f32_to_f16(float("nan")) & 0x3ff)
    assert (oracle.f32_to_bf16(float("nan")) & 0x7f80) == 0x7f80 and (oracle.f32_to_bf16(float("nan")) & 0x7f)
    assert oracle.f32_to_f16(-0.0) == 0x8000 and oracle.f32_to_bf16(-0.0) == 0x8000


def test_round_trip_identity(oracle):
    for fmt in ("f16", "bf16"):
        pats = _finite16(fmt)
        dec = oracle.f16_to_f32_array(pats) if fmt == "f16" else oracle.bf16_to_f32_array(pats)
        enc = oracle.f32_to_f16_array(dec) if fmt == "f16" else oracle.f32_to_bf16_array(dec)
        assert np.array_equal(enc, pats)
