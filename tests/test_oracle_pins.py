"""Pins for the oracle's operator (CPU only): exact brute force, closed forms,
exact invariants, agreement of the summation variants, and an independent
torch-CPU evaluation.  Together they are chosen so that a dropped term, a
wrong sign or index, a transposed operand, eps in the wrong place, the wrong
multiply order or normalising the rounded sum instead of the unrounded one
fails at least one test.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from exact import (bits_to_fraction, fraction_to_bits, f32_fraction,
                   is_correctly_rounded_rsqrt, round_to_format)
from ulp import ulp_distance
from paper_2601_12698_amd import workloads as W

DT = {"bf16": 0, "fp16": 1, "fp16_res32": 2, "fp32": 3}


def _gen(M, N, dtype, seed, eps=1e-6, **kw):
    wl = W.Workload("t", M, N, dtype, eps, seed, **kw)
    d = W.generate(wl)
    return W.to_bits(d["x"]), W.to_bits(d["r"]), W.to_bits(d["w"]), d


def _fmt16(dtype):
    return "bf16" if dtype == "bf16" else "f16"


def _to_frac(bits, dtype, which):
    """Exact value of one stored element (which: 'x' or 'r')."""
    is32 = dtype == "fp32" or (which == "r" and dtype == "fp16_res32")
    if is32:
        return Fraction(float(bits))
    return bits_to_fraction(int(bits), _fmt16(dtype))


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp16_res32", "fp32"])
@pytest.mark.parametrize("seed,N", [(0, 16), (1, 5), (2, 12)])
def test_exact_rational_brute_force(oracle, dtype, seed, N):
    M = 3
    eps = 1e-6
    xb, rb, wb, _ = _gen(M, N, dtype, seed, eps=eps, x_std=1.5, r_std=0.7)
    y, res, rstd = oracle.addrms(xb, rb, wb, eps, DT[dtype], return_rstd=True)
    eps_q = f32_fraction(np.float32(eps))
    x_out_fmt = "f32" if dtype == "fp32" else _fmt16(dtype)
    r_out_fmt = "f32" if dtype in ("fp32", "fp16_res32") else _fmt16(dtype)
    for i in range(M):
        h = []
        for j in range(N):
            kind, hj = round_to_format(_to_frac(xb[i, j], dtype, "x") + _to_frac(rb[i, j], dtype, "r"), "f32")
            assert kind == "fin"
            h.append(hj)
            kind, rj = round_to_format(hj, r_out_fmt)
            got = res[i, j]
            got_q = Fraction(float(got)) if r_out_fmt == "f32" else bits_to_fraction(int(got), r_out_fmt)
            assert got_q == rj, ("residual", i, j)
        D = sum(v * v for v in h) / N + eps_q
        f = Fraction(float(rstd[i]))
        assert is_correctly_rounded_rsqrt(f, D), ("rstd", i)
        for j in range(N):
            _, t = round_to_format(h[j] * f, "f32")
            _, v = round_to_format(t * _to_frac(wb[j], dtype, "x"), "f32")
            _, yq = round_to_format(v, x_out_fmt)
            got = y[i, j]
            got_q = Fraction(float(got)) if x_out_fmt == "f32" else bits_to_fraction(int(got), x_out_fmt)
            assert got_q == yq, ("y", i, j)


def test_residual_rounding_all_bf16_x_against_sampled_r(oracle):
    """residual_out == RNE_bf16(RNE_f32(x + r)) for every finite bf16 x against
    sampled r, decided with exact rationals; and the double rounding equals the
    single rounding of the exact sum on these inputs."""
    rng = np.random.default_rng(5)
    pats = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    fin = pats[(pats & 0x7f80) != 0x7f80]
    # keep magnitudes where the sum cannot overflow
    fin = fin[((fin & 0x7f80) >> 7) < 0xf0]
    x = fin.reshape(1, -1)
    for trial in range(2):
        r = fin[rng.integers(0, fin.size, fin.size)].reshape(1, -1)
        w = np.full((x.shape[1],), 0x3f80, dtype=np.uint16)
        _, res = oracle.addrms(x, r, w, 1e-6, 0)
        idx = rng.integers(0, fin.size, 4000)
        for j in idx.tolist():
            s = bits_to_fraction(int(x[0, j]), "bf16") + bits_to_fraction(int(r[0, j]), "bf16")
            _, s32 = round_to_format(s, "f32")
            _, want = round_to_format(s32, "bf16")
            assert bits_to_fraction(int(res[0, j]), "bf16") == want
            _, single = round_to_format(s, "bf16")
            assert single == want


def test_residual_rounding_all_pairs_in_binades(oracle):
    """All pairs of bf16 values from two adjacent binades (and mixed signs):
    residual_out vs torch CPU's independent add-then-round."""
    a = np.arange(0x3f80, 0x4080, dtype=np.uint16)          # [1, 4): 256 values
    vals = np.concatenate([a, a | 0x8000])
    X, R = np.meshgrid(vals, vals, indexing="ij")
    x = np.ascontiguousarray(X.reshape(1, -1))
    r = np.ascontiguousarray(R.reshape(1, -1))
    w = np.full((x.shape[1],), 0x3f80, dtype=np.uint16)
    _, res = oracle.addrms(x, r, w, 1e-6, 0)
    tx = torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).float()
    tr = torch.from_numpy(r.view(np.int16).copy()).view(torch.bfloat16).float()
    want = (tx + tr).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(res, want)


# ---------------------------------------------------------------- closed forms
def test_unit_weight_rms_closed_form(oracle):
    """With w = 1, RMS(y64 row) = sqrt(ms / (ms + eps)) exactly, which is
    1 - eps/(2 ms) to first order: within 1e-6 of 1 on unit-scale rows."""
    eps = 1e-6
    xb, rb, _, d = _gen(8, 512, "bf16", 11, eps=eps)
    w1 = np.full((512,), 0x3f80, dtype=np.uint16)
    y64 = oracle.addrms_y64(xb, rb, w1, eps, 0)
    h = d["x"].double().numpy() + d["r"].double().numpy()
    ms = (h * h).mean(axis=1)
    rms = np.sqrt((y64 * y64).mean(axis=1))
    assert np.allclose(rms, np.sqrt(ms / (ms + eps)), rtol=1e-12, atol=0)
    assert np.all(np.abs(rms - 1.0) < 1e-6)
    # the rounded bf16 output has RMS 1 up to its own rounding error
    y, _ = oracle.addrms(xb, rb, w1, eps, 0)
    yf = oracle.bf16_to_f32_array(y).astype(np.float64)
    assert np.all(np.abs(np.sqrt((yf * yf).mean(axis=1)) - 1.0) < 2e-3)


def test_tiny_rows_follow_closed_form_not_unit_rms(oracle):
    """For ms comparable to eps the RMS is sqrt(ms/(ms+eps)), far from 1."""
    eps = 1e-6
    N = 64
    x = np.full((1, N), oracle.f32_to_bf16(2.0 ** -10), dtype=np.uint16)
    r = np.zeros((1, N), dtype=np.uint16)
    w1 = np.full((N,), 0x3f80, dtype=np.uint16)
    y64 = oracle.addrms_y64(x, r, w1, eps, 0)
    ms = 2.0 ** -20
    assert math.isclose(math.sqrt((y64 ** 2).mean()), math.sqrt(ms / (ms + eps)), rel_tol=1e-12)


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
def test_constant_row(oracle, dtype):
    """h = c everywhere: y_j = c / sqrt(c^2 + eps) * w_j."""
    N, eps = 96, 1e-3
    _, _, wb, d = _gen(1, N, dtype, 3)
    enc = {"bf16": oracle.f32_to_bf16_array, "fp16": oracle.f32_to_f16_array,
           "fp32": lambda a: np.asarray(a, dtype=np.float32)}[dtype]
    x = enc(np.full((1, N), 1.5, dtype=np.float32))
    r = enc(np.full((1, N), -0.25, dtype=np.float32))
    y, res, rstd = oracle.addrms(x, r, wb, eps, DT[dtype], return_rstd=True)
    c = 1.25
    assert rstd[0] == np.float32(1.0 / math.sqrt(c * c + np.float32(eps).astype(np.float64)))
    wf = d["w"].float().numpy()
    want32 = (np.float32(c) * rstd[0]) * wf
    want = enc(want32)
    assert np.array_equal(y[0], want)
    assert np.array_equal(res, enc(np.full((1, N), c, dtype=np.float32)))


def test_one_hot_row(oracle):
    """h = a e_k with N = 4096: y_k = a / sqrt(a^2/4096 + eps) * w_k, about
    64 w_k; every other output is an exact zero."""
    N, k, eps = 4096, 1234, 1e-6
    x = np.zeros((1, N), dtype=np.uint16)
    r = np.zeros((1, N), dtype=np.uint16)
    x[0, k] = oracle.f32_to_bf16(3.0)
    _, _, wb, d = _gen(1, N, "bf16", 4)
    y, res = oracle.addrms(x, r, wb, eps, 0)
    others = np.delete(y[0], k)
    assert np.all(others == 0)
    wk = float(d["w"].float()[k])
    want = 3.0 / math.sqrt(9.0 / 4096 + float(np.float32(eps))) * wk
    got = float(oracle.bf16_to_f32(int(y[0, k])))
    assert abs(got - want) <= 2.0 ** -8 * abs(want)           # half a bf16 ulp, relative
    assert abs(got / wk - 64.0) < 0.3
    assert res[0, k] == x[0, k] and np.all(np.delete(res[0], k) == 0)


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp16_res32", "fp32"])
def test_zero_row(oracle, dtype):
    N = 40
    _, _, wb, _ = _gen(1, N, dtype, 6)
    xz = np.zeros((2, N), dtype=np.float32 if dtype == "fp32" else np.uint16)
    rz = np.zeros((2, N), dtype=np.float32 if dtype in ("fp32", "fp16_res32") else np.uint16)
    y, res, rstd = oracle.addrms(xz, rz, wb, 1e-6, DT[dtype], return_rstd=True)
    assert np.all(np.isfinite(rstd)) and rstd[0] == np.float32(1.0 / math.sqrt(float(np.float32(1e-6))))
    assert np.all(y == 0) and np.all(res == 0)


def test_rstd_canonical_is_correctly_rounded(oracle):
    rng = np.random.default_rng(9)
    for N in (1000, 4096, 7168):
        for ss in np.exp(rng.uniform(-20, 25, 60)):
            eps = np.float32(1e-6)
            f = oracle.rstd_canonical(float(ss), N, float(eps))
            D = Fraction(float(ss)) / N + f32_fraction(eps)
            # ss/N is rounded once in fp64 inside the oracle; the exact test
            # tolerates that because fp64 error is 2^29 times finer than fp32
            assert is_correctly_rounded_rsqrt(Fraction(float(f)), D)


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("dtype", ["bf16", "fp16_res32"])
@pytest.mark.parametrize("variant", ["canonical", "seq32", "pair32"])
def test_row_permutation_invariance(oracle, dtype, variant):
    xb, rb, wb, _ = _gen(37, 200, dtype, 12)
    y, res = oracle.addrms(xb, rb, wb, 1e-6, DT[dtype], variant=variant)
    perm = np.random.default_rng(0).permutation(37)
    y2, res2 = oracle.addrms(xb[perm], rb[perm], wb, 1e-6, DT[dtype], variant=variant, nthreads=3)
    assert np.array_equal(y2.view(np.uint8), y[perm].view(np.uint8))
    assert np.array_equal(res2.view(np.uint8), res[perm].view(np.uint8))


def _negate(bits):
    if bits.dtype == np.uint16:
        return bits ^ np.uint16(0x8000)
    return -bits


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp16_res32", "fp32"])
def test_negation_symmetry(oracle, dtype):
    xb, rb, wb, _ = _gen(5, 333, dtype, 13)
    y, res = oracle.addrms(xb, rb, wb, 1e-6, DT[dtype])
    y2, res2 = oracle.addrms(_negate(xb), _negate(rb), wb, 1e-6, DT[dtype])
    assert np.array_equal(_negate(y2).view(np.uint8), y.view(np.uint8))
    assert np.array_equal(_negate(res2).view(np.uint8), res.view(np.uint8))


@pytest.mark.parametrize("k", [-3, 4])
def test_power_of_two_scaling(oracle, k):
    """(2^k x, 2^k r, 4^k eps) gives the same y bits and 2^k-scaled residual."""
    xb, rb, wb, _ = _gen(6, 256, "bf16", 14)
    eps = 2.0 ** -20
    y, res = oracle.addrms(xb, rb, wb, eps, 0)
    shift = np.uint16((k << 7) & 0xffff)
    assert np.all(((xb >> 7) & 0xff) > 8) and np.all(((rb >> 7) & 0xff) > 8)   # normals stay normal
    y2, res2 = oracle.addrms(xb + shift, rb + shift, wb, eps * 4.0 ** k, 0)
    assert np.array_equal(y2, y)
    nz = (res & 0x7fff) != 0
    assert np.array_equal(res2[nz], (res + shift)[nz])


def test_column_permutation(oracle):
    xb, rb, wb, _ = _gen(9, 384, "bf16", 15)
    perm = np.random.default_rng(1).permutation(384)
    y, res = oracle.addrms(xb, rb, wb, 1e-6, 0)
    y2, res2 = oracle.addrms(xb[:, perm].copy(), rb[:, perm].copy(), wb[perm].copy(), 1e-6, 0)
    # fp64 left-to-right sums in two orders differ by ~1e-16 relative, which
    # moves the fp32 rstd with probability ~1e-8 per row: equal bits expected
    assert np.array_equal(y2, y[:, perm]) and np.array_equal(res2, res[:, perm])
    y3, _ = oracle.addrms(xb[:, perm].copy(), rb[:, perm].copy(), wb[perm].copy(), 1e-6, 0, variant="seq32")
    assert ulp_distance(y3, y[:, perm]).max() <= 1


@pytest.mark.parametrize("dtype,N", [("bf16", 4096), ("fp16", 1000), ("fp16_res32", 2880), ("fp32", 1536)])
def test_variants_agree_within_one_ulp(oracle, dtype, N):
    xb, rb, wb, _ = _gen(24, N, dtype, 16)
    y0, r0, s0 = oracle.addrms(xb, rb, wb, 1e-6, DT[dtype], return_rstd=True)
    for v in ("seq32", "pair32"):
        y1, r1, s1 = oracle.addrms(xb, rb, wb, 1e-6, DT[dtype], variant=v, return_rstd=True)
        assert np.array_equal(r0.view(np.uint8), r1.view(np.uint8))
        # a left-to-right fp32 sum of N terms is off by about sqrt(N) roundings
        # (worst case N), a pairwise tree by about log2(N); rstd halves that
        s_bound = 64 if v == "seq32" else 8
        assert ulp_distance(s0, s1).max() <= s_bound
        if dtype == "fp32":
            assert ulp_distance(y1, y0).max() <= s_bound + 2   # fp32 output sees rstd's last bits
        else:
            assert ulp_distance(y1, y0).max() <= 1


# ---------------------------------------------------------------- library special case
@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp16_res32"])
def test_against_torch_cpu(oracle, dtype):
    """Independent evaluation with torch CPU ops: fp32 add, storage rounding by
    torch's own casts, mean of squares in fp64, rsqrt rounded to fp32."""
    eps = 1e-6
    xb, rb, wb, d = _gen(33, 1000, dtype, 17, eps=eps)
    y, res = oracle.addrms(xb, rb, wb, eps, DT[dtype])
    h = d["x"].float() + d["r"].float()
    want_res = W.to_bits(h.to(d["r"].dtype))
    assert np.array_equal(res.view(np.uint8), want_res.view(np.uint8))
    ms = h.double().pow(2).mean(dim=1, keepdim=True)
    rstd = (1.0 / torch.sqrt(ms + float(np.float32(eps)))).float()
    want_y = W.to_bits(((h * rstd) * d["w"].float()).to(d["x"].dtype))
    dist = ulp_distance(y, want_y)
    assert dist.max() <= 1 and (dist > 0).mean() < 1e-3


def test_uses_unrounded_sum_for_normalisation(oracle):
    """y is computed from the fp32 sum, not from the rounded residual_out.  Every element has x = 1 and
    r = 2^-9, so h = 1 + 2^-9 in fp32 (not a bf16 value; residual_out rounds to 1.0, tie to even) and, with
    w = 1, the two readings land in different bf16 cells:
        unrounded h:  y = h * rstd = 1 / sqrt(1 + eps / h^2) = 1 - 5e-7      -> bf16 1.0          (0x3f80)
        rounded h:    y = 1 * rstd = 1 / sqrt(h^2 + eps)     = 0.998050...   -> bf16 1 - 2^-9     (0x3f7f)
    (bf16 values just below 1 are 2^-9 apart: 0.998046875 and 1.0; the midpoint is 0.9990234375.)"""
    N = 8
    one, tiny = 0x3f80, 0x3b00                      # bf16 bit patterns of 1.0 and 2^-9
    x = np.full((1, N), one, dtype=np.uint16)
    r = np.full((1, N), tiny, dtype=np.uint16)
    w = np.full((N,), one, dtype=np.uint16)
    y, res, rstd = oracle.addrms(x, r, w, 1e-6, 0, return_rstd=True)
    assert np.all(res == one)
    h = 1.0 + 2.0 ** -9
    exact_rstd = 1.0 / math.sqrt(h * h + float(np.float32(1e-6)))
    assert rstd[0] == np.float32(exact_rstd)
    want_value, alt_value = h * exact_rstd, 1.0 * exact_rstd
    midpoint = 1.0 - 2.0 ** -10
    assert alt_value < midpoint - 1e-4 and want_value > midpoint + 1e-4     # the two readings are far from the boundary
    want, alt = one, 0x3f7f
    assert want != alt
    assert np.all(y == want), [hex(v) for v in y.ravel()]


def test_threads_do_not_change_results(oracle):
    xb, rb, wb, _ = _gen(64, 300, "bf16", 18)
    a = oracle.addrms(xb, rb, wb, 1e-6, 0, nthreads=1)
    b = oracle.addrms(xb, rb, wb, 1e-6, 0, nthreads=8)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
