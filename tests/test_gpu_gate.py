"""The correctness gate (Algorithm 1 line 13, Validate; Section 3.1: d(S~(x), S(x)) <= eps) must reject what it
is meant to reject.  Every kernel here exits normally; the mistakes are planted in the data the gate compares."""
import numpy as np
import pytest
import torch

from paper_2601_12698_amd import binding as B

pytestmark = pytest.mark.gpu

X_T = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp16_res32": torch.float16, "fp32": torch.float32}
R_T = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp16_res32": torch.float32, "fp32": torch.float32}


def int_view(t):
    return t.view(torch.int16) if t.element_size() == 2 else t.view(torch.int32)


def make_pair(dtype, n, seed):
    g = torch.Generator().manual_seed(seed)
    y = (torch.randn(n, generator=g) * 3).to(X_T[dtype])
    r = torch.randn(n, generator=g).to(R_T[dtype])
    y[y == 0] = 1                                        # keep the planted one-step moves inside one sign
    return y.cuda(), r.cuda()


def step_ulps(t, idx, k):
    """Moves element idx of t by k units in the last place, away from zero (bit pattern + k)."""
    v = int_view(t)
    v[idx] += k


def run_gate(y, y_ref, r, r_ref, dtype, tol):
    out = torch.full((4,), -1, dtype=torch.int32, device="cuda")
    B.addrms_gate_probe(y, y_ref, r, r_ref, dtype, tol, out)
    c = out.cpu().numpy().astype(np.int64) & 0xffffffff
    assert c[3] == 0
    return int(c[0]), int(c[1]), int(c[2])


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp16_res32", "fp32"])
@pytest.mark.parametrize("n", [1, 255, 4097, 1_000_003])     # none but 1 is a multiple of the workgroup size
def test_gate_counts_planted_mismatches(dtype, n):
    y_ref, r_ref = make_pair(dtype, n, seed=n)
    y, r = y_ref.clone(), r_ref.clone()
    assert run_gate(y, y_ref, r, r_ref, dtype, 1) == (0, 0, 0)

    # one flipped residual bit, in the last element
    int_view(r)[n - 1] ^= 1
    assert run_gate(y, y_ref, r, r_ref, dtype, 1) == (1, 0, 0)
    assert run_gate(y, y_ref, r, r_ref, dtype, 0) == (1, 0, 0)
    int_view(r)[n - 1] ^= 1

    # y one unit off in the last element: passes at tol 1, fails at tol 0
    step_ulps(y, n - 1, 1)
    assert run_gate(y, y_ref, r, r_ref, dtype, 1) == (0, 0, 1)
    assert run_gate(y, y_ref, r, r_ref, dtype, 0) == (0, 1, 1)
    # two units off: fails at tol 1
    step_ulps(y, n - 1, 1)
    assert run_gate(y, y_ref, r, r_ref, dtype, 1) == (0, 1, 2)
    step_ulps(y, n - 1, -2)
    assert run_gate(y, y_ref, r, r_ref, dtype, 0) == (0, 0, 0)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_gate_treats_signed_zeros_as_equal_and_counts_every_element(dtype):
    n = 70_001
    y_ref, r_ref = make_pair(dtype, n, seed=5)
    y_ref[17] = 0.0
    y_ref[n - 1] = -0.0
    y, r = y_ref.clone(), r_ref.clone()
    y[17] = -0.0
    y[n - 1] = 0.0
    assert run_gate(y, y_ref, r, r_ref, dtype, 0) == (0, 0, 0)
    # +0 against the smallest subnormal of the other sign is one step, not a sign-bit-sized jump
    int_view(y)[17] = -32767 if y.element_size() == 2 else -2147483647      # sign bit + 1: the smallest negative subnormal
    assert run_gate(y, y_ref, r, r_ref, dtype, 0) == (0, 1, 1)
    # everything wrong: the counts are exact, not saturated or sampled
    r2 = r_ref.clone()
    int_view(r2)[:] ^= 1
    y_ref[17] = 1.0
    y_ref[n - 1] = 1.0                  # no zeros left: every element is exactly three steps away
    y2 = y_ref.clone()
    int_view(y2)[:] += 3
    assert run_gate(y2, y_ref, r2, r_ref, dtype, 1) == (n, n, 3)
    assert run_gate(y2, y_ref, r2, r_ref, dtype, 3) == (n, 0, 3)


def test_gate_rejects_outputs_of_another_eps_through_the_run_path():
    """End to end: the operator run with a different eps differs from the reference run, and the gate says so."""
    from paper_2601_12698_amd import workloads as W
    wl = W.SMOKE
    d = W.generate(wl)
    x0, r0, w = d["x"].cuda(), d["r"].cuda(), d["w"].cuda()
    outs = []
    for eps in (wl.eps, 1.0):                  # mean square is about 2: rstd moves by a fifth
        x, r = x0.clone(), r0.clone()
        B.addrms_run(x, r, w, eps, wl.M, wl.N, wl.dtype)
        outs.append((x, r))
    torch.cuda.synchronize()
    (ya, ra), (yb, rb) = outs
    rbad, ybad, ymax = run_gate(yb.view(-1), ya.view(-1), rb.view(-1), ra.view(-1), wl.dtype, 1)
    assert rbad == 0                     # the residual does not depend on eps
    assert ybad > 0 and ymax > 1         # the normalised output does
    assert run_gate(ya.view(-1), ya.view(-1), ra.view(-1), ra.view(-1), wl.dtype, 0) == (0, 0, 0)


def test_gate_argument_errors():
    y = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(4, dtype=torch.int32, device="cuda")
    lib = B.load()
    assert lib.addrms_gate_probe(y.data_ptr(), y.data_ptr(), y.data_ptr(), y.data_ptr(), -1, B.BF16, 1, out.data_ptr(), None) == B.ERR_INVALID_ARG
    assert lib.addrms_gate_probe(y.data_ptr(), y.data_ptr(), y.data_ptr(), y.data_ptr(), 1 << 32, B.BF16, 1, out.data_ptr(), None) == B.ERR_INVALID_ARG
    assert "32-bit counters" in B.addrms_last_error()
    assert lib.addrms_gate_probe(y.data_ptr(), y.data_ptr(), y.data_ptr(), y.data_ptr(), 8, 9, 1, out.data_ptr(), None) == B.ERR_UNSUPPORTED_DTYPE
    assert lib.addrms_gate_probe(None, y.data_ptr(), y.data_ptr(), y.data_ptr(), 8, B.BF16, 1, out.data_ptr(), None) == B.ERR_INVALID_ARG
    assert lib.addrms_gate_probe(y.data_ptr(), y.data_ptr(), y.data_ptr(), y.data_ptr(), 8, B.BF16, 1, None, None) == B.ERR_INVALID_ARG
    assert lib.addrms_gate_probe(y.data_ptr() + 1, y.data_ptr(), y.data_ptr(), y.data_ptr(), 4, B.BF16, 1, out.data_ptr(), None) == B.ERR_MISALIGNED
    # n == 0: a successful no-op that reports nothing wrong
    out.fill_(7)
    assert lib.addrms_gate_probe(None, None, None, None, 0, B.BF16, 1, out.data_ptr(), None) == B.OK
    assert out.cpu().tolist() == [0, 0, 0, 0]
