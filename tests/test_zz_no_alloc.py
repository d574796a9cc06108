"""addrms_gate_probe_noalloc (the entry point for callers that cannot allocate) must give the verdict of
addrms_gate_probe, call after call, although every call on the GPU reuses one scratch array that keeps the
previous call's contents."""
import numpy as np
import pytest
import torch

from paper_2601_12698_amd import binding as B

pytestmark = pytest.mark.gpu

X_T = {"bf16": torch.bfloat16, "fp16_res32": torch.float16, "fp32": torch.float32}
R_T = {"bf16": torch.bfloat16, "fp16_res32": torch.float32, "fp32": torch.float32}


def planted(dtype, n, seed, n_rbad, n_y1, n_y3):
    """A reference pair and a copy with n_rbad residual bit flips, n_y1 y elements one step off and n_y3 three steps off."""
    g = torch.Generator().manual_seed(seed)
    y_ref = (torch.randn(n, generator=g) * 2 + 5).to(X_T[dtype])        # positive: bit pattern + k is k steps
    r_ref = torch.randn(n, generator=g).to(R_T[dtype])
    y, r = y_ref.clone(), r_ref.clone()
    idx = torch.randperm(n, generator=g)
    iv = (lambda t: t.view(torch.int16) if t.element_size() == 2 else t.view(torch.int32))
    iv(r)[idx[:n_rbad]] ^= 4
    iv(y)[idx[n_rbad:n_rbad + n_y1]] += 1
    iv(y)[idx[n_rbad + n_y1:n_rbad + n_y1 + n_y3]] += 3
    iv(y)[n - 1] += 3                                                    # and the very last element
    return tuple(t.cuda() for t in (y, y_ref, r, r_ref))


def counts(fn, args, dtype, tol):
    out = torch.full((4,), 0x5a5a5a5a, dtype=torch.int32, device="cuda")
    fn(*args, dtype, tol, out)
    torch.cuda.synchronize()
    return tuple(int(v) & 0xffffffff for v in out.cpu().tolist())


@pytest.mark.parametrize("dtype", ["bf16", "fp16_res32", "fp32"])
def test_no_alloc_gate_matches_the_allocating_gate_on_consecutive_calls(dtype):
    big = planted(dtype, 20_000_003, 1, 1234, 77, 55)       # 4096 workgroups: every scratch slot is written
    small = planted(dtype, 100_001, 2, 3, 5, 2)             # 25 workgroups: most slots keep the big call's counts
    tiny = planted(dtype, 1, 3, 0, 0, 0)
    for tol in (1, 0):
        for args in (big, small, tiny, small, big):         # the second and third calls are smaller than the one before
            want = counts(B.addrms_gate_probe, args, dtype, tol)
            got = counts(B.addrms_gate_probe_noalloc, args, dtype, tol)
            assert got == want, (dtype, tol, args[0].numel(), got, want)
    # what the planted mistakes must add up to (checks the reference entry point itself on this input)
    assert counts(B.addrms_gate_probe_noalloc, small, dtype, 1) == (3, 3, 3, 0)      # 2 planted + the last element
    assert counts(B.addrms_gate_probe_noalloc, small, dtype, 0) == (3, 8, 3, 0)
    assert counts(B.addrms_gate_probe_noalloc, big, dtype, 1) == (1234, 56, 3, 0)


def test_no_alloc_gate_back_to_back_without_waiting():
    """Calls on one stream are ordered: enqueue several without synchronising, each with its own output."""
    big = planted("bf16", 3_000_001, 7, 11, 0, 4)
    small = planted("bf16", 5_003, 8, 2, 1, 0)
    outs = [torch.zeros(4, dtype=torch.int32, device="cuda") for _ in range(4)]
    for out, args in zip(outs, (big, small, big, small)):
        B.addrms_gate_probe_noalloc(*args, "bf16", 1, out)
    torch.cuda.synchronize()
    got = [tuple(o.cpu().tolist()) for o in outs]
    assert got[0] == got[2] == (11, 5, 3, 0)
    assert got[1] == got[3] == (2, 1, 3, 0)


def test_no_alloc_gate_rejects_what_it_cannot_count():
    y = torch.zeros(8, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(4, dtype=torch.int32, device="cuda")
    lib = B.load()
    p = y.data_ptr()
    assert lib.addrms_gate_probe_noalloc(p, p, p, p, 1 << 32, B.BF16, 1, out.data_ptr(), None) == B.ERR_INVALID_ARG
    assert "32-bit counters" in B.addrms_last_error()
    assert lib.addrms_gate_probe_noalloc(p, p, p, p, 8, B.BF16, 1, None, None) == B.ERR_INVALID_ARG
    out.fill_(9)
    assert lib.addrms_gate_probe_noalloc(None, None, None, None, 0, B.BF16, 1, out.data_ptr(), None) == B.OK
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [0, 0, 0, 0]
