"""The row-holding copy probe: moves exactly the operator's bytes and nothing else."""
import pytest
import torch

from paper_2601_12698_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,M,N,threads,wgs", [
    ("bf16", 37, 7168, 448, 3),        # two pieces per thread, exact cover
    ("bf16", 5, 7168, 1024, 0),        # one piece per thread, idle tail lanes
    ("fp16", 9, 1000, 64, 2),          # 125 pieces over 64 threads: ragged last chunk
    ("fp16_res32", 11, 5120, 256, 1),  # fp32 residual: two residual pieces per x piece
    ("fp32", 3, 4096, 64, 16),         # sixteen pieces per thread
])
def test_row_probe_complements_both_streams_and_nothing_else(dtype, M, N, threads, wgs):
    xt = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp16_res32": torch.float16, "fp32": torch.float32}[dtype]
    rt = torch.float32 if dtype in ("fp16_res32", "fp32") else xt
    g = torch.Generator().manual_seed(5)
    guard = 64
    xbuf = torch.randn(M * N + 2 * guard, generator=g).to(xt).cuda()
    rbuf = torch.randn(M * N + 2 * guard, generator=g).to(rt).cuda()
    x, r = xbuf[guard:guard + M * N], rbuf[guard:guard + M * N]
    x0, r0 = xbuf.clone(), rbuf.clone()
    B.addrms_row_probe(x, r, M, N, dtype, threads, wgs)
    torch.cuda.synchronize()
    as_int = lambda t: t.view(torch.int16 if t.element_size() == 2 else torch.int32)
    assert torch.equal(as_int(x), ~as_int(x0[guard:guard + M * N]))
    assert torch.equal(as_int(r), ~as_int(r0[guard:guard + M * N]))
    for buf, ref in ((xbuf, x0), (rbuf, r0)):                                   # nothing outside [M, N] is touched
        assert torch.equal(as_int(buf[:guard]), as_int(ref[:guard]))
        assert torch.equal(as_int(buf[-guard:]), as_int(ref[-guard:]))
    B.addrms_row_probe(x, r, M, N, dtype, threads, wgs)                          # twice = identity
    torch.cuda.synchronize()
    assert torch.equal(as_int(xbuf), as_int(x0)) and torch.equal(as_int(rbuf), as_int(r0))


def test_row_probe_refuses_shapes_it_cannot_cover():
    x = torch.zeros(4 * 7168, dtype=torch.bfloat16, device="cuda")
    r = torch.zeros_like(x)
    with pytest.raises(B.AddrmsError):
        B.addrms_row_probe(x, r, 4, 7168, "bf16", 100, 0)          # not whole waves
    with pytest.raises(B.AddrmsError):
        B.addrms_row_probe(x, r, 2, 14336, "bf16", 64, 0)          # 28 pieces per thread
    with pytest.raises(B.AddrmsError):
        B.addrms_row_probe(x[:4 * 7164], r[:4 * 7164], 4, 7164, "bf16", 448, 0)   # rows of 14,328 bytes
