"""addrms_run under HIP graph capture (needs an MI355X).

The run entry point neither synchronises nor allocates, so a launch-bound decode loop
can be captured once and replayed.  A chain of launches (the output of one is the input
of the next, as across the layers of a decoder) is captured with the restoring copies,
replayed several times with eager work and synchronisations in between, and every replay
is compared with the eager chain and with the CPU oracle applied the same number of times.
"""
import numpy as np
import pytest
import torch

from gpu_util import compare
from paper_2601_12698_amd import binding as B
from paper_2601_12698_amd import workloads as W

pytestmark = pytest.mark.gpu

CHAIN = 3


def _cfgs(M, N, dtype):
    out = [("default", B.addrms_default_cfg(N, dtype))]
    feas, _ = B.addrms_enumerate_feasible(M, N, dtype)
    pick = {}
    for c in feas:
        if c.flags == 3 and c.max_waves_per_simd == 0 and c.rows_per_wg == 2:
            pick.setdefault("streaming_xcd", c)
        if c.max_waves_per_simd == 2 and c.threads_per_row == 256:
            pick.setdefault("capped", c)            # padded LDS allocation above 64 KB
        if c.reduce == 1 and c.threads_per_row == 512 and c.flags == 0 and c.max_waves_per_simd == 0:
            pick.setdefault("lds_tree", c)
    return out + sorted(pick.items())


@pytest.mark.parametrize("M,N,dtype", [(64, 8192, "bf16"), (16, 4096, "fp16_res32")])
def test_captured_chain_replays_like_eager(oracle, M, N, dtype):
    wl = W.Workload(f"graph_{M}x{N}_{dtype}", M, N, dtype, 1e-5, 77, x_std=2.0, r_std=2.0)
    d = W.generate(wl)
    dev = torch.device("cuda:0")
    x0, r0, w = d["x"].to(dev), d["r"].to(dev), d["w"].to(dev)
    x, r = torch.empty_like(x0), torch.empty_like(r0)
    # oracle applied CHAIN times (each application takes the previous outputs as inputs)
    xb, rb, wb = W.to_bits(d["x"]), W.to_bits(d["r"]), W.to_bits(d["w"])
    for _ in range(CHAIN):
        xb, rb = oracle.addrms(xb, rb, wb, wl.eps, B.DTYPE_IDS[dtype], nthreads=8)
    cases = _cfgs(M, N, dtype)
    assert len(cases) >= 3
    for name, cfg in cases:
        def chain():
            x.copy_(x0)
            r.copy_(r0)
            for _ in range(CHAIN):
                B.addrms_run(x, r, w, wl.eps, M, N, dtype, cfg)
        chain()                                   # eager (also performs any one-time kernel attribute set-up)
        torch.cuda.synchronize()
        y_eager, r_eager = W.to_bits(x), W.to_bits(r)
        assert compare(y_eager, r_eager, xb, rb, dtype, f"eager chain {name}")["n_diff"] == 0
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            chain()
        torch.cuda.synchronize()
        for rep in range(4):
            x.fill_(1.0)                          # eager work between replays: clobber the buffers
            r.fill_(-1.0)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            y, rr = W.to_bits(x), W.to_bits(r)
            assert np.array_equal(y, y_eager) and np.array_equal(rr, r_eager), f"{name}: replay {rep} differs from eager"
        del g
