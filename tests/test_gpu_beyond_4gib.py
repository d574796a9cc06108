"""Tensors larger than 4 GiB: the byte offset of a row no longer fits 32 bits (needs an MI355X).

The input is one seeded block of B rows tiled T times on the device, with B chosen so that
2^32 bytes is not a whole number of blocks: an address that wrapped at 32 bits would land on
a different row of the block (or between rows), and both the row it failed to write and the
row it overwrote would differ from the expected tile.  Every tile of the output is compared,
on the device, with the oracle's output for the block.
"""
import numpy as np
import pytest
import torch

from paper_2601_12698_amd import binding as B
from paper_2601_12698_amd import workloads as W

pytestmark = pytest.mark.gpu


def _tiles_equal(out2d, ref_block_bits_dev, tiles, rows):
    got = out2d.view(torch.int16 if out2d.element_size() == 2 else torch.int32).view(tiles, rows, -1)
    bad = 0
    for t in range(tiles):                       # tile by tile: no multi-gigabyte temporary
        bad += int((got[t] != ref_block_bits_dev).sum())
    return bad


def test_addrms_rows_beyond_4gib(oracle):
    rows, tiles, N, dtype = 4099, 75, 8192, "bf16"
    M = rows * tiles
    row_bytes = N * 2
    assert M * row_bytes > 2 ** 32 and (2 ** 32) % (rows * row_bytes) != 0 and (2 ** 32 // row_bytes) % rows != 0
    wl = W.Workload("block_4099x8192_bf16", rows, N, dtype, 1e-6, 404)
    d = W.generate(wl)
    y_ref, r_ref = oracle.addrms(W.to_bits(d["x"]), W.to_bits(d["r"]), W.to_bits(d["w"]), wl.eps, B.DTYPE_IDS[dtype],
                                 nthreads=16)
    dev = torch.device("cuda:0")
    xb, rb, w = d["x"].to(dev), d["r"].to(dev), d["w"].to(dev)
    y_ref_d = torch.from_numpy(y_ref.view(np.int16)).to(dev)
    r_ref_d = torch.from_numpy(r_ref.view(np.int16)).to(dev)
    x = torch.empty((M, N), dtype=xb.dtype, device=dev)
    r = torch.empty((M, N), dtype=rb.dtype, device=dev)
    cfgs = [None, B.make_cfg(8, 128, 2, unroll=2), B.make_cfg(8, 256, 2, unroll=1, flags=B.FLAG_XCD_CONTIG | B.FLAG_NONTEMPORAL),
            B.make_cfg(8, 256, 4, reduce=1, unroll=4, flags=7), B.make_cfg(4, 1024, 1, unroll=2, flags=2, max_waves_per_simd=4)]
    for c in cfgs:
        if c is not None:
            st, why, _ = B.addrms_cfg_feasible(c, M, N, dtype)
            assert st == 0, why
        x.view(tiles, rows, N).copy_(xb)         # broadcast the block over the tiles
        r.view(tiles, rows, N).copy_(rb)
        print(f"addrms {M}x{N} {dtype} ({M * row_bytes / 2**30:.2f} GiB per tensor) cfg={c}", flush=True)
        B.addrms_run(x, r, w, wl.eps, M, N, dtype, c)
        torch.cuda.synchronize()
        assert _tiles_equal(r, r_ref_d, tiles, rows) == 0, f"residual differs, cfg={c}"
        assert _tiles_equal(x, y_ref_d, tiles, rows) == 0, f"y differs, cfg={c}"


def test_silumul_rows_beyond_4gib(oracle):
    rows, tiles, d, dtype = 1021, 100, 11008, "bf16"
    M = rows * tiles
    in_row_bytes = 2 * d * 2
    assert M * in_row_bytes > 2 ** 32 and (2 ** 32) % in_row_bytes != 0
    wl = W.GatedWorkload("block_1021x11008_bf16", rows, d, dtype, 405)
    xb_host = W.generate_gated(wl)
    ref = oracle.silumul(W.to_bits(xb_host), B.DTYPE_IDS[dtype], nthreads=16)
    dev = torch.device("cuda:0")
    xb = xb_host.to(dev)
    ref_d = torch.from_numpy(ref.view(np.int16)).to(dev)
    x = torch.empty((M, 2 * d), dtype=xb.dtype, device=dev)
    x.view(tiles, rows, 2 * d).copy_(xb)
    out = torch.empty((M, d), dtype=xb.dtype, device=dev)
    cfgs = [None, B.make_cfg(8, 704, 1, unroll=1, flags=2), B.make_cfg(8, 512, 2, unroll=1, flags=7)]
    for c in cfgs:
        if c is not None:
            st, why, _ = B.silumul_cfg_feasible(c, M, d, dtype)
            assert st == 0, why
        out.fill_(float("nan"))
        print(f"silumul {M}x{d} {dtype} ({M * in_row_bytes / 2**30:.2f} GiB in) cfg={c}", flush=True)
        B.silumul_run(x, out, M, d, dtype, c)
        torch.cuda.synchronize()
        got = out.view(torch.int16).view(tiles, rows, d)
        worst = 0
        for t in range(tiles):
            diff = (got[t].to(torch.int32) - ref_d.to(torch.int32)).abs()     # same-sign neighbours differ by 1 in bits
            worst = max(worst, int(diff.max()))
        assert worst <= 1, f"silumul beyond 1 ulp (bit distance {worst}), cfg={c}"
