"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI
and compare with the CPU oracle, element by element."""
from __future__ import annotations

import numpy as np
import torch

from paper_2601_12698_amd import binding as B
from paper_2601_12698_amd import workloads as W
from ulp import ulp_distance

MAX_ABS_CAP = 2e-2     # stated cap on the absolute error of the normalised output


def to_float64(bits: np.ndarray, dtype: str, which: str) -> np.ndarray:
    if bits.dtype == np.float32:
        return bits.astype(np.float64)
    t = torch.from_numpy(bits.view(np.int16).copy())
    return t.view(torch.bfloat16 if dtype == "bf16" else torch.float16).double().numpy()


def oracle_outputs(oracle, d, wl, nthreads=16):
    return oracle.addrms(W.to_bits(d["x"]), W.to_bits(d["r"]), W.to_bits(d["w"]), wl.eps,
                         B.DTYPE_IDS[wl.dtype], nthreads=nthreads)


def compare(y, res, y_ref, res_ref, dtype, what=""):
    """The parity bar: residual bit-exact; y within 1 unit in the last place of
    its storage format and within the absolute cap.  Returns the mismatch stats."""
    assert np.array_equal(res.view(np.uint8), res_ref.view(np.uint8)), f"{what}: residual not bit-exact"
    stats = {"n": int(y.size), "n_diff": 0, "max_ulp": 0, "max_abs": 0.0}
    if np.array_equal(y.view(np.uint8), y_ref.view(np.uint8)):
        return stats
    idx = np.nonzero(y != y_ref) if y.dtype == np.uint16 else np.nonzero(y.view(np.uint32) != y_ref.view(np.uint32))
    dist = ulp_distance(y[idx], y_ref[idx])
    nbad = int((dist > 0).sum())          # +0 and -0 are the same value
    stats["n_diff"] = nbad
    if nbad:
        stats["max_ulp"] = int(dist.max())
        a = to_float64(y[idx], dtype, "x")
        b = to_float64(y_ref[idx], dtype, "x")
        stats["max_abs"] = float(np.abs(a - b).max())
    assert stats["max_ulp"] <= 1, f"{what}: y off by {stats['max_ulp']} ulp ({nbad} elements differ)"
    assert stats["max_abs"] <= MAX_ABS_CAP, f"{what}: y abs error {stats['max_abs']} above cap"
    return stats


class DeviceCase:
    """Pristine device copies of one workload, re-used across configurations."""

    def __init__(self, d, wl):
        dev = torch.device("cuda:0")
        self.wl = wl
        self.x0 = d["x"].to(dev)
        self.r0 = d["r"].to(dev)
        self.w = d["w"].to(dev)
        self.x = torch.empty_like(self.x0)
        self.r = torch.empty_like(self.r0)

    def run(self, cfg=None):
        self.x.copy_(self.x0)
        self.r.copy_(self.r0)
        B.addrms_run(self.x, self.r, self.w, self.wl.eps, self.wl.M, self.wl.N, self.wl.dtype, cfg)
        torch.cuda.synchronize()
        return W.to_bits(self.x), W.to_bits(self.r)
