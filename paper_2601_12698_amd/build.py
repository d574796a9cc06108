"""Builds ``libaddrms.so`` for gfx950 with hipcc, in-tree.

Steps: generate the kernel instantiation units; compile them (in parallel)
while capturing the compiler's per-kernel resource report; turn that report
into the table the feasible-region deriver reads; compile the host units;
link.  Objects live under ``_build/`` next to this file; the shared library
is written into the package directory.

    python -m paper_2601_12698_amd.build [--force] [-j N]
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libaddrms.so")
ARCH = "gfx950"

# -packed-fp32-ops off: packed fp32 instruction selection stays disabled for all device code.
# -ffp-contract=off: the operator rounds every fp32 product before the next step (and before the
# conversion to storage); contraction would fuse multiply+convert into one mixed-precision
# instruction with a single rounding, which is a different result on exact ties.
DEVICE_FLAGS = [f"--offload-arch={ARCH}", "-O3", "-fPIC", "-std=c++17", "-ffp-contract=off",
                "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                "-Wno-unused-command-line-argument"]
HOST_FLAGS = ["-O2", "-fPIC", "-std=c++17", "-Wall", "-Wextra"]
INCLUDES = ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", BUILD]


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, **kw)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        raise RuntimeError(f"command failed: {cmd[0]} ... {cmd[-1]}")
    return r


def _newer(target: str, *deps: str) -> bool:
    if not os.path.exists(target):
        return False
    t = os.path.getmtime(target)
    return all(os.path.getmtime(d) <= t for d in deps)


_FIELD = re.compile(r"(Function Name|TotalSGPRs|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|"
                    r"LDS Size \[bytes/block\]|Occupancy \[waves/SIMD\]):\s+(\S+)")


def parse_remarks(text: str) -> dict:
    """kernel name -> {vgprs, agprs, sgprs, scratch, lds, occupancy} from
    ``-Rpass-analysis=kernel-resource-usage`` output."""
    out, cur = {}, None
    keys = {"VGPRs": "vgprs", "AGPRs": "agprs", "TotalSGPRs": "sgprs",
            "ScratchSize [bytes/lane]": "scratch", "LDS Size [bytes/block]": "lds",
            "Occupancy [waves/SIMD]": "occupancy"}
    for line in text.splitlines():
        m = _FIELD.search(line)
        if not m:
            continue
        k, v = m.group(1).strip(), m.group(2)
        if k == "Function Name":
            cur = out.setdefault(v, {})
        elif cur is not None and k in keys:
            cur[keys[k]] = int(v)
    return out


def _compile_kernel_unit(src: str, force: bool) -> str:
    obj = src[:-4] + ".o"
    rem = src[:-4] + ".remarks"
    if (not force and os.path.exists(rem) and
            _newer(obj, src, os.path.join(CSRC, "addrms_kernel.h"), os.path.join(CSRC, "silumul_kernel.h"),
                   os.path.join(CSRC, "mergestates_kernel.h"))):
        return open(rem).read()
    r = _run(["hipcc", *DEVICE_FLAGS, *INCLUDES, "-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", obj])
    with open(rem, "w") as f:
        f.write(r.stderr)
    return r.stderr


def build(force: bool = False, jobs: int = 8, verbose: bool = False) -> str:
    sys.path.insert(0, CSRC)
    try:
        import gen_kernels
    finally:
        sys.path.pop(0)
    os.makedirs(BUILD, exist_ok=True)
    gen_kernels.main(BUILD)
    wanted = {f"kern_{gen_kernels.OP_PREFIX[op]}_d{dt}_v{vec}.hip" for op, dt, vec, *_ in gen_kernels.instances()}
    for f in os.listdir(BUILD):          # units of an older instance list must not be linked in
        if f.startswith("kern_") and f.split(".")[0] + ".hip" not in wanted:
            os.remove(os.path.join(BUILD, f))
    units = sorted(os.path.join(BUILD, f) for f in wanted)
    with cf.ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
        remarks = list(ex.map(lambda s: _compile_kernel_unit(s, force), units))
    res = {}
    for text in remarks:
        res.update(parse_remarks(text))
    rows = []
    for op, dt, vec, cpt, unr, nt, df, _maxt in gen_kernels.instances():
        r = res.get(gen_kernels.name(op, dt, vec, cpt, unr, nt, df))
        if r is None or any(k not in r for k in ("vgprs", "agprs", "sgprs", "scratch", "lds", "occupancy")):
            raise RuntimeError(f"no resource report for {gen_kernels.name(op, dt, vec, cpt, unr, nt, df)}")
        rows.append(f"    {{{r['vgprs']}, {r['agprs']}, {r['sgprs']}, {r['scratch']}, {r['lds']}, {r['occupancy']}}},")
    gen_kernels._write(os.path.join(BUILD, "gen_resources.inc"), "\n".join(rows) + "\n")

    objs = [u[:-4] + ".o" for u in units]
    hdrs = [os.path.join(ROOT, "include", "addrms.h"), os.path.join(ROOT, "include", "silumul.h"), os.path.join(ROOT, "include", "mergestates.h"),
            os.path.join(CSRC, "addrms_internal.h")]
    gen = [os.path.join(BUILD, f) for f in ("gen_instances.inc", "gen_resources.inc",
                                             "gen_dispatch_decl.inc", "gen_dispatch_rows.inc")]
    for name in ("addrms_cfg.cpp", "addrms_table.cpp", "addrms_search.cpp", "addrms_general.cpp", "addrms_audit.cpp"):
        src = os.path.join(CSRC, name)
        obj = os.path.join(BUILD, name + ".o")
        if force or not _newer(obj, src, *hdrs, *gen):
            _run(["hipcc", "-x", "c++", *HOST_FLAGS, *INCLUDES, "-c", src, "-o", obj])
        objs.append(obj)
    src = os.path.join(CSRC, "addrms_runtime.hip")
    obj = os.path.join(BUILD, "addrms_runtime.o")
    if force or not _newer(obj, src, os.path.join(CSRC, "addrms_kernel.h"), os.path.join(CSRC, "silumul_kernel.h"),
                           os.path.join(CSRC, "mergestates_kernel.h"), *hdrs, *gen):
        _run(["hipcc", *DEVICE_FLAGS, *INCLUDES, "-c", src, "-o", obj])
    objs.append(obj)
    tmp = LIB + f".{os.getpid()}.tmp"
    _run(["hipcc", "-shared", "-fPIC", f"--offload-arch={ARCH}", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB}: {len(rows)} kernel instances")
    return LIB


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--force", action="store_true")
    ap.add_argument("-j", type=int, default=8)
    a = ap.parse_args()
    build(force=a.force, jobs=a.j, verbose=True)
