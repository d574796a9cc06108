"""Writes the instantiation list of the kernel template.

The templates in ``addrms_kernel.h`` and ``silumul_kernel.h`` have four
compile-time knobs (VEC, CPT, UNR, NT) per storage format; the register-cached
form of add+RMSNorm has a fifth, DF (residual store deferred to the write phase).  CPT = 0 names the
two-pass form of add+RMSNorm, which loops over the row instead of caching it
(rows beyond the register row cache), CPT = 200 + k the aligned-span form with
k chunks per thread, and CPT = 300 + k the form whose cache continues in LDS
after k register-held chunks (and re-reads what fits neither).  This script emits,
into a build directory:

  kern_<op>_d<DT>_v<VEC>.hip  one translation unit per (operator, format, vector width),
                          each kernel an ``extern "C"`` wrapper with a readable
                          name so the compiler's resource remarks can be
                          matched back to knob values;
  gen_dispatch_decl.inc   declarations of every kernel, and
  gen_dispatch_rows.inc   the rows of the table of their addresses, both
                          included by the runtime;
  gen_instances.inc       the list of instances (knob values, workgroup bound),
                          included by the host-only deriver.

The set must agree with the index arithmetic in ``addrms_internal.h``.
"""
from __future__ import annotations

import os
import sys

DTS = (0, 1, 2, 3)                      # bf16, fp16, fp16+fp32 residual, fp32
VECS = (1, 2, 4, 8)
CPTS = (1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16)
UNRS = (1, 2, 4, 8)
X_BYTES = {0: 2, 1: 2, 2: 2, 3: 4}      # bytes per x element of each format
MAX_ELEMS = 64                          # register row cache: VEC * CPT fp32 values per thread
BIG_ELEMS = 32                          # above this the instance is compiled for <= 256 threads
SPAN_BASE = 200                         # cpt code of the aligned-span form: 200 + chunks per thread
HYBRID_BASE = 300                       # cpt code of the hybrid long-row form: 300 + register-held chunks
HYBRID_BIG_BASE = 400                   # the same body for workgroups of at most 512 threads: 400 + register-held chunks
HYBRID_BIG_ELEMS = 144                  # ... which keeps this many values per thread in registers (vec 4 and 8 only)
SPAN_CPTS = (1, 2, 4)
R_BYTES = {0: 2, 1: 2, 2: 4, 3: 4}      # bytes per residual element of each format


OP_ADDRMS, OP_SILUMUL, OP_MERGE = 0, 1, 2
OP_PREFIX = {OP_ADDRMS: "addrms", OP_SILUMUL: "silumul", OP_MERGE: "mergestates"}
MERGE_DTS = (0, 1)                      # merge_attn_states: 16-bit partial outputs, fp32 scores
MERGE_CPTS = (1, 2, 3, 4)               # head sizes are small: a row is a few chunks at most
SILU_DTS = (0, 1, 3)                    # silu_and_mul has no mixed-precision residual stream
SILU_CPTS = (1, 2, 3, 4, 5, 6, 7, 8)


def instances():
    """(op, dt, vec, cpt, unr, nt, df, maxt) of every compiled kernel, in table order."""
    for op, dts, cpts in ((OP_ADDRMS, DTS, CPTS), (OP_SILUMUL, SILU_DTS, SILU_CPTS),
                          (OP_MERGE, MERGE_DTS, MERGE_CPTS)):
        for dt in dts:
            for vec in VECS:
                if vec * X_BYTES[dt] > 16:           # wider than one global access: never selectable
                    continue
                for cpt in cpts:
                    if vec * cpt > MAX_ELEMS:
                        continue
                    for unr in UNRS:
                        if unr > cpt:
                            continue
                        maxt = 1024 if vec * cpt <= BIG_ELEMS else 256
                        for nt in (0, 1):
                            for df in ((0, 1) if op == OP_ADDRMS else (0,)):
                                yield op, dt, vec, cpt, unr, nt, df, maxt
                if op == OP_ADDRMS:                  # two-pass form: no row cache, any row length
                    for unr in UNRS:
                        for nt in (0, 1):
                            yield op, dt, vec, 0, unr, nt, 0, 1024
                    if vec * X_BYTES[dt] <= 16 and vec * R_BYTES[dt] == 16:   # aligned-span form: 16-byte residual pieces
                        for cpt in SPAN_CPTS:
                            for unr in UNRS:
                                if unr > cpt:
                                    continue
                                for nt in (0, 1):
                                    for df in (0, 1):
                                        yield op, dt, vec, SPAN_BASE + cpt, unr, nt, df, 1024
                    hyb_cpt = 48 // vec              # row cache continued in LDS: 48 values in registers, then LDS; what fits
                                                     # neither (hybrid form) is read twice
                    for unr in UNRS:
                        if unr > hyb_cpt:
                            continue
                        for nt in (0, 1):
                            yield op, dt, vec, HYBRID_BASE + hyb_cpt, unr, nt, 0, 1024
                    if vec in (4, 8) and X_BYTES[dt] == 2:   # half the threads, twice the registers per lane: 144 values
                        for unr in (1, 2, 4):                # (with fp32 x, or eight chunks in flight, the body spills)
                            for nt in (0, 1):
                                yield op, dt, vec, HYBRID_BIG_BASE + HYBRID_BIG_ELEMS // vec, unr, nt, 0, 512


def name(op, dt, vec, cpt, unr, nt, df=0):
    return f"{OP_PREFIX[op]}_k_d{dt}_v{vec}_c{cpt}_u{unr}_n{nt}" + ("_s1" if df else "")


ARGS = {
    OP_ADDRMS: ("void* x, void* r, const void* w, float eps, double inv_n, "
                "long long M, int N, unsigned flags, int reduce, unsigned nblocks"),
    OP_SILUMUL: "const void* x, void* out, long long M, int d, unsigned flags, unsigned nblocks",
    OP_MERGE: ("const void* va, const float* sa, const void* vb, const float* sb, void* vo, float* so, "
               "long long rows, int d, unsigned flags, unsigned nblocks"),
}
CALL = {
    OP_ADDRMS: "addrms::addrms_body<{dt}, {vec}, {cpt}, {unr}, {nt}, {df}>(x, r, w, eps, inv_n, M, N, flags, reduce, nblocks);",
    OP_SILUMUL: "addrms::silumul_body<{dt}, {vec}, {cpt}, {unr}, {nt}>(x, out, M, d, flags, nblocks);",
    OP_MERGE: ("addrms::mergestates_body<{dt}, {vec}, {cpt}, {unr}, {nt}>"
               "(va, sa, vb, sb, vo, so, rows, d, flags, nblocks);"),
}
TWO_PASS_CALL = "addrms::addrms_twopass_body<{dt}, {vec}, {unr}, {nt}>(x, r, w, eps, inv_n, M, N, flags, reduce, nblocks);"
HYBRID_CALL = ("addrms::addrms_hybrid_body<{dt}, {vec}, {cpt}, {unr}, {nt}>"
               "(x, r, w, eps, inv_n, M, N, flags, reduce, nblocks);")
SPAN_CALL = ("addrms::addrms_span_body<{dt}, {vec}, {cpt}, {unr}, {nt}, {df}>"
             "(x, r, w, eps, inv_n, M, N, flags, reduce, nblocks);")
HEADER = {OP_ADDRMS: "addrms_kernel.h", OP_SILUMUL: "silumul_kernel.h", OP_MERGE: "mergestates_kernel.h"}


def main(outdir: str) -> None:
    os.makedirs(outdir, exist_ok=True)
    units = {}
    for op, dt, vec, cpt, unr, nt, df, maxt in instances():
        units.setdefault((op, dt, vec), []).append((cpt, unr, nt, df, maxt))
    for (op, dt, vec), lst in units.items():
        lines = [f'#include "{HEADER[op]}"', ""]
        for cpt, unr, nt, df, maxt in lst:
            fmt = CALL[op]
            if op == OP_ADDRMS and cpt == 0:
                fmt = TWO_PASS_CALL
            elif op == OP_ADDRMS and cpt >= HYBRID_BASE:
                fmt = HYBRID_CALL
            elif op == OP_ADDRMS and cpt >= SPAN_BASE:
                fmt = SPAN_CALL
            call = fmt.format(dt=dt, vec=vec, cpt=cpt % 100, unr=unr, nt="true" if nt else "false",
                              df="true" if df else "false")
            lines.append(f'extern "C" __global__ __launch_bounds__({maxt}) void {name(op, dt, vec, cpt, unr, nt, df)}'
                         f"({ARGS[op]})\n{{ {call} }}")
        _write(os.path.join(outdir, f"kern_{OP_PREFIX[op]}_d{dt}_v{vec}.hip"), "\n".join(lines) + "\n")
    decl, table, inst = [], [], []
    for op, dt, vec, cpt, unr, nt, df, maxt in instances():
        n = name(op, dt, vec, cpt, unr, nt, df)
        decl.append(f'extern "C" __global__ void {n}({ARGS[op]});')
        table.append(f"    {{{op}, {dt}, {vec}, {cpt}, {unr}, {nt}, {df}, reinterpret_cast<const void*>(&{n})}},")
        inst.append(f"    {{{op}, {dt}, {vec}, {cpt}, {unr}, {nt}, {df}, {maxt}}},")
    _write(os.path.join(outdir, "gen_dispatch_decl.inc"), "\n".join(decl) + "\n")
    _write(os.path.join(outdir, "gen_dispatch_rows.inc"), "\n".join(table) + "\n")
    _write(os.path.join(outdir, "gen_instances.inc"), "\n".join(inst) + "\n")


def _write(path: str, text: str) -> None:
    if os.path.exists(path) and open(path).read() == text:
        return
    with open(path, "w") as f:
        f.write(text)


if __name__ == "__main__":
    main(sys.argv[1])
