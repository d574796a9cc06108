"""ctypes front end of the plain C oracle in ``addrms_oracle.c``.

Test infrastructure only (see the header of the C file).  The wrapper does no
arithmetic of the method: it compiles the C file with gcc when the shared
object is missing or older than the source, marshals numpy arrays, and calls
it.  16-bit formats travel as raw ``uint16`` bit patterns, fp32 as ``float32``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

BF16, FP16, FP16_RES32, FP32 = 0, 1, 2, 3
VARIANTS = {"canonical": 0, "seq32": 1, "pair32": 2}

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "addrms_oracle.c")
_SRC2 = os.path.join(_HERE, "silumul_oracle.c")
_SRC3 = os.path.join(_HERE, "mergestates_oracle.c")
_LIB = os.path.join(_HERE, "libaddrms_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no contraction, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC2), os.path.getmtime(_SRC3))
    if force or stale:
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
             "-fPIC", "-shared", "-o", tmp, _SRC, _SRC2, _SRC3, "-lm"],
            check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
            lib.oracle_addrms.argtypes = [vp, vp, vp, ctypes.c_float, i64, i64, ci, ci, vp, vp, vp, ci]
            lib.oracle_addrms.restype = ci
            lib.oracle_addrms_y64.argtypes = [vp, vp, vp, ctypes.c_double, i64, i64, ci, vp]
            lib.oracle_addrms_y64.restype = ci
            lib.oracle_rstd_canonical.argtypes = [ctypes.c_double, i64, ctypes.c_float]
            lib.oracle_rstd_canonical.restype = ctypes.c_float
            lib.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
            lib.oracle_bf16_to_f32.restype = ctypes.c_float
            lib.oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
            lib.oracle_f16_to_f32.restype = ctypes.c_float
            lib.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
            lib.oracle_f32_to_bf16.restype = ctypes.c_uint16
            lib.oracle_f32_to_f16.argtypes = [ctypes.c_float]
            lib.oracle_f32_to_f16.restype = ctypes.c_uint16
            lib.oracle_mergestates.argtypes = [vp, vp, vp, vp, i64, i64, ci, vp, vp, vp]
            lib.oracle_mergestates.restype = ci
            lib.oracle_silumul.argtypes = [vp, i64, i64, ci, vp, ci]
            lib.oracle_silumul.restype = ci
            lib.oracle_silumul_f64.argtypes = [vp, i64, i64, ci, vp]
            lib.oracle_silumul_f64.restype = ci
            for name in ("oracle_f32_to_bf16_array", "oracle_f32_to_f16_array",
                         "oracle_bf16_to_f32_array", "oracle_f16_to_f32_array"):
                getattr(lib, name).argtypes = [vp, vp, i64]
                getattr(lib, name).restype = None
            _lib = lib
    return _lib


def _x_np(dtype: int):
    return np.float32 if dtype == FP32 else np.uint16


def _r_np(dtype: int):
    return np.float32 if dtype in (FP32, FP16_RES32) else np.uint16


def _check(a: np.ndarray, want, shape, name: str) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != want:
        raise TypeError(f"{name}: expected {np.dtype(want)}, got {a.dtype}")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {shape}, got {a.shape}")
    return a


def addrms(x, r, w, eps: float, dtype: int, variant: str = "canonical",
           nthreads: int = 1, return_rstd: bool = False):
    """Run the oracle.  Returns ``(y, residual_out)`` (and ``rstd`` if asked).

    x, r: [M, N]; w: [N].  uint16 bit patterns for bf16/fp16 tensors, float32
    for fp32 tensors (the residual of FP16_RES32, everything of FP32).
    """
    M, N = x.shape
    x = _check(x, _x_np(dtype), (M, N), "x")
    r = _check(r, _r_np(dtype), (M, N), "r")
    w = _check(w, _x_np(dtype), (N,), "w")
    y = np.empty((M, N), dtype=_x_np(dtype))
    res = np.empty((M, N), dtype=_r_np(dtype))
    rstd = np.empty((M,), dtype=np.float32)
    rc = _load().oracle_addrms(
        x.ctypes.data, r.ctypes.data, w.ctypes.data, float(eps), M, N, dtype,
        VARIANTS[variant], y.ctypes.data, res.ctypes.data, rstd.ctypes.data, int(nthreads))
    if rc != 0:
        raise RuntimeError(f"oracle_addrms failed with {rc}")
    return (y, res, rstd) if return_rstd else (y, res)


def addrms_y64(x, r, w, eps: float, dtype: int) -> np.ndarray:
    """Unrounded fp64 evaluation h*w/sqrt(mean(h^2)+eps) with h = x + r."""
    M, N = x.shape
    x = _check(x, _x_np(dtype), (M, N), "x")
    r = _check(r, _r_np(dtype), (M, N), "r")
    w = _check(w, _x_np(dtype), (N,), "w")
    y64 = np.empty((M, N), dtype=np.float64)
    rc = _load().oracle_addrms_y64(x.ctypes.data, r.ctypes.data, w.ctypes.data,
                                   float(eps), M, N, dtype, y64.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_addrms_y64 failed with {rc}")
    return y64


def silumul(x, dtype: int, nthreads: int = 1) -> np.ndarray:
    """silu_and_mul oracle: x [M, 2d] (uint16 bit patterns or float32) -> out [M, d], same storage."""
    M, two_d = x.shape
    if two_d % 2:
        raise ValueError("row length must be even")
    d = two_d // 2
    x = _check(x, _x_np(dtype), (M, two_d), "x")
    out = np.empty((M, d), dtype=_x_np(dtype))
    rc = _load().oracle_silumul(x.ctypes.data, M, d, dtype, out.ctypes.data, int(nthreads))
    if rc != 0:
        raise RuntimeError(f"oracle_silumul failed with {rc}")
    return out


def silumul_f64(x, dtype: int) -> np.ndarray:
    """The unrounded fp64 values silu(gate) * up."""
    M, two_d = x.shape
    d = two_d // 2
    x = _check(x, _x_np(dtype), (M, two_d), "x")
    out = np.empty((M, d), dtype=np.float64)
    rc = _load().oracle_silumul_f64(x.ctypes.data, M, d, dtype, out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_silumul_f64 failed with {rc}")
    return out


def mergestates(va, sa, vb, sb, dtype: int, want_f64: bool = False):
    """merge_attn_states oracle.  va, vb: [rows, d] uint16 bit patterns; sa, sb: [rows] float32.
    Returns (v_out bits, s_out fp32) and, if asked, the unrounded fp64 v_out as a third item."""
    rows, d = va.shape
    va = _check(va, np.uint16, (rows, d), "va")
    vb = _check(vb, np.uint16, (rows, d), "vb")
    sa = _check(sa, np.float32, (rows,), "sa")
    sb = _check(sb, np.float32, (rows,), "sb")
    vout = np.empty((rows, d), dtype=np.uint16)
    sout = np.empty((rows,), dtype=np.float32)
    v64 = np.empty((rows, d), dtype=np.float64) if want_f64 else None
    rc = _load().oracle_mergestates(va.ctypes.data, sa.ctypes.data, vb.ctypes.data, sb.ctypes.data, rows, d, dtype,
                                    vout.ctypes.data, sout.ctypes.data, v64.ctypes.data if want_f64 else None)
    if rc != 0:
        raise RuntimeError(f"oracle_mergestates failed with {rc}")
    return (vout, sout, v64) if want_f64 else (vout, sout)


def rstd_canonical(ss: float, N: int, eps: float) -> np.float32:
    return np.float32(_load().oracle_rstd_canonical(float(ss), int(N), float(eps)))


def _convert(name: str, a: np.ndarray, src, dst) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=src)
    out = np.empty(a.shape, dtype=dst)
    getattr(_load(), name)(a.ctypes.data, out.ctypes.data, a.size)
    return out


def f32_to_bf16_array(a):
    return _convert("oracle_f32_to_bf16_array", a, np.float32, np.uint16)


def f32_to_f16_array(a):
    return _convert("oracle_f32_to_f16_array", a, np.float32, np.uint16)


def bf16_to_f32_array(a):
    return _convert("oracle_bf16_to_f32_array", a, np.uint16, np.float32)


def f16_to_f32_array(a):
    return _convert("oracle_f16_to_f32_array", a, np.uint16, np.float32)


def bf16_to_f32(b: int) -> np.float32:
    return np.float32(_load().oracle_bf16_to_f32(int(b)))


def f16_to_f32(b: int) -> np.float32:
    return np.float32(_load().oracle_f16_to_f32(int(b)))


def f32_to_bf16(f) -> int:
    return int(_load().oracle_f32_to_bf16(float(np.float32(f))))


def f32_to_f16(f) -> int:
    return int(_load().oracle_f32_to_f16(float(np.float32(f))))
