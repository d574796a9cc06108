"""ctypes binding of ``libaddrms.so`` -- argument marshalling only.

Every function here has the name of the C entry point it calls
(``include/addrms.h``); no step of the operator, the deriver or the search is
computed in Python.  Tensors are torch tensors used purely as device memory;
``stream`` defaults to torch's current stream on the tensor's device.

The library is loaded on first use.  If it has not been built the call raises
:class:`AddrmsLibraryMissing` -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (CFUNCTYPE, POINTER, Structure, byref, c_char_p, c_double, c_float, c_int, c_int32,
                    c_int64, c_size_t, c_void_p)
from typing import List, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaddrms.so")

BF16, FP16, FP16_RES32, FP32 = 0, 1, 2, 3
DTYPE_IDS = {"bf16": BF16, "fp16": FP16, "fp16_res32": FP16_RES32, "fp32": FP32}
REDUCE_WAVE, REDUCE_LDS = 0, 1
FLAG_XCD_CONTIG = 1
FLAG_NONTEMPORAL = 2
FLAG_PERSISTENT = 4
FLAG_TWO_PASS = 8
FLAG_LDS_CACHE = 16
FLAG_DEFER_STORE = 32
FLAG_ALIGNED_SPAN = 64
SEARCH_GUIDED, SEARCH_EXHAUSTIVE = 0, 1
FAMILY_STREAMING, FAMILY_OCCUPANCY_CAP, FAMILY_GRID_MAPPING, FAMILY_BASE_ONLY, FAMILY_STORE_PHASE = 1, 2, 4, 8, 16
MAX_ROUNDS = 5
HINT_LOWER_OCCUPANCY, HINT_HIGHER_OCCUPANCY, HINT_FEWER_LARGER_WORKGROUPS, HINT_WIDER_VECTORS = 1, 2, 4, 8
MAX_TOPK = 8

OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED_DTYPE, ERR_INFEASIBLE_CFG, ERR_MISALIGNED = -1, -2, -3, -4
ERR_HIP, ERR_IO, ERR_NO_RESULT, ERR_UNSUPPORTED_SHAPE = -5, -6, -7, -8


class AddrmsLibraryMissing(RuntimeError):
    pass


class AddrmsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"addrms status {status}: {message}")
        self.status = status
        self.message = message


class Cfg(Structure):
    _fields_ = [("vec", c_int32), ("threads_per_row", c_int32), ("rows_per_wg", c_int32),
                ("reduce", c_int32), ("unroll", c_int32), ("flags", c_int32),
                ("max_waves_per_simd", c_int32), ("walk", c_int32)]

    def as_tuple(self) -> Tuple[int, int, int, int, int, int, int, int]:
        return (self.vec, self.threads_per_row, self.rows_per_wg, self.reduce, self.unroll, self.flags,
                self.max_waves_per_simd, self.walk)

    def as_dict(self) -> dict:
        return dict(vec=self.vec, threads_per_row=self.threads_per_row, rows_per_wg=self.rows_per_wg,
                    reduce=self.reduce, unroll=self.unroll, flags=self.flags,
                    max_waves_per_simd=self.max_waves_per_simd, walk=self.walk)

    def __repr__(self) -> str:
        return ("Cfg(vec=%d, threads_per_row=%d, rows_per_wg=%d, reduce=%d, unroll=%d, flags=%d, "
                "max_waves_per_simd=%d, walk=%d)" % self.as_tuple())


def make_cfg(vec: int, threads_per_row: int, rows_per_wg: int = 1, reduce: int = REDUCE_WAVE,
             unroll: int = 1, flags: int = 0, max_waves_per_simd: int = 0, walk: int = 0) -> Cfg:
    c = Cfg()
    c.vec, c.threads_per_row, c.rows_per_wg, c.reduce, c.unroll, c.flags, c.max_waves_per_simd, c.walk = (
        vec, threads_per_row, rows_per_wg, reduce, unroll, flags, max_waves_per_simd, walk)
    return c


class Resources(Structure):
    _fields_ = [("chunks_per_thread", c_int32), ("vgprs", c_int32), ("agprs", c_int32), ("sgprs", c_int32),
                ("scratch_bytes", c_int32), ("lds_bytes", c_int32), ("max_threads", c_int32),
                ("waves_per_wg", c_int32), ("waves_per_simd_regs", c_int32), ("wgs_per_cu", c_int32),
                ("waves_per_simd", c_int32), ("reserved", c_int32 * 5)]

    def as_dict(self) -> dict:
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved"}


class Budget(Structure):
    _fields_ = [("max_wall_ms", c_double), ("max_candidates", c_int32), ("strategy", c_int32),
                ("top_k", c_int32), ("warmup", c_int32), ("reps", c_int32), ("coarse_warmup", c_int32),
                ("coarse_reps", c_int32), ("skip_validation", c_int32), ("eps", c_float),
                ("hints", c_int32), ("log_path", c_char_p),
                ("family_mask", c_int32), ("no_resume", c_int32)]


class TuneReport(Structure):
    _fields_ = [("n_grid", c_int64), ("n_feasible", c_int64), ("n_measured", c_int64), ("n_failed", c_int64),
                ("best_found_at", c_int64), ("best_us", c_double), ("default_us", c_double),
                ("wall_ms", c_double), ("time_to_best_ms", c_double), ("best", Cfg), ("default_cfg", Cfg),
                ("n_topk", c_int32), ("n_resumed", c_int32), ("topk", Cfg * MAX_TOPK),
                ("topk_us", c_double * MAX_TOPK)]

    def as_dict(self) -> dict:
        return dict(n_grid=self.n_grid, n_feasible=self.n_feasible, n_measured=self.n_measured,
                    n_failed=self.n_failed, n_resumed=self.n_resumed, best_found_at=self.best_found_at, best_us=self.best_us,
                    default_us=self.default_us, wall_ms=self.wall_ms, time_to_best_ms=self.time_to_best_ms,
                    best=self.best.as_dict(), default_cfg=self.default_cfg.as_dict(),
                    topk=[(self.topk[i].as_dict(), self.topk_us[i]) for i in range(self.n_topk)])


VALIDATE_FN = CFUNCTYPE(c_int, c_void_p, POINTER(Cfg))
MEASURE_FN = CFUNCTYPE(c_int, c_void_p, POINTER(Cfg), c_int, c_int, POINTER(c_double))


class Backend(Structure):
    _fields_ = [("user", c_void_p), ("validate", VALIDATE_FN), ("measure", MEASURE_FN)]


MAX_SHAPES = 16


class Shape(Structure):
    _fields_ = [("M", c_int64), ("N", c_int64)]


class GeneralReport(Structure):
    _fields_ = [("n_shapes", c_int32), ("n_pool", c_int32), ("geomean_speedup_general", c_double),
                ("geomean_speedup_specialized", c_double), ("mean_speedup_general", c_double),
                ("wall_ms", c_double), ("default_us", c_double * MAX_SHAPES), ("general_us", c_double * MAX_SHAPES),
                ("specialized_us", c_double * MAX_SHAPES), ("specialized", Cfg * MAX_SHAPES)]

    def as_dict(self) -> dict:
        n = self.n_shapes
        return dict(n_shapes=n, n_pool=self.n_pool, geomean_speedup_general=self.geomean_speedup_general,
                    geomean_speedup_specialized=self.geomean_speedup_specialized,
                    mean_speedup_general=self.mean_speedup_general, wall_ms=self.wall_ms,
                    default_us=list(self.default_us[:n]), general_us=list(self.general_us[:n]),
                    specialized_us=list(self.specialized_us[:n]),
                    specialized=[self.specialized[i].as_dict() for i in range(n)])


class TimeStats(Structure):
    _fields_ = [("mean_us", c_double), ("per_launch_mean_us", c_double), ("median_us", c_double),
                ("min_us", c_double), ("max_us", c_double), ("reps", c_int32), ("buffer_sets", c_int32)]

    def as_dict(self) -> dict:
        return {k: getattr(self, k) for k, _ in self._fields_}


class HwLimits(Structure):
    _fields_ = [("compute_units", c_int32), ("xcds", c_int32), ("simds_per_cu", c_int32), ("wave_size", c_int32),
                ("max_waves_per_simd", c_int32), ("regs_per_lane", c_int32), ("reg_granule", c_int32),
                ("lds_bytes_per_cu", c_int32), ("lds_granule", c_int32), ("max_threads_per_wg", c_int32),
                ("max_access_bytes", c_int32), ("reserved", c_int32), ("hbm_bytes_per_s", c_double),
                ("last_level_cache_bytes", c_int64), ("l2_bytes_per_xcd", c_int64)]

    def as_dict(self) -> dict:
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved"}


class RoundInfo(Structure):
    _fields_ = [("families", c_int32), ("passed", c_int32), ("score", c_double),
                ("geomean_speedup_general", c_double), ("general", Cfg)]


class RoundsReport(Structure):
    _fields_ = [("n_rounds", c_int32), ("best_round", c_int32), ("wall_ms", c_double),
                ("rounds", RoundInfo * MAX_ROUNDS), ("best", GeneralReport)]

    def as_dict(self) -> dict:
        return dict(n_rounds=self.n_rounds, best_round=self.best_round, wall_ms=self.wall_ms,
                    rounds=[dict(families=r.families, passed=bool(r.passed), score=r.score,
                                 geomean_speedup_general=r.geomean_speedup_general, general=r.general.as_dict())
                            for r in self.rounds[:self.n_rounds]],
                    best=self.best.as_dict())


AUDIT_RULES = 6


class AuditRule(Structure):
    _fields_ = [("rule", ctypes.c_char * 24), ("n_pruned", c_int64), ("n_measured", c_int32), ("n_failed", c_int32),
                ("n_in_top_decile", c_int32), ("n_beating_best", c_int32), ("best_us", c_double),
                ("median_us", c_double), ("best", Cfg)]

    def as_dict(self) -> dict:
        return dict(rule=self.rule.decode(), n_pruned=self.n_pruned, n_measured=self.n_measured, n_failed=self.n_failed,
                    n_in_top_decile=self.n_in_top_decile, n_beating_best=self.n_beating_best, best_us=self.best_us,
                    median_us=self.median_us, best=self.best.as_dict())


class AuditReport(Structure):
    _fields_ = [("n_retained", c_int64), ("n_retained_measured", c_int32), ("n_retained_failed", c_int32),
                ("retained_best_us", c_double), ("retained_decile_us", c_double), ("retained_median_us", c_double),
                ("wall_ms", c_double), ("truncated", c_int32), ("reserved", c_int32), ("retained_best", Cfg),
                ("rules", AuditRule * AUDIT_RULES)]

    def as_dict(self) -> dict:
        return dict(n_retained=self.n_retained, n_retained_measured=self.n_retained_measured,
                    n_retained_failed=self.n_retained_failed, retained_best_us=self.retained_best_us,
                    retained_decile_us=self.retained_decile_us, retained_median_us=self.retained_median_us,
                    wall_ms=self.wall_ms, truncated=bool(self.truncated), retained_best=self.retained_best.as_dict(),
                    rules=[r.as_dict() for r in self.rules])


OPEN_FN = CFUNCTYPE(c_int, c_void_p, c_int64, c_int64, c_int, POINTER(Backend))
CLOSE_FN = CFUNCTYPE(None, c_void_p, POINTER(Backend))


class BackendFactory(Structure):
    _fields_ = [("user", c_void_p), ("open", OPEN_FN), ("close", CLOSE_FN)]


# name -> (restype, argtypes); mirrors include/addrms.h one to one
SIGNATURES = {
    "addrms_run": (c_int, [c_void_p, c_void_p, c_void_p, c_float, c_int64, c_int64, c_int, POINTER(Cfg), c_void_p]),
    "addrms_default_cfg": (c_int, [c_int64, c_int, POINTER(Cfg)]),
    "addrms_cfg_feasible": (c_int, [POINTER(Cfg), c_int64, c_int64, c_int, c_char_p, c_size_t, POINTER(Resources)]),
    "addrms_enumerate_feasible": (c_int64, [c_int64, c_int64, c_int, POINTER(Cfg), c_int64, POINTER(c_int64)]),
    "addrms_tune": (c_int, [c_int64, c_int64, c_int, POINTER(Budget), POINTER(Cfg), POINTER(TuneReport)]),
    "addrms_tune_with_backend": (c_int, [c_int64, c_int64, c_int, POINTER(Budget), POINTER(Backend),
                                         POINTER(Cfg), POINTER(TuneReport)]),
    "addrms_select_general": (c_int, [POINTER(Shape), c_int32, c_int, POINTER(Budget), POINTER(Cfg),
                                      POINTER(GeneralReport)]),
    "addrms_select_general_with_backend": (c_int, [POINTER(Shape), c_int32, c_int, POINTER(Budget),
                                                   POINTER(BackendFactory), POINTER(Cfg), POINTER(GeneralReport)]),
    "addrms_tune_rounds": (c_int, [POINTER(Shape), c_int32, c_int, POINTER(Budget), POINTER(Cfg),
                                   POINTER(RoundsReport)]),
    "addrms_tune_rounds_with_backend": (c_int, [POINTER(Shape), c_int32, c_int, POINTER(Budget),
                                                POINTER(BackendFactory), POINTER(Cfg), POINTER(RoundsReport)]),
    "addrms_audit_rules": (c_int, [c_int64, c_int64, c_int, POINTER(Budget), POINTER(AuditReport)]),
    "addrms_audit_rules_with_backend": (c_int, [c_int64, c_int64, c_int, POINTER(Budget), POINTER(Backend),
                                                POINTER(AuditReport)]),
    "addrms_measure": (c_int, [POINTER(Cfg), c_int64, c_int64, c_int, c_float, c_int, c_int, c_int, POINTER(c_double)]),
    "addrms_measure_stats": (c_int, [POINTER(Cfg), c_int64, c_int64, c_int, c_float, c_int, c_int, c_int,
                                     POINTER(TimeStats)]),
    "addrms_get_hw_limits": (c_int, [POINTER(HwLimits)]),
    "addrms_table_insert": (c_int, [c_int64, c_int64, c_int, POINTER(Cfg), c_double]),
    "addrms_table_lookup": (c_int, [c_int64, c_int64, c_int, POINTER(Cfg)]),
    "addrms_table_size": (c_int64, []),
    "addrms_table_clear": (None, []),
    "addrms_table_save": (c_int, [c_char_p]),
    "addrms_table_load": (c_int, [c_char_p]),
    "addrms_device_resources": (c_int, [POINTER(Cfg), c_int64, c_int64, c_int, POINTER(Resources)]),
    "addrms_rstd_probe": (c_int, [c_void_p, c_int64, c_int64, c_float, c_void_p, c_void_p]),
    "addrms_stream_probe": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_int, c_void_p]),
    "addrms_row_probe": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_int, c_int, c_int, c_void_p]),
    "addrms_gate_probe": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int, ctypes.c_uint32, c_void_p,
                                  c_void_p]),
    "addrms_gate_probe_noalloc": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int, ctypes.c_uint32,
                                          c_void_p, c_void_p]),
    "addrms_algorithmic_bytes": (c_int64, [c_int64, c_int64, c_int]),
    "silumul_run": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_int, POINTER(Cfg), c_void_p]),
    "silumul_default_cfg": (c_int, [c_int64, c_int, POINTER(Cfg)]),
    "silumul_cfg_feasible": (c_int, [POINTER(Cfg), c_int64, c_int64, c_int, c_char_p, c_size_t, POINTER(Resources)]),
    "silumul_enumerate_feasible": (c_int64, [c_int64, c_int64, c_int, POINTER(Cfg), c_int64, POINTER(c_int64)]),
    "silumul_tune": (c_int, [c_int64, c_int64, c_int, POINTER(Budget), POINTER(Cfg), POINTER(TuneReport)]),
    "silumul_tune_with_backend": (c_int, [c_int64, c_int64, c_int, POINTER(Budget), POINTER(Backend),
                                          POINTER(Cfg), POINTER(TuneReport)]),
    "silumul_select_general": (c_int, [POINTER(Shape), c_int32, c_int, POINTER(Budget), POINTER(Cfg), POINTER(GeneralReport)]),
    "silumul_tune_rounds": (c_int, [POINTER(Shape), c_int32, c_int, POINTER(Budget), POINTER(Cfg), POINTER(RoundsReport)]),
    "silumul_measure": (c_int, [POINTER(Cfg), c_int64, c_int64, c_int, c_int, c_int, c_int, POINTER(c_double)]),
    "silumul_table_lookup": (c_int, [c_int64, c_int64, c_int, POINTER(Cfg)]),
    "silumul_algorithmic_bytes": (c_int64, [c_int64, c_int64, c_int]),
    "mergestates_run": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int,
                                POINTER(Cfg), c_void_p]),
    "mergestates_default_cfg": (c_int, [c_int64, c_int, POINTER(Cfg)]),
    "mergestates_cfg_feasible": (c_int, [POINTER(Cfg), c_int64, c_int64, c_int, c_char_p, c_size_t, POINTER(Resources)]),
    "mergestates_enumerate_feasible": (c_int64, [c_int64, c_int64, c_int, POINTER(Cfg), c_int64, POINTER(c_int64)]),
    "mergestates_tune": (c_int, [c_int64, c_int64, c_int, POINTER(Budget), POINTER(Cfg), POINTER(TuneReport)]),
    "mergestates_tune_with_backend": (c_int, [c_int64, c_int64, c_int, POINTER(Budget), POINTER(Backend),
                                              POINTER(Cfg), POINTER(TuneReport)]),
    "mergestates_select_general": (c_int, [POINTER(Shape), c_int32, c_int, POINTER(Budget), POINTER(Cfg),
                                           POINTER(GeneralReport)]),
    "mergestates_tune_rounds": (c_int, [POINTER(Shape), c_int32, c_int, POINTER(Budget), POINTER(Cfg),
                                        POINTER(RoundsReport)]),
    "mergestates_measure": (c_int, [POINTER(Cfg), c_int64, c_int64, c_int, c_int, c_int, c_int, POINTER(c_double)]),
    "mergestates_table_lookup": (c_int, [c_int64, c_int64, c_int, POINTER(Cfg)]),
    "mergestates_algorithmic_bytes": (c_int64, [c_int64, c_int64, c_int]),
    "addrms_last_error": (c_char_p, []),
    "addrms_version": (c_char_p, []),
}

_lib = None


def load() -> ctypes.CDLL:
    """Load libaddrms.so (once) and declare every entry point."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise AddrmsLibraryMissing(
                f"{LIB_PATH} not found: build it with `python -m paper_2601_12698_amd.build` "
                "(there is no fallback implementation)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(status: int) -> int:
    if status < 0:
        raise AddrmsError(int(status), load().addrms_last_error().decode("utf-8", "replace"))
    return status


def _dtype_id(dtype) -> int:
    return DTYPE_IDS[dtype] if isinstance(dtype, str) else int(dtype)


def _stream_ptr(stream, tensor=None) -> Optional[int]:
    if stream is not None:
        return int(getattr(stream, "cuda_stream", stream))
    import torch
    return int(torch.cuda.current_stream(tensor.device if tensor is not None else None).cuda_stream)


def _ptr(t) -> int:
    return int(t.data_ptr())


_X_ELEM = {BF16: "bfloat16", FP16: "float16", FP16_RES32: "float16", FP32: "float32"}
_R_ELEM = {BF16: "bfloat16", FP16: "float16", FP16_RES32: "float32", FP32: "float32"}


def _expect_elem(name: str, t, want: str) -> None:
    """The C ABI sees only pointers, so a tensor whose element type is narrower than the
    storage format named by ``dtype`` would be read and written past its end: refuse it here."""
    got = str(t.dtype).replace("torch.", "")
    if got != want:
        raise ValueError(f"{name} is {got} but dtype asks for {want}")


def _expect_device_tensor(name: str, t, numel: int, elem: str) -> None:
    _expect_elem(name, t, elem)
    if t.numel() != numel:
        raise ValueError(f"{name} has {t.numel()} elements, expected {numel}")
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


# ---- entry points --------------------------------------------------------------

def addrms_version() -> str:
    return load().addrms_version().decode()


def addrms_last_error() -> str:
    return load().addrms_last_error().decode("utf-8", "replace")


def addrms_algorithmic_bytes(M: int, N: int, dtype) -> int:
    return _check(load().addrms_algorithmic_bytes(M, N, _dtype_id(dtype)))


def addrms_run(x, residual, weight, eps: float, M: int, N: int, dtype, cfg: Optional[Cfg] = None,
               stream=None) -> None:
    """In place: residual <- round(x + residual), x <- rmsnorm(x + residual) * weight."""
    dt = _dtype_id(dtype)
    if dt not in _X_ELEM:
        raise ValueError(f"unknown dtype {dtype!r}")
    _expect_device_tensor("x", x, M * N, _X_ELEM[dt])
    _expect_device_tensor("residual", residual, M * N, _R_ELEM[dt])
    _expect_device_tensor("weight", weight, N, _X_ELEM[dt])
    _check(load().addrms_run(_ptr(x), _ptr(residual), _ptr(weight), float(eps), M, N, _dtype_id(dtype),
                             byref(cfg) if cfg is not None else None, _stream_ptr(stream, x)))


def addrms_default_cfg(N: int, dtype) -> Cfg:
    c = Cfg()
    _check(load().addrms_default_cfg(N, _dtype_id(dtype), byref(c)))
    return c


def addrms_cfg_feasible(cfg: Cfg, M: int, N: int, dtype) -> Tuple[int, str, Resources]:
    """Returns (status, reason, resources); status 0 means feasible."""
    buf = ctypes.create_string_buffer(512)
    res = Resources()
    st = load().addrms_cfg_feasible(byref(cfg), M, N, _dtype_id(dtype), buf, len(buf), byref(res))
    return int(st), buf.value.decode("utf-8", "replace"), res


def addrms_enumerate_feasible(M: int, N: int, dtype) -> Tuple[List[Cfg], int]:
    """Returns (feasible cfgs, knob-grid size)."""
    lib = load()
    grid = c_int64(0)
    n = _check(lib.addrms_enumerate_feasible(M, N, _dtype_id(dtype), None, 0, byref(grid)))
    arr = (Cfg * max(n, 1))()
    _check(lib.addrms_enumerate_feasible(M, N, _dtype_id(dtype), arr, n, byref(grid)))
    out = []
    for i in range(n):
        c = Cfg()
        ctypes.memmove(byref(c), byref(arr[i]), ctypes.sizeof(Cfg))
        out.append(c)
    return out, int(grid.value)


def make_budget(max_wall_ms: float = 0.0, max_candidates: int = 0, strategy: int = SEARCH_GUIDED, top_k: int = 0,
                warmup: int = 0, reps: int = 0, coarse_warmup: int = 0, coarse_reps: int = 0,
                skip_validation: bool = False, eps: float = 0.0, log_path: Optional[str] = None,
                hints: int = 0, family_mask: int = 0, no_resume: bool = False) -> Budget:
    b = Budget()
    b.max_wall_ms, b.max_candidates, b.strategy, b.top_k = max_wall_ms, max_candidates, strategy, top_k
    b.warmup, b.reps, b.coarse_warmup, b.coarse_reps = warmup, reps, coarse_warmup, coarse_reps
    b.skip_validation, b.eps, b.hints, b.family_mask = int(skip_validation), eps, hints, family_mask
    b.no_resume = int(no_resume)
    b.log_path = log_path.encode() if log_path else None
    return b


def addrms_tune(M: int, N: int, dtype, budget: Optional[Budget] = None) -> Tuple[Cfg, TuneReport]:
    c, rep = Cfg(), TuneReport()
    _check(load().addrms_tune(M, N, _dtype_id(dtype), byref(budget) if budget is not None else None,
                              byref(c), byref(rep)))
    return c, rep


def addrms_tune_with_backend(M: int, N: int, dtype, budget: Optional[Budget], measure, validate=None
                             ) -> Tuple[Cfg, TuneReport]:
    """``measure(cfg, warmup, reps) -> microseconds`` (raise or return None to
    signal a failed candidate); ``validate(cfg) -> bool``."""
    def _m(_user, cfg_p, warmup, reps, out):
        try:
            us = measure(cfg_p.contents, warmup, reps)
        except Exception:
            return 1
        if us is None:
            return 1
        out[0] = float(us)
        return 0

    def _v(_user, cfg_p):
        try:
            return 0 if validate(cfg_p.contents) else 1
        except Exception:
            return 1

    be = Backend()
    be.user = None
    be.measure = MEASURE_FN(_m)
    be.validate = VALIDATE_FN(_v) if validate is not None else VALIDATE_FN()
    c, rep = Cfg(), TuneReport()
    _check(load().addrms_tune_with_backend(M, N, _dtype_id(dtype), byref(budget) if budget is not None else None,
                                           byref(be), byref(c), byref(rep)))
    return c, rep


def _wrap_measure(measure):
    def _m(_user, cfg_p, warmup, reps, out):
        try:
            us = measure(cfg_p.contents, warmup, reps)
        except Exception:
            return 1
        if us is None:
            return 1
        out[0] = float(us)
        return 0
    return MEASURE_FN(_m)


def _wrap_validate(validate):
    if validate is None:
        return VALIDATE_FN()

    def _v(_user, cfg_p):
        try:
            return 0 if validate(cfg_p.contents) else 1
        except Exception:
            return 1
    return VALIDATE_FN(_v)


def _shape_array(shapes):
    arr = (Shape * len(shapes))()
    for i, (m, n) in enumerate(shapes):
        arr[i].M, arr[i].N = m, n
    return arr


def addrms_select_general(shapes, dtype, budget: Optional[Budget] = None) -> Tuple[Cfg, GeneralReport]:
    """shapes: list of (M, N).  Returns (theta_gen, report)."""
    c, rep = Cfg(), GeneralReport()
    _check(load().addrms_select_general(_shape_array(shapes), len(shapes), _dtype_id(dtype),
                                        byref(budget) if budget is not None else None, byref(c), byref(rep)))
    return c, rep


def _python_factory(make_backend, keep):
    def _open(_user, M, N, _dt, out):
        try:
            measure, validate = make_backend(M, N)
        except Exception:
            return 1
        m, v = _wrap_measure(measure), _wrap_validate(validate)
        keep.append((m, v))
        out.contents.user = None
        out.contents.measure = m
        out.contents.validate = v
        return 0

    def _close(_user, _be):
        return None

    fac = BackendFactory()
    fac.user = None
    fac.open = OPEN_FN(_open)
    fac.close = CLOSE_FN(_close)
    keep.append((fac.open, fac.close))
    return fac


def addrms_audit_rules(M: int, N: int, dtype, budget: Optional[Budget] = None) -> AuditReport:
    """Times what the deriver's efficiency rules prune beside what they retain."""
    rep = AuditReport()
    _check(load().addrms_audit_rules(M, N, _dtype_id(dtype), byref(budget) if budget is not None else None, byref(rep)))
    return rep


def addrms_audit_rules_with_backend(M: int, N: int, dtype, budget: Optional[Budget], measure, validate=None
                                    ) -> AuditReport:
    be = Backend()
    be.user = None
    be.measure = _wrap_measure(measure)
    be.validate = _wrap_validate(validate)
    rep = AuditReport()
    _check(load().addrms_audit_rules_with_backend(M, N, _dtype_id(dtype), byref(budget) if budget is not None else None,
                                                  byref(be), byref(rep)))
    return rep


def addrms_tune_rounds(shapes, dtype, budget: Optional[Budget] = None) -> Tuple[Cfg, RoundsReport]:
    c, rep = Cfg(), RoundsReport()
    _check(load().addrms_tune_rounds(_shape_array(shapes), len(shapes), _dtype_id(dtype),
                                     byref(budget) if budget is not None else None, byref(c), byref(rep)))
    return c, rep


def addrms_tune_rounds_with_backend(shapes, dtype, budget: Optional[Budget], make_backend
                                    ) -> Tuple[Cfg, RoundsReport]:
    keep = []
    fac = _python_factory(make_backend, keep)
    c, rep = Cfg(), RoundsReport()
    _check(load().addrms_tune_rounds_with_backend(_shape_array(shapes), len(shapes), _dtype_id(dtype),
                                                  byref(budget) if budget is not None else None, byref(fac),
                                                  byref(c), byref(rep)))
    return c, rep


def addrms_select_general_with_backend(shapes, dtype, budget: Optional[Budget], make_backend
                                       ) -> Tuple[Cfg, GeneralReport]:
    """``make_backend(M, N) -> (measure, validate_or_None)`` with the callables of
    :func:`addrms_tune_with_backend`."""
    keep = []

    def _open(_user, M, N, _dt, out):
        try:
            measure, validate = make_backend(M, N)
        except Exception:
            return 1
        m, v = _wrap_measure(measure), _wrap_validate(validate)
        keep.append((m, v))
        out.contents.user = None
        out.contents.measure = m
        out.contents.validate = v
        return 0

    def _close(_user, _be):
        return None

    fac = BackendFactory()
    fac.user = None
    fac.open = OPEN_FN(_open)
    fac.close = CLOSE_FN(_close)
    c, rep = Cfg(), GeneralReport()
    _check(load().addrms_select_general_with_backend(_shape_array(shapes), len(shapes), _dtype_id(dtype),
                                                     byref(budget) if budget is not None else None, byref(fac),
                                                     byref(c), byref(rep)))
    return c, rep


def addrms_measure(cfg: Optional[Cfg], M: int, N: int, dtype, eps: float = 1e-6, warmup: int = 20,
                   reps: int = 100, rotate: bool = True) -> float:
    us = c_double(0.0)
    _check(load().addrms_measure(byref(cfg) if cfg is not None else None, M, N, _dtype_id(dtype), float(eps),
                                 warmup, reps, int(rotate), byref(us)))
    return float(us.value)


def addrms_measure_stats(cfg: Optional[Cfg], M: int, N: int, dtype, eps: float = 1e-6, warmup: int = 20,
                         reps: int = 100, rotate: bool = True) -> TimeStats:
    out = TimeStats()
    _check(load().addrms_measure_stats(byref(cfg) if cfg is not None else None, M, N, _dtype_id(dtype), float(eps),
                                       warmup, reps, int(rotate), byref(out)))
    return out


def addrms_get_hw_limits() -> HwLimits:
    out = HwLimits()
    _check(load().addrms_get_hw_limits(byref(out)))
    return out


def addrms_table_insert(M: int, N: int, dtype, cfg: Cfg, mean_us: float = 0.0) -> None:
    _check(load().addrms_table_insert(M, N, _dtype_id(dtype), byref(cfg), float(mean_us)))


def addrms_table_lookup(M: int, N: int, dtype) -> Optional[Cfg]:
    c = Cfg()
    st = load().addrms_table_lookup(M, N, _dtype_id(dtype), byref(c))
    if st == ERR_NO_RESULT:
        return None
    _check(st)
    return c


def addrms_table_size() -> int:
    return int(load().addrms_table_size())


def addrms_table_clear() -> None:
    load().addrms_table_clear()


def addrms_table_save(path: str) -> None:
    _check(load().addrms_table_save(path.encode()))


def addrms_table_load(path: str) -> None:
    _check(load().addrms_table_load(path.encode()))


def addrms_device_resources(cfg: Cfg, M: int, N: int, dtype) -> Resources:
    res = Resources()
    _check(load().addrms_device_resources(byref(cfg), M, N, _dtype_id(dtype), byref(res)))
    return res


def addrms_rstd_probe(ss, N: int, eps: float, out, stream=None) -> None:
    """ss: device fp64 [n]; out: device fp32 [n]."""
    _expect_device_tensor("ss", ss, ss.numel(), "float64")
    _expect_device_tensor("out", out, ss.numel(), "float32")
    _check(load().addrms_rstd_probe(_ptr(ss), ss.numel(), N, float(eps), _ptr(out), _stream_ptr(stream, ss)))


def addrms_stream_probe(x, residual, M: int, N: int, dtype, stream=None) -> None:
    dt = _dtype_id(dtype)
    if dt not in _X_ELEM:
        raise ValueError(f"unknown dtype {dtype!r}")
    _expect_device_tensor("x", x, M * N, _X_ELEM[dt])
    _expect_device_tensor("residual", residual, M * N, _R_ELEM[dt])
    _check(load().addrms_stream_probe(_ptr(x), _ptr(residual), M, N, _dtype_id(dtype), _stream_ptr(stream, x)))


def addrms_row_probe(x, residual, M: int, N: int, dtype, threads_per_row: int, wgs_per_cu: int = 0, stream=None) -> None:
    dt = _dtype_id(dtype)
    if dt not in _X_ELEM:
        raise ValueError(f"unknown dtype {dtype!r}")
    _expect_device_tensor("x", x, M * N, _X_ELEM[dt])
    _expect_device_tensor("residual", residual, M * N, _R_ELEM[dt])
    _check(load().addrms_row_probe(_ptr(x), _ptr(residual), M, N, dt, int(threads_per_row), int(wgs_per_cu),
                                   _stream_ptr(stream, x)))


class GateCounts(Structure):
    _fields_ = [("residual_mismatches", ctypes.c_uint32), ("y_beyond_tol", ctypes.c_uint32),
                ("y_max_distance", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


def _gate_args(y, y_ref, residual, residual_ref, dtype, counts_out):
    dt = _dtype_id(dtype)
    if dt not in _X_ELEM:
        raise ValueError(f"unknown dtype {dtype!r}")
    n = y.numel()
    _expect_device_tensor("y", y, n, _X_ELEM[dt])
    _expect_device_tensor("y_ref", y_ref, n, _X_ELEM[dt])
    _expect_device_tensor("residual", residual, n, _R_ELEM[dt])
    _expect_device_tensor("residual_ref", residual_ref, n, _R_ELEM[dt])
    if not counts_out.is_cuda or counts_out.numel() * counts_out.element_size() < 16:
        raise ValueError("counts_out must be a device tensor of at least 16 bytes")
    return n, dt


def addrms_gate_probe(y, y_ref, residual, residual_ref, dtype, tol: int, counts_out, stream=None) -> None:
    """counts_out: device tensor of four 32-bit counters (residual mismatches, y beyond tol, max y distance, 0)."""
    n, dt = _gate_args(y, y_ref, residual, residual_ref, dtype, counts_out)
    _check(load().addrms_gate_probe(_ptr(y), _ptr(y_ref), _ptr(residual), _ptr(residual_ref), n, dt, int(tol),
                                    _ptr(counts_out), _stream_ptr(stream, y)))


def addrms_gate_probe_noalloc(y, y_ref, residual, residual_ref, dtype, tol: int, counts_out, stream=None) -> None:
    """Same verdict as addrms_gate_probe; allocates nothing and does not wait for the stream."""
    n, dt = _gate_args(y, y_ref, residual, residual_ref, dtype, counts_out)
    _check(load().addrms_gate_probe_noalloc(_ptr(y), _ptr(y_ref), _ptr(residual), _ptr(residual_ref), n, dt, int(tol),
                                            _ptr(counts_out), _stream_ptr(stream, y)))


# ---- silu_and_mul (include/silumul.h) -------------------------------------------------

def silumul_algorithmic_bytes(M: int, d: int, dtype) -> int:
    return _check(load().silumul_algorithmic_bytes(M, d, _dtype_id(dtype)))


def silumul_run(x, out, M: int, d: int, dtype, cfg: Optional[Cfg] = None, stream=None) -> None:
    """out[i, j] = silu(x[i, j]) * x[i, d + j]; x is [M, 2d], out is [M, d], both on the device."""
    dt = _dtype_id(dtype)
    if dt not in _X_ELEM:
        raise ValueError(f"unknown dtype {dtype!r}")
    _expect_device_tensor("x", x, 2 * M * d, _X_ELEM[dt])
    _expect_device_tensor("out", out, M * d, _X_ELEM[dt])
    _check(load().silumul_run(_ptr(x), _ptr(out), M, d, _dtype_id(dtype),
                              byref(cfg) if cfg is not None else None, _stream_ptr(stream, x)))


def silumul_default_cfg(d: int, dtype) -> Cfg:
    c = Cfg()
    _check(load().silumul_default_cfg(d, _dtype_id(dtype), byref(c)))
    return c


def silumul_cfg_feasible(cfg: Cfg, M: int, d: int, dtype) -> Tuple[int, str, Resources]:
    buf = ctypes.create_string_buffer(512)
    res = Resources()
    st = load().silumul_cfg_feasible(byref(cfg), M, d, _dtype_id(dtype), buf, len(buf), byref(res))
    return int(st), buf.value.decode("utf-8", "replace"), res


def silumul_enumerate_feasible(M: int, d: int, dtype) -> Tuple[List[Cfg], int]:
    lib = load()
    grid = c_int64(0)
    n = _check(lib.silumul_enumerate_feasible(M, d, _dtype_id(dtype), None, 0, byref(grid)))
    arr = (Cfg * max(n, 1))()
    _check(lib.silumul_enumerate_feasible(M, d, _dtype_id(dtype), arr, n, byref(grid)))
    out = []
    for i in range(n):
        c = Cfg()
        ctypes.memmove(byref(c), byref(arr[i]), ctypes.sizeof(Cfg))
        out.append(c)
    return out, int(grid.value)


def silumul_tune(M: int, d: int, dtype, budget: Optional[Budget] = None) -> Tuple[Cfg, TuneReport]:
    c, rep = Cfg(), TuneReport()
    _check(load().silumul_tune(M, d, _dtype_id(dtype), byref(budget) if budget is not None else None,
                               byref(c), byref(rep)))
    return c, rep


def silumul_tune_with_backend(M: int, d: int, dtype, budget: Optional[Budget], measure, validate=None
                              ) -> Tuple[Cfg, TuneReport]:
    be = Backend()
    be.user = None
    be.measure = _wrap_measure(measure)
    be.validate = _wrap_validate(validate)
    c, rep = Cfg(), TuneReport()
    _check(load().silumul_tune_with_backend(M, d, _dtype_id(dtype), byref(budget) if budget is not None else None,
                                            byref(be), byref(c), byref(rep)))
    return c, rep


def silumul_select_general(shapes, dtype, budget: Optional[Budget] = None) -> Tuple[Cfg, GeneralReport]:
    """shapes: sequence of (M, d)."""
    c, rep = Cfg(), GeneralReport()
    _check(load().silumul_select_general(_shape_array(shapes), len(shapes), _dtype_id(dtype),
                                         byref(budget) if budget is not None else None, byref(c), byref(rep)))
    return c, rep


def silumul_tune_rounds(shapes, dtype, budget: Optional[Budget] = None) -> Tuple[Cfg, RoundsReport]:
    c, rep = Cfg(), RoundsReport()
    _check(load().silumul_tune_rounds(_shape_array(shapes), len(shapes), _dtype_id(dtype),
                                      byref(budget) if budget is not None else None, byref(c), byref(rep)))
    return c, rep


def silumul_measure(cfg: Optional[Cfg], M: int, d: int, dtype, warmup: int = 20, reps: int = 100,
                    rotate: bool = True) -> float:
    us = c_double(0.0)
    _check(load().silumul_measure(byref(cfg) if cfg is not None else None, M, d, _dtype_id(dtype), warmup, reps,
                                  int(rotate), byref(us)))
    return float(us.value)


def silumul_table_lookup(M: int, d: int, dtype) -> Optional[Cfg]:
    c = Cfg()
    st = load().silumul_table_lookup(M, d, _dtype_id(dtype), byref(c))
    if st == ERR_NO_RESULT:
        return None
    _check(st)
    return c


# ---- merge_attn_states (include/mergestates.h) ----------------------------------------

def _enumerate(fn_name: str, M: int, N: int, dtype) -> Tuple[List[Cfg], int]:
    fn = getattr(load(), fn_name)
    grid = c_int64(0)
    n = _check(fn(M, N, _dtype_id(dtype), None, 0, byref(grid)))
    arr = (Cfg * max(n, 1))()
    _check(fn(M, N, _dtype_id(dtype), arr, n, byref(grid)))
    out = []
    for i in range(n):
        c = Cfg()
        ctypes.memmove(byref(c), byref(arr[i]), ctypes.sizeof(Cfg))
        out.append(c)
    return out, int(grid.value)


def mergestates_algorithmic_bytes(rows: int, d: int, dtype) -> int:
    return _check(load().mergestates_algorithmic_bytes(rows, d, _dtype_id(dtype)))


def mergestates_run(v_a, s_a, v_b, s_b, v_out, s_out, rows: int, d: int, dtype, cfg: Optional[Cfg] = None,
                    stream=None) -> None:
    """Merge two partial attention states; v tensors [rows, d], scores fp32 [rows], all on the device."""
    dt = _dtype_id(dtype)
    if dt not in _X_ELEM:
        raise ValueError(f"unknown dtype {dtype!r}")
    for name, t in (("v_a", v_a), ("v_b", v_b), ("v_out", v_out)):
        _expect_device_tensor(name, t, rows * d, _X_ELEM[dt])
    for name, t in (("s_a", s_a), ("s_b", s_b), ("s_out", s_out)):
        _expect_device_tensor(name, t, rows, "float32")
    _check(load().mergestates_run(_ptr(v_a), _ptr(s_a), _ptr(v_b), _ptr(s_b), _ptr(v_out), _ptr(s_out), rows, d,
                                  _dtype_id(dtype), byref(cfg) if cfg is not None else None, _stream_ptr(stream, v_a)))


def mergestates_default_cfg(d: int, dtype) -> Cfg:
    c = Cfg()
    _check(load().mergestates_default_cfg(d, _dtype_id(dtype), byref(c)))
    return c


def mergestates_cfg_feasible(cfg: Cfg, rows: int, d: int, dtype) -> Tuple[int, str, Resources]:
    buf = ctypes.create_string_buffer(512)
    res = Resources()
    st = load().mergestates_cfg_feasible(byref(cfg), rows, d, _dtype_id(dtype), buf, len(buf), byref(res))
    return int(st), buf.value.decode("utf-8", "replace"), res


def mergestates_enumerate_feasible(rows: int, d: int, dtype) -> Tuple[List[Cfg], int]:
    return _enumerate("mergestates_enumerate_feasible", rows, d, dtype)


def mergestates_tune(rows: int, d: int, dtype, budget: Optional[Budget] = None) -> Tuple[Cfg, TuneReport]:
    c, rep = Cfg(), TuneReport()
    _check(load().mergestates_tune(rows, d, _dtype_id(dtype), byref(budget) if budget is not None else None,
                                   byref(c), byref(rep)))
    return c, rep


def mergestates_tune_with_backend(rows: int, d: int, dtype, budget: Optional[Budget], measure, validate=None
                                  ) -> Tuple[Cfg, TuneReport]:
    be = Backend()
    be.user = None
    be.measure = _wrap_measure(measure)
    be.validate = _wrap_validate(validate)
    c, rep = Cfg(), TuneReport()
    _check(load().mergestates_tune_with_backend(rows, d, _dtype_id(dtype),
                                                byref(budget) if budget is not None else None, byref(be),
                                                byref(c), byref(rep)))
    return c, rep


def mergestates_select_general(shapes, dtype, budget: Optional[Budget] = None) -> Tuple[Cfg, GeneralReport]:
    """shapes: sequence of (rows, d)."""
    c, rep = Cfg(), GeneralReport()
    _check(load().mergestates_select_general(_shape_array(shapes), len(shapes), _dtype_id(dtype),
                                             byref(budget) if budget is not None else None, byref(c), byref(rep)))
    return c, rep


def mergestates_tune_rounds(shapes, dtype, budget: Optional[Budget] = None) -> Tuple[Cfg, RoundsReport]:
    c, rep = Cfg(), RoundsReport()
    _check(load().mergestates_tune_rounds(_shape_array(shapes), len(shapes), _dtype_id(dtype),
                                          byref(budget) if budget is not None else None, byref(c), byref(rep)))
    return c, rep


def mergestates_measure(cfg: Optional[Cfg], rows: int, d: int, dtype, warmup: int = 20, reps: int = 100,
                        rotate: bool = True) -> float:
    us = c_double(0.0)
    _check(load().mergestates_measure(byref(cfg) if cfg is not None else None, rows, d, _dtype_id(dtype), warmup, reps,
                                      int(rotate), byref(us)))
    return float(us.value)


def mergestates_table_lookup(rows: int, d: int, dtype) -> Optional[Cfg]:
    c = Cfg()
    st = load().mergestates_table_lookup(rows, d, _dtype_id(dtype), byref(c))
    if st == ERR_NO_RESULT:
        return None
    _check(st)
    return c
