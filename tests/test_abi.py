"""The C-ABI library loads without a GPU and exports every symbol the header
declares; the binding declares the same set."""
import ctypes
import os
import re

from paper_2601_12698_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for header in ("addrms.h", "silumul.h", "mergestates.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b((?:addrms|silumul|mergestates)_[a-z_0-9]+)\s*\(", text))
    return names


def test_header_symbols_are_exported():
    lib = ctypes.CDLL(B.LIB_PATH)
    names = _declared()
    assert len(names) >= 30 and any(n.startswith('silumul_') for n in names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in addrms.h but not exported"


def test_binding_covers_header():
    assert set(B.SIGNATURES) == _declared()
    for n in B.SIGNATURES:
        assert callable(getattr(B, n)), f"binding has no function named {n}"


def test_struct_sizes_match_c_layout():
    # addrms_cfg: 8 x int32; addrms_resources: 16 x int32
    assert ctypes.sizeof(B.Cfg) == 32
    assert ctypes.sizeof(B.Resources) == 64
    assert ctypes.sizeof(B.Budget) == 8 + 4 * 10 + 8 + 8
    assert ctypes.sizeof(B.RoundInfo) == 4 + 4 + 8 + 8 + 32
    assert ctypes.sizeof(B.RoundsReport) == 4 + 4 + 8 + B.MAX_ROUNDS * 56 + ctypes.sizeof(B.GeneralReport)
    assert ctypes.sizeof(B.GeneralReport) == 8 + 8 * 4 + 8 * 16 * 3 + 32 * 16
    assert ctypes.sizeof(B.Shape) == 16
    assert ctypes.sizeof(B.TuneReport) == 8 * 5 + 8 * 4 + 32 * 2 + 8 + 32 * 8 + 8 * 8


def test_version_and_bytes_formula():
    assert "gfx950" in B.addrms_version()
    assert B.addrms_algorithmic_bytes(4096, 4096, "bf16") == 134225920
    assert B.addrms_algorithmic_bytes(32768, 7168, "bf16") == 1879062528
    assert B.addrms_algorithmic_bytes(8192, 5120, "fp16_res32") == 8192 * 5120 * 12 + 5120 * 2
    assert B.addrms_algorithmic_bytes(1, 8192, "bf16") == 81920
    assert B.load().addrms_algorithmic_bytes(4, 4, 7) == B.ERR_UNSUPPORTED_DTYPE
    assert B.load().addrms_algorithmic_bytes(4, 0, 0) == B.ERR_INVALID_ARG


def test_run_rejects_bad_arguments_without_a_gpu():
    lib = B.load()
    c = B.make_cfg(8, 256, 1, unroll=2)
    assert lib.addrms_run(None, None, None, 1e-6, 4, 4096, B.BF16, c, None) == B.ERR_INVALID_ARG
    assert "NULL" in B.addrms_last_error()
    assert lib.addrms_run(None, None, None, 1e-6, 0, 4096, B.BF16, c, None) == B.OK       # M == 0: no-op
    assert lib.addrms_run(None, None, None, 1e-6, 4, -1, B.BF16, c, None) == B.ERR_INVALID_ARG
    assert lib.addrms_run(None, None, None, 1e-6, 4, 4096, 11, c, None) == B.ERR_UNSUPPORTED_DTYPE
    # an infeasible cfg is reported before pointers are looked at only if pointers are valid; use fake aligned ones
    bad = B.make_cfg(8, 1000, 1)
    assert lib.addrms_run(4096, 8192, 12288, 1e-6, 4, 4096, B.BF16, bad, None) == B.ERR_INFEASIBLE_CFG
    ok = B.make_cfg(8, 256, 1, unroll=2)
    assert lib.addrms_run(4098, 8192, 12288, 1e-6, 4, 4096, B.BF16, ok, None) == B.ERR_MISALIGNED
