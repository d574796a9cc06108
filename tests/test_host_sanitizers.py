"""The host-only part of the library (deriver, table, search, general selection, outer loop, rule audit)
built with the address and undefined-behaviour sanitizers and driven through its C entry points.
No GPU and no HIP: these sources make no HIP call, so a plain g++ build of them is the same code."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_12698_amd", "csrc")
BUILD = os.path.join(ROOT, "paper_2601_12698_amd", "_build")
HOST_SOURCES = ["addrms_cfg.cpp", "addrms_table.cpp", "addrms_search.cpp", "addrms_general.cpp", "addrms_audit.cpp"]


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    if not os.path.exists(os.path.join(BUILD, "gen_resources.inc")):
        pytest.skip("the generated instance and resource tables are not present (build the library first)")
    exe = str(tmp_path / "host_sanitize_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", BUILD,
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), *[os.path.join(CSRC, s) for s in HOST_SOURCES],
           "-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe, str(tmp_path)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600, env=env)
    assert r.returncode == 0 and "host sanitize driver: ok" in r.stdout, r.stdout[-6000:]
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout, r.stdout[-6000:]
