"""Specialised table D_spec (host logic, no GPU): insert, exact and nearest-M
lookup, persistence, and refusal of missing or corrupt files."""
import os

import pytest

from paper_2601_12698_amd import binding as B


@pytest.fixture(autouse=True)
def clean_table():
    B.addrms_table_clear()
    yield
    B.addrms_table_clear()


def test_insert_lookup_exact_and_nearest():
    a = B.make_cfg(8, 1024, 1)
    b = B.make_cfg(8, 256, 4, unroll=2, flags=B.FLAG_NONTEMPORAL)
    B.addrms_table_insert(1, 8192, "bf16", a, 3.0)
    B.addrms_table_insert(256, 8192, "bf16", b, 9.0)
    assert B.addrms_table_size() == 2
    assert B.addrms_table_lookup(1, 8192, "bf16").as_tuple() == a.as_tuple()
    assert B.addrms_table_lookup(256, 8192, "bf16").as_tuple() == b.as_tuple()
    assert B.addrms_table_lookup(2, 8192, "bf16").as_tuple() == a.as_tuple()        # nearest in ratio
    assert B.addrms_table_lookup(100, 8192, "bf16").as_tuple() == b.as_tuple()
    assert B.addrms_table_lookup(100000, 8192, "bf16").as_tuple() == b.as_tuple()
    # b packs 4 rows per workgroup: not feasible for M = 3, so the fallback must skip it
    assert B.addrms_table_lookup(3, 8192, "bf16").as_tuple() == a.as_tuple()
    assert B.addrms_table_lookup(16, 4096, "bf16") is None                           # other N
    assert B.addrms_table_lookup(16, 8192, "fp16") is None                           # other dtype


def test_insert_rejects_infeasible():
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_table_insert(4096, 4096, "bf16", B.make_cfg(8, 1024, 1))
    assert e.value.status == B.ERR_INFEASIBLE_CFG
    assert B.addrms_table_size() == 0


def test_save_load_round_trip(tmp_path):
    a = B.make_cfg(8, 576, 1, flags=B.FLAG_NONTEMPORAL, max_waves_per_simd=5)
    b = B.make_cfg(4, 128, 2, reduce=B.REDUCE_LDS, unroll=2)
    B.addrms_table_insert(4096, 4096, "bf16", a, 23.5)
    B.addrms_table_insert(8192, 1000, "fp16_res32", b, 17.25)
    path = str(tmp_path / "table.txt")
    B.addrms_table_save(path)
    B.addrms_table_clear()
    assert B.addrms_table_size() == 0
    B.addrms_table_load(path)
    assert B.addrms_table_size() == 2
    assert B.addrms_table_lookup(4096, 4096, "bf16").as_tuple() == a.as_tuple()
    assert B.addrms_table_lookup(8192, 1000, "fp16_res32").as_tuple() == b.as_tuple()


HDR = "addrms-table 4\narch gfx950\nlibrary %s\n" % B.addrms_version().split()[0]
GOOD = "0 0 1 8192 8 1024 1 0 1 0 0 0 3.0\n"


@pytest.mark.parametrize("content", [
    "",                                                     # empty
    "not a table\n" + GOOD,                                 # wrong magic
    "addrms-table 3 gfx950\n0 0 1 8192 8 1024 1 0 1 0 0 3.0\n",   # older format version
    "addrms-table 4\n" + GOOD,                              # no arch line
    "addrms-table 4\narch gfx950\n" + GOOD,                 # no library line
    "addrms-table 4\narch gfx942\nlibrary 0.2.0\n" + GOOD,  # tuned on another architecture
    "addrms-table 4\narch gfx9500\nlibrary 0.2.0\n" + GOOD,
    "addrms-table 4\narch gfx950\nlibrary 0.1.0\n" + GOOD,  # written by a library with other kernel instances
    "addrms-table 4\narch gfx950\nlibrary 1.2.0\n" + GOOD,
    "addrms-table 4\narch gfx950\nlibrary 0.20.0\n" + GOOD,
    HDR,                                                    # a header alone is a valid, empty table: must NOT fail (see below)
    HDR + "0 0 1 8192 8 1024 1 0 1 0 0\n",                  # truncated entry
    HDR + "0 0 1 8192 8 1024 1 0 1 0 0 3.0\n",              # entry of the previous format (no walk column)
    HDR + "0 0 1 8192 8 1024 1 0 1 0 0 0 3.0 junk\n",
    HDR + "0 0 4096 4096 8 1024 1 0 1 0 0 0 3.0\n",         # parses, but cfg infeasible for that shape
    HDR + "0 7 1 8192 8 1024 1 0 1 0 0 0 3.0\n",            # bad dtype
    HDR + "5 0 1 8192 8 1024 1 0 1 0 0 0 3.0\n",            # unknown operator
    HDR + "0 0 1 8192 8 1024 1 0 1 0 0 4 3.0\n",            # a walk length without a persistent grid
])
def test_corrupt_file_leaves_table_unchanged(tmp_path, content):
    keep = B.make_cfg(8, 1024, 1)
    B.addrms_table_insert(1, 8192, "bf16", keep, 3.0)
    path = str(tmp_path / "bad.txt")
    with open(path, "w") as f:
        f.write(content)
    if content == HDR:                                      # control: the header itself is accepted
        B.addrms_table_load(path)
        assert B.addrms_table_size() == 1
        return
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_table_load(path)
    assert e.value.status == B.ERR_IO
    assert B.addrms_table_size() == 1
    assert B.addrms_table_lookup(1, 8192, "bf16").as_tuple() == keep.as_tuple()


def test_missing_file_and_unwritable_path(tmp_path):
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_table_load(str(tmp_path / "nope.txt"))
    assert e.value.status == B.ERR_IO
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_table_save(str(tmp_path / "no_such_dir" / "t.txt"))
    assert e.value.status == B.ERR_IO


def test_two_pass_entries_round_trip_and_resolve_long_rows(tmp_path):
    """A table entry for a row beyond the register cache carries the two-pass flag through save/load, and the
    nearest-M fallback hands it to other row counts of the same N."""
    c = B.make_cfg(8, 768, 1, reduce=B.REDUCE_LDS, unroll=4, flags=B.FLAG_TWO_PASS | B.FLAG_NONTEMPORAL)
    B.addrms_table_insert(4096, 40960, "bf16", c, 261.7)
    with pytest.raises(B.AddrmsError):                       # a single-pass cfg cannot hold such a row
        B.addrms_table_insert(4096, 40960, "bf16", B.make_cfg(8, 1024, 1), 1.0)
    with pytest.raises(B.AddrmsError):                       # and the two-pass form is refused where one pass does
        B.addrms_table_insert(4096, 4096, "bf16", B.make_cfg(8, 256, 1, unroll=2, flags=B.FLAG_TWO_PASS), 1.0)
    path = str(tmp_path / "t.txt")
    B.addrms_table_save(path)
    B.addrms_table_clear()
    B.addrms_table_load(path)
    assert B.addrms_table_lookup(4096, 40960, "bf16").as_tuple() == c.as_tuple()
    assert B.addrms_table_lookup(100, 40960, "bf16").as_tuple() == c.as_tuple()
    assert B.addrms_table_lookup(100, 40968, "bf16") is None


def test_file_names_its_architecture_and_library_and_a_patch_release_may_read_it(tmp_path):
    c = B.make_cfg(8, 256, 1, unroll=2, flags=B.FLAG_NONTEMPORAL | B.FLAG_PERSISTENT | B.FLAG_DEFER_STORE, walk=4)
    B.addrms_table_insert(32768, 4096, "bf16", c, 100.0)
    path = str(tmp_path / "t.txt")
    B.addrms_table_save(path)
    lines = open(path).read().splitlines()
    assert lines[0] == "addrms-table 4" and lines[1] == "arch gfx950"
    version = B.addrms_version().split()[0]
    assert lines[2] == "library " + version
    major, minor, _ = version.split(".")
    with open(path, "w") as f:                              # same major.minor, another patch level: same instances
        f.write("\n".join([lines[0], lines[1], f"library {major}.{minor}.99"] + lines[3:]) + "\n")
    B.addrms_table_clear()
    B.addrms_table_load(path)
    got = B.addrms_table_lookup(32768, 4096, "bf16")
    assert got.as_tuple() == c.as_tuple() and got.walk == 4
    with open(path, "w") as f:
        f.write("\n".join([lines[0], "arch gfx90a", lines[2]] + lines[3:]) + "\n")
    with pytest.raises(B.AddrmsError) as e:
        B.addrms_table_load(path)
    assert e.value.status == B.ERR_IO and "gfx90a" in e.value.message


def _run_py(code, env_extra):
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, PYTHONPATH=root, **env_extra)
    r = subprocess.run([sys.executable, "-c", code], env=env, cwd=root, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=300)
    assert r.returncode == 0, r.stdout
    return r.stdout


def test_tune_cache_file_named_by_the_environment(tmp_path):
    """ADDRMS_TABLE_FILE: what one process inserts is what the next process looks up, without either
    calling save or load; a file the library cannot load is neither read nor overwritten."""
    path = str(tmp_path / "cache.txt")
    writer = ("from paper_2601_12698_amd import binding as B\n"
              "assert B.addrms_table_size() == 0\n"
              "B.addrms_table_insert(4096, 4096, 'bf16', B.make_cfg(8, 128, 8, 0, 4, 7, 0), 22.5)\n"
              "B.addrms_table_insert(64, 8192, 'bf16', B.make_cfg(8, 512, 1, 0, 2, 0, 0), 3.5)\n")
    _run_py(writer, {"ADDRMS_TABLE_FILE": path})
    text = open(path).read().splitlines()
    assert text[0].startswith("addrms-table") and text[1] == "arch gfx950" and len([l for l in text if l and l[0].isdigit()]) == 2
    assert not os.path.exists(path + ".tmp")
    reader = ("from paper_2601_12698_amd import binding as B\n"
              "print(B.addrms_table_lookup(4096, 4096, 'bf16').as_tuple())\n"
              "print(B.addrms_table_lookup(128, 8192, 'bf16').as_tuple())\n"
              "print(B.addrms_table_size())\n")
    out = _run_py(reader, {"ADDRMS_TABLE_FILE": path}).splitlines()
    assert out[-3:] == ["(8, 128, 8, 0, 4, 7, 0, 0)", "(8, 512, 1, 0, 2, 0, 0, 0)", "2"]
    # without the variable the same process sees an empty table
    out = _run_py("from paper_2601_12698_amd import binding as B\nprint(B.addrms_table_lookup(4096, 4096, 'bf16'))\n"
                  "print(B.addrms_table_size())\n", {"ADDRMS_TABLE_FILE": ""}).splitlines()
    assert out[-2:] == ["None", "0"]
    # a file for another architecture: not loaded, and an insertion does not write over it
    foreign = str(tmp_path / "foreign.txt")
    body = "addrms-table 4\narch gfx942\nlibrary 0.2.0\n0 0 4096 4096 8 128 8 0 4 7 0 0 22.5\n"
    open(foreign, "w").write(body)
    out = _run_py(writer.replace("assert B.addrms_table_size() == 0\n", "") + "print(B.addrms_table_size())\n",
                  {"ADDRMS_TABLE_FILE": foreign}).splitlines()
    assert out[-1] == "2" and open(foreign).read() == body
