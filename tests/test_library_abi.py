"""CPU-side checks of the built library: it loads, exports every declared symbol, and its host-only
entry points (sizes, tables, error strings) agree with the oracle.  No GPU work is started."""
import os
import re

import numpy as np
import pytest

from oracle import eden_oracle as o

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def eden():
    from paper_2108_08842_amd import eden as e
    if not os.path.exists(e._LIB_PATH):
        from paper_2108_08842_amd import build
        build.build(verbose=False)
    e.lib()
    return e


def test_every_declared_symbol_is_exported(eden):
    header = open(os.path.join(ROOT, "include", "eden.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(eden_[a-z_]+)\s*\(", header))
    assert {"eden_encode", "eden_decode_accumulate", "eden_finalize_mean", "eden_create"} <= declared
    assert declared == set(eden.EXPORTS)
    for name in declared:
        assert getattr(eden.lib(), name) is not None


def test_message_bytes_matches_oracle(eden):
    for d in (1, 2, 3, 64, 1000, 1024, 4097, 1 << 20, 11_173_962, 1 << 27):
        for b in (128, 256, 512, 1024):
            if b == 128 and d == 1:
                assert eden.message_bytes(d, b) == 0
                continue
            assert eden.message_bytes(d, b) == o.message_bytes(d, b)
        for b in (384, 896, eden.B_COIN(1.5), eden.B_COIN(3.99), eden.B_GRID(0.5), 1536, eden.B_HALF_PRE, eden.B_SPARSE(9)):
            if d >= 2:
                assert eden.message_bytes(d, b) == o.message_bytes(d, b), (d, b)
    assert eden.message_bytes(0, 256) == 0
    assert eden.message_bytes(100, 300) == 0
    assert eden.message_bytes(100, 0x40000 | 512) == 0 and eden.message_bytes(100, 0x40000 | 1100) == 0


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 6, 7, 8])
def test_library_tables_match_oracle_tables(eden, bits):
    # two independent Lloyd-Max solvers (C++ on the positive half line, numpy on the full line; above 32 levels both
    # shoot from the smallest level, where the end of the chain is the least accurate: 3e-10 at 256 levels)
    t, q = eden.get_tables(bits)
    to, qo = o.tables(bits)
    tol = 2e-12 if bits <= 5 else 1e-9
    np.testing.assert_allclose(t, to, atol=tol)
    np.testing.assert_allclose(q, qo, atol=tol)
    # and fp32 rounding of either is the same number almost everywhere
    assert np.sum(np.float32(q) != np.float32(qo)) <= (0 if bits <= 5 else 2)


def test_message_length_from_a_header(eden):
    # what has to travel: the whole buffer for every budget but the coin budgets, whose second part follows the coins
    x = np.random.default_rng(3).standard_normal(3000)
    for b in (256, 512, 384, eden.B_GRID(0.5), eden.B_HALF_PRE, eden.B_SPARSE(7), eden.B_COIN(1.3), eden.B_COIN(3.5)):
        m = o.encode(x, 4, 1, b)
        raw = m.to_bytes()
        assert eden.message_length(raw) == len(raw) <= eden.message_bytes(3000, b)
    assert eden.message_length(bytes(64)) == 0


def test_no_wide_buffer_store_keeps_its_offset_in_a_scalar_register(tmp_path):
    # the build's own check (a 128-bit buffer store with a scalar offset lost its first dword under load on the MI355X):
    # it recognises the instruction form, and the assembly the last build left has none
    import glob
    from paper_2108_08842_amd import build
    sample = tmp_path / "k-hip-amdgcn-amd-amdhsa-gfx950.s"
    sample.write_text("\tbuffer_store_dwordx4 v[6:9], v98, s[4:7], s0 offen nt\n"
                      "\tbuffer_store_dwordx4 v[2:5], v12, s[4:7], 0 offen nt\n"
                      "\tbuffer_store_dwordx2 v[2:3], v12, s[4:7], s1 offen\n")
    bad = build.wide_stores_with_scalar_offset(str(tmp_path))
    assert len(bad) == 1 and ":1:" in bad[0]
    if not glob.glob(os.path.join(build.OBJ_DIR, "*-hip-amdgcn-amd-amdhsa-gfx950.s")):
        pytest.skip("no device assembly from a build in this tree")
    assert build.wide_stores_with_scalar_offset() == []


def test_error_strings(eden):
    assert eden.strerror(0) == "ok"
    assert "argument" in eden.strerror(eden.ERR_INVALID_ARG)
    assert "small" in eden.strerror(eden.ERR_CAPACITY)


def test_header_is_plain_c_and_library_links_from_c(eden, tmp_path):
    """A C99 program that includes include/eden.h, links the library and calls the entry points that need no GPU."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    libdir = os.path.join(ROOT, "paper_2108_08842_amd")
    exe = tmp_path / "abi_check"
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c", "abi_check.c"), "-o", str(exe), "-L", libdir, "-leden_hip", "-lm",
           f"-Wl,-rpath,{libdir}"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True)
    assert "abi ok" in out.stdout
