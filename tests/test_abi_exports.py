"""The C-ABI library loads without a GPU and exports every symbol include/srs.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "srs.h")
LIB = os.path.join(ROOT, "paper_2605_07330_amd", "libsrs.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(srs_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_calls():
    names = declared_functions()
    for n in ("srs_extract", "srs_apply", "srs_extract_multi", "srs_apply_multi"):
        assert n in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        from paper_2605_07330_amd import build
        build.build_lib()
    lib = ctypes.CDLL(LIB)
    for n in declared_functions():
        assert hasattr(lib, n), f"libsrs.so does not export {n}"


def test_binding_lists_the_same_symbols():
    from paper_2605_07330_amd import srs
    assert sorted(srs.EXPORTS) == declared_functions()
    assert srs.version() >= 100
    assert srs._lib.srs_strerror(-1).decode() == "invalid argument"


def test_host_side_argument_checks_need_no_gpu():
    """Calls that must be rejected before anything touches a device."""
    from paper_2605_07330_amd import srs
    lib = srs._lib
    assert lib.srs_create(None, 0) == srs.ERR_INVALID
    assert lib.srs_destroy(None) == srs.ERR_INVALID
    assert lib.srs_extract(None, None, None, 8, 8, None, None, None, 8, None) == srs.ERR_INVALID
    assert lib.srs_apply(None, None, 8, 8, None, None, None, 8, None) == srs.ERR_INVALID
    assert lib.srs_plan_destroy(None) == srs.ERR_INVALID
    assert lib.srs_stream_probe_sink_words(1 << 20) >= 32


def test_a_missing_library_fails_loudly_and_nothing_stands_in_for_it(tmp_path):
    """The binding has no fallback: without libsrs.so the import itself fails, naming the file and how to build it."""
    import subprocess
    import sys
    env = dict(os.environ, SRS_LIBRARY=str(tmp_path / "no_such_libsrs.so"))
    r = subprocess.run([sys.executable, "-c", "from paper_2605_07330_amd import srs"], capture_output=True, text=True,
                       env=env, cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))), timeout=300)
    assert r.returncode != 0
    assert "no_such_libsrs.so is missing" in r.stderr and "no fallback" in r.stderr
