"""The boundary is a C ABI: include/srs.h must be plain C, and a C program that knows nothing but that header
and the HIP runtime's C API must get the oracle's result out of libsrs.so (tests/c_abi/roundtrip.c, built by
__graft_entry__.build())."""
import os
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CONSUMER = os.path.join(ROOT, "tests", "c_abi", "roundtrip")


def test_header_is_plain_c99(tmp_path):
    src = tmp_path / "only_header.c"
    src.write_text('#include "srs.h"\nint main(void) { int (*f)(void) = srs_version; return f != 0 ? 0 : 1; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_c_consumer_is_built_and_links_against_the_library():
    if not os.path.exists(CONSUMER):                  # a tree that was never built: gcc takes a fraction of a second
        from paper_2605_07330_amd import build
        if not os.path.exists(build.LIB):
            build.build_lib()
        build.build_c_consumer()
    r = subprocess.run(["readelf", "-d", CONSUMER], capture_output=True, text=True)
    assert r.returncode == 0 and "libsrs.so" in r.stdout and "libamdhip64" in r.stdout


@pytest.mark.gpu
@pytest.mark.parametrize("n,be,cap,density,mode", [(1_000_003, 300_000, 300_000, 0.01, ""), (70_001, 70_001, 512, 0.02, ""),
                                                   (4096, 1000, 1000, 1.0, ""), (1_000_003, 300_000, 300_000, 0.01, "noalloc"),
                                                   (1_000_003, 300_000, 300_000, 0.01, "secondpass"),
                                                   (500_001, 70_001, 512, 0.02, "secondpass")])
def test_c_program_round_trip_matches_oracle(tmp_path, n, be, cap, density, mode):
    assert os.path.exists(CONSUMER), "run __graft_entry__.build() first"
    rng = np.random.default_rng(n)
    old = rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    new = old.copy()
    pos = np.flatnonzero(rng.random(n) < density)
    new[pos] ^= rng.integers(1, 1 << 16, size=pos.size, dtype=np.uint16)
    (tmp_path / "old.u16").write_bytes(old.tobytes()); (tmp_path / "new.u16").write_bytes(new.tobytes())
    out = tmp_path / "out.bin"
    print(f"c consumer: n={n} be={be} cap={cap} density={density} {mode}", flush=True)
    r = subprocess.run([CONSUMER, str(tmp_path / "old.u16"), str(tmp_path / "new.u16"), str(n), str(be), str(cap),
                        str(out)] + ([mode] if mode else []), capture_output=True, text=True, timeout=100)
    assert r.returncode == 0, r.stdout + r.stderr
    nb = -(-n // be)
    raw = np.fromfile(out, dtype=np.uint8)
    o = 0
    def take(count, dtype):
        nonlocal o
        nbytes = count * np.dtype(dtype).itemsize
        a = raw[o:o + nbytes].view(dtype); o += nbytes
        return a
    counts = take(nb, np.uint32); I = take(nb * cap, np.int32).reshape(nb, cap); V = take(nb * cap, np.uint16).reshape(nb, cap)
    snap = take(n, np.uint16); roll = take(n, np.uint16); flags = int(take(1, np.uint32)[0])
    assert o == raw.size

    want_snap = old.copy()
    wI, wV, wc, overflowed = oracle.extract(want_snap, new, be, cap=cap)
    assert np.array_equal(counts, wc) and np.array_equal(I, wI) and np.array_equal(V, wV)
    assert np.array_equal(snap, new) and np.array_equal(want_snap, new)
    want_roll = old.copy()
    assert oracle.apply(want_roll, be, wI, wV, wc) == oracle.OK
    assert np.array_equal(roll, want_roll)
    assert (flags != 0) == (overflowed > 0)
    if not overflowed:
        assert np.array_equal(roll, new)
