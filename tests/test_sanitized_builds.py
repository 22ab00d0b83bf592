"""CPU-only sanitizer pass (opt-in: SRS_RUN_SANITIZERS=1, about three minutes).

  * the oracle, compiled with gcc -fsanitize=address,undefined, under every oracle test of the CPU suite;
  * the host code of libsrs.so (bucket / segment / tile tables, argument checks), compiled with hipcc and
    -Xarch_host -fsanitize=address / undefined, under the host-layout and ABI tests.

Each leg runs pytest in a child process with the sanitizer runtime preloaded into the interpreter and the library
under test selected by SRS_ORACLE_LIBRARY / SRS_LIBRARY.  Never run on a GPU machine: device code is not instrumented
and no test selected here touches a device."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.skipif(os.environ.get("SRS_RUN_SANITIZERS") != "1",
                                reason="opt-in: set SRS_RUN_SANITIZERS=1 (CPU only, about three minutes)")


def _run(env_extra, preload, tests):
    env = dict(os.environ)
    env.pop("SRS_RUN_SANITIZERS", None)
    env.update(env_extra)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", *tests], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=1500)
    assert r.returncode == 0, (r.stdout[-3000:] + r.stderr[-3000:])
    assert "passed" in r.stdout and "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
    return r.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    sys.path.insert(0, ROOT)
    import oracle
    lib = oracle.build_sanitized(str(tmp_path / "libsrs_oracle_san.so"))
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    tests = sorted(os.path.join("tests", f) for f in os.listdir(os.path.join(ROOT, "tests")) if f.startswith("test_oracle"))
    out = _run({"SRS_ORACLE_LIBRARY": lib}, asan, tests)
    print(out[-300:])


def test_host_code_of_the_library_under_asan_and_ubsan(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2605_07330_amd import build
    rt = build.clang_asan_runtime()
    if not rt:
        pytest.skip("clang's ASan runtime is not installed")
    lib = build.build_lib_host_sanitized(str(tmp_path / "libsrs_san.so"))
    out = _run({"SRS_LIBRARY": lib}, rt, ["tests/test_host_layout.py", "tests/test_abi_exports.py"])
    print(out[-300:])
