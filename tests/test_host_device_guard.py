"""The device guard of the C ABI layer, exercised on the host with a counting stand-in for the GPU runtime
(a guard that restored the caller's device through a nested guard recursed without end when the caller's
device differed from the context's; one-GPU machines never take that branch)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_device_guard_switches_and_restores_once(tmp_path):
    exe = str(tmp_path / "device_guard_test")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-Wall", "-Wextra", "-Werror",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-I", os.path.join(ROOT, "paper_2605_07330_amd", "csrc"),
                           os.path.join(HERE, "host", "device_guard_test.cpp"), "-o", exe])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "FAILED" not in out.stdout and out.stdout.count(": ok") == 9, out.stdout
