"""Host AddressSanitizer + UBSan pass over the C ABI's argument validation and host-side plan building: the library is
rebuilt with its host code instrumented (device code untouched; nothing here needs or uses a GPU) and a small host
program (tests/abi_sanitizer_driver.cpp) walks the validation paths.  A sanitizer report or an unexpected return code
fails the test."""
import os
import subprocess

from paper_2407_08296_amd import build as qg_build

HERE = os.path.dirname(os.path.abspath(__file__))


def test_abi_validation_paths_under_asan_ubsan():
    exe = qg_build.build_sanitized(os.path.join(HERE, "abi_sanitizer_driver.cpp"))
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"   # the HIP runtime keeps allocations until exit
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    p = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    out = p.stdout + p.stderr
    assert p.returncode == 0, out[-4000:]
    assert "sanitizer driver ok" in p.stdout
    assert "ERROR: AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
