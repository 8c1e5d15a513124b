"""The host side of the C ABI under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only):
argument checks of every entry point, tpla_validate_block_table and the host eigen-solver behind
tpla_pca_basis, driven by tests/host_sanitizers/abi_host_driver.cpp.  Device code is compiled as
usual and never runs here."""
import os
import subprocess

from paper_2508_15881_amd import build as tb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_abi_host_side_is_clean_under_asan_and_ubsan():
    exe = os.path.join(ROOT, "_build", "host_sanitized", "abi_host_driver")
    tb.build_host_sanitized(os.path.join(ROOT, "tests", "host_sanitizers", "abi_host_driver.cpp"), exe)
    syms = subprocess.run(["nm", exe], capture_output=True, text=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms          # the build really is instrumented
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "all expectations held" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
