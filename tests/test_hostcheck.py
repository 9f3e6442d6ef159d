"""The host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): a second build of
flux_api.hip as plain C++ with launchers that report "no device", driven by a C++ program that calls every entry
point with ordinary and extreme arguments.  Any sanitizer report aborts the program."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2604_07394_amd", "lib")


def test_c_abi_host_side_is_clean_under_asan_and_ubsan():
    exe = os.path.join(LIB, "flux_hostcheck")
    if not (os.path.exists(exe) and os.path.exists(os.path.join(LIB, "libflux_hostcheck.so"))):
        from paper_2604_07394_amd import build
        build.build_hostcheck()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    proc = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert proc.returncode == 0, proc.stdout + proc.stderr
    assert "hostcheck ok" in proc.stdout
    assert "runtime error" not in proc.stderr and "AddressSanitizer" not in proc.stderr
