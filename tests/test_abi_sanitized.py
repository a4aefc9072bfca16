"""Host-side sanitizer run of the C ABI (no GPU): the library's host code and
tests/abi_host_check.cpp are compiled with -fsanitize=address,undefined (host side only) and the
program walks the argument checks and error paths of every entry point.  Any heap error or
undefined behaviour on those paths aborts the program."""
import os
import subprocess


def test_abi_argument_checks_under_asan_and_ubsan():
    from paper_2601_19278_amd import build
    exe = build.build_sanitized(verbose=False)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "abi host check: ok" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
