"""The host side of the C ABI (argument validation and workspace carving) under the undefined-behaviour
sanitizer: tests/test_abi.py is run again, in a child process, against a library whose api.hip host code is
built with -fsanitize=undefined in trap mode.  No GPU is touched: every call returns before its first
launch.  A trap (signed overflow in a size computation, a misaligned or out-of-bounds access, a bad shift,
a truncating conversion) kills the child with SIGILL and fails this test.

AddressSanitizer is not used here: an instrumented shared library needs its runtime loaded ahead of
everything else in the process, which an uninstrumented Python cannot give it."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_abi_host_code_is_clean_under_ubsan():
    from paper_2512_07993_amd.build import build_host_sanitized
    lib = build_host_sanitized()
    env = dict(os.environ, SKIPKV_ABI_TEST_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_abi.py")], cwd=ROOT, env=env, capture_output=True, text=True,
                       timeout=600)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, "ABI tests against the sanitized build failed (rc %d; -4 = sanitizer trap):\n%s" % (r.returncode, tail)
    assert " passed" in r.stdout
