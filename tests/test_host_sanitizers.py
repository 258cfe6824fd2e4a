"""The host side of the library (graph and CSR ingestion, eigen-solve, consensus factors and their on-chip
program, the neighbour-table and polynomial builders, argument checks) under AddressSanitizer and
UndefinedBehaviorSanitizer: the library is rebuilt with the host code instrumented and tests/test_abi_host.py
runs against it in a child process.  No GPU is involved: device entry points return DETAG_EHIP there."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_abi_tests_are_clean_under_asan_and_ubsan():
    from paper_2006_08085_amd import build as B
    try:
        runtime = B.sanitizer_runtime()
    except RuntimeError as e:
        pytest.skip(str(e))
    lib = B.build(verbose=False, sanitize_host=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0"     # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["DETAG_LIB"] = lib
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi_host.py"), "-x", "-q", "-s",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "runtime error" not in tail and "AddressSanitizer" not in tail, tail
    assert " passed" in r.stdout
