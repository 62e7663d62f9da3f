"""The oracle is the checker, so it is checked too: the pins of test_oracle_pins.py run once more against
a build of oracle/sparq_oracle.c with AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no
GPU involved).  An out-of-bounds access, a use after free, signed overflow or a misaligned access in the
oracle aborts the child process and fails this test."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_under_address_and_ub_sanitizers():
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("gcc has no libasan here")
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    oracle_build.build(force=True, sanitize=True)
    env = dict(os.environ)
    env["SPARQ_ORACLE_SANITIZED"] = "1"
    env["LD_PRELOAD"] = libasan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # python itself is not instrumented: its own allocations are not this test's business
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
