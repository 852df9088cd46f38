"""The oracle's pins once more against a build of the same C source with AddressSanitizer and
UndefinedBehaviorSanitizer: an out-of-bounds access, a use of uninitialised stack, a signed overflow or a
misaligned load in the checker would make its agreement with the pins worth less.  Runs in a child process
(the sanitizer runtime has to be loaded before anything else).  No GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_pass_under_address_and_ub_sanitizers():
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("the AddressSanitizer runtime (libasan.so) is not installed next to gcc")
    sys.path.insert(0, ROOT)
    import oracle
    try:
        san = oracle.build_sanitized()
    except subprocess.CalledProcessError as e:
        pytest.skip("gcc cannot build with -fsanitize=address,undefined here: %s" % e)
    env = dict(os.environ)
    env["USL_ORACLE_LIB"] = san
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # Python itself is not instrumented: its allocations at exit are not leaks of the oracle
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    p = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (p.stdout + p.stderr)[-3000:]
    assert p.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert " passed" in p.stdout
