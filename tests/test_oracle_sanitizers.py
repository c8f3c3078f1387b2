"""The CPU checker under AddressSanitizer and UndefinedBehaviorSanitizer: its pins (the tests of
tests/test_oracle_*.py that need no GPU) are run once more in a child process that loads the
instrumented build of es_oracle.c, with the sanitizer runtime preloaded.  Any out-of-bounds access,
use after free, signed overflow or misaligned access in the checker aborts the child."""
import os
import subprocess
import sys
from pathlib import Path

import oracle

ROOT = Path(__file__).resolve().parent.parent
PINS = ["tests/test_oracle_noise.py", "tests/test_oracle_rollout.py", "tests/test_oracle_update.py",
        "tests/test_oracle_siblings.py"]


def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers():
    oracle.build(sanitize=True)
    env = dict(os.environ)
    env["ORACLE_SANITIZE"] = "1"
    # the runtime goes in front of whatever is preloaded already; the interpreter itself is not instrumented,
    # so leak checking (which would list the interpreter's own allocations) is off
    env["LD_PRELOAD"] = " ".join(x for x in (oracle.sanitizer_runtime(), env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "2"
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS],
                         cwd=str(ROOT), env=env, capture_output=True, text=True, timeout=900)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert " passed" in run.stdout and "runtime error" not in tail and "AddressSanitizer" not in tail, tail
