"""The oracle's pins once more, against a build of the oracle with AddressSanitizer and
UndefinedBehaviorSanitizer (gcc, -O1): an out-of-bounds access, a use after free, a signed overflow
or a misaligned access anywhere in the code the pins reach aborts the child process.  CPU only."""
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_pass_under_address_and_ub_sanitizers():
    oracle.build(sanitize=True)
    env = dict(os.environ)
    env["PKV_ORACLE_SANITIZE"] = "1"
    pre = [oracle.sanitizer_runtime()] + [x for x in env.get("LD_PRELOAD", "").split(":") if x]
    env["LD_PRELOAD"] = ":".join(pre)
    # the interpreter itself is not instrumented: leak reports would be its own arenas
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "libprefixkv_oracle_san.so" not in tail or "ERROR" not in tail, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
