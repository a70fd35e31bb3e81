"""The oracle's pins once more, against a build of oracle/dmath_oracle.c with AddressSanitizer and
UndefinedBehaviorSanitizer (host code only): an out-of-bounds read of a padded operand, a signed
overflow in an index or a misaligned access in the oracle would otherwise only show up as a wrong
reference value, or not at all.  Runs the pins in a child interpreter that preloads the sanitizer
runtime; CPU only."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers():
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    oracle_build.build(force=False, sanitize=True)
    env = dict(os.environ)
    preload = [oracle_build.sanitizer_runtime()] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
    env["LD_PRELOAD"] = ":".join(preload)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["DMATH_ORACLE_SANITIZE"] = "1"
    env["OMP_NUM_THREADS"] = env.get("OMP_NUM_THREADS", "8")
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=1500)
    tail = res.stdout[-3000:]
    assert res.returncode == 0, tail
    assert "AddressSanitizer" not in res.stdout and "runtime error" not in res.stdout, tail
    assert " passed" in res.stdout, tail
