"""The C oracle under AddressSanitizer + UndefinedBehaviorSanitizer: every pin of
tests/test_oracle_pins.py is run again, in a child process, against a build of the same
source in which a shift by a bad amount, a signed overflow, a misaligned or out-of-bounds
access aborts the process instead of passing silently (the bug class of rounding-shift code)."""
import os
import subprocess
import sys

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_pass_on_the_sanitizer_build_of_the_oracle():
    lib = oracle_build.build_sanitized()
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    env = dict(os.environ)
    # the sanitizer runtime has to come first among the preloaded libraries of the child
    env["LD_PRELOAD"] = ":".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"       # python itself never frees everything
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["F8REF_LIB"] = lib
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                          "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True,
                         timeout=1500)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "runtime error" not in tail and "AddressSanitizer" not in tail, tail
