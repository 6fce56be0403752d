"""The oracle's C source under AddressSanitizer and UndefinedBehaviorSanitizer.

The pins of test_oracle_pins.py say that the oracle computes the right values;
this says that it does so without reading or writing out of bounds, overflowing
a signed integer, shifting too far or misaligning an access, on all the shapes
the pins use (empty batches, ragged tails, duplicate rows, n_kept = 0, ...).
Host code only: the sanitizer build is a CPU library, loaded by a child
interpreter that has the ASan runtime preloaded.
"""
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    lib = oracle.build_sanitized(str(tmp_path / "libss_oracle_san.so"))
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True,
                          capture_output=True, text=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), asan
    env = dict(os.environ)
    # the ASan runtime has to come first; whatever is preloaded already stays
    env["LD_PRELOAD"] = ":".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["SS_ORACLE_LIB"] = lib
    run = subprocess.run(
        [sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
         "-x", "-q", "-p", "no:cacheprovider"],
        cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert " passed" in run.stdout and "failed" not in run.stdout, tail
    assert "runtime error" not in tail and "AddressSanitizer" not in tail, tail
