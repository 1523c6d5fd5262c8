"""The host-only native code of the test infrastructure (the CPU oracle and the input generators) built with
AddressSanitizer + UndefinedBehaviorSanitizer, and the oracle's own pin tests run against those builds in a
child process that has the sanitizer runtime preloaded.  A heap overflow, a use after free, a signed overflow
or a misaligned access in that code fails this test."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_generators_are_clean_under_asan_and_ubsan():
    import oracle
    import synth
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no AddressSanitizer runtime on this machine")
    env = dict(os.environ)
    env["DCI_ORACLE_LIB"] = oracle.build_sanitized()
    env["DCI_SYNTH_LIB"] = synth.build_sanitized()
    # the runtime must come first in the preload list; whatever is already preloaded stays
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # CPython's own allocations are not of interest; leak checking would report interpreter noise
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    tests = ["tests/test_oracle_rng_sampler.py", "tests/test_oracle_counts_fill.py", "tests/test_oracle_sage.py",
             "tests/test_synth_inputs.py"]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + tests, cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    assert " passed" in out
