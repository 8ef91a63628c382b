"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer: the pins of the quantizers, of Algorithm 1 and of
the half-INT8 variant run against a sanitized build of oracle/intfa_oracle.c in a child process (the sanitizer
runtime must be the first library of the process, so it cannot be loaded into this one).  Any report aborts the child."""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(900)
def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no AddressSanitizer runtime next to gcc")
    lib = oracle.build_sanitized()
    env = dict(os.environ)
    env["INTFA_ORACLE_LIB"] = lib
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")   # in front of what is there
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"       # the interpreter's own leaks are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    files = ["tests/test_oracle_quantize.py", "tests/test_oracle_attention.py", "tests/test_oracle_half.py"]
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=850)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
