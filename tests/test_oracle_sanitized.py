"""Opt-in: every CPU pin of the oracle once more, with the oracle built under AddressSanitizer and
UndefinedBehaviorSanitizer (an out-of-bounds read in the checker would make every parity claim worthless).
Off by default because it takes a minute: YGG_ORACLE_SANITIZE=1 python -m pytest tests/test_oracle_sanitized.py
"""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(os.environ.get("YGG_ORACLE_SANITIZE") != "1", reason="opt-in: set YGG_ORACLE_SANITIZE=1")
def test_oracle_pins_pass_under_asan_and_ubsan():
    sys.path.insert(0, ROOT)
    import oracle

    lib = oracle.build_sanitized()
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    env = dict(os.environ, YGG_ORACLE_LIB=lib, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               LD_PRELOAD=":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x))
    del env["YGG_ORACLE_SANITIZE"]   # the child must not start this test again
    files = sorted(f for f in glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")) if not f.endswith("_sanitized.py"))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-4000:]
    assert " passed" in r.stdout
