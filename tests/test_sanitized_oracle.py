"""Sanitizer leg of the CPU suite: the oracle's C code is rebuilt with gcc's UndefinedBehaviorSanitizer and,
where the interpreter can take a preloaded runtime, AddressSanitizer, and the oracle's own tests run against
that build in a child interpreter.  Any report (out-of-bounds access, use after free, signed overflow,
misaligned access, invalid shift, ...) ends the child with a failure."""
import glob
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
FILES = sorted(glob.glob(os.path.join(HERE, "test_oracle_*.py")))


def _run(sanitize, preload=None):
    env = dict(os.environ)
    env["ADASD_ORACLE_SANITIZE"] = sanitize
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["ASAN_OPTIONS"] = "detect_leaks=0"          # the interpreter itself is not instrumented
    if preload:
        env["LD_PRELOAD"] = preload
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + FILES,
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=1500)
    tail = r.stdout[-4000:]
    assert r.returncode == 0, tail
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout, tail
    assert " passed" in r.stdout, tail


def test_oracle_tests_under_ubsan():
    assert FILES
    _run("undefined")


def test_oracle_tests_under_asan_and_ubsan():
    preloads = os.environ.get("LD_PRELOAD", "")
    if os.path.exists("/etc/ld.so.preload") and open("/etc/ld.so.preload").read().strip():
        preloads += " (ld.so.preload)"
    if preloads:
        pytest.skip("this environment preloads libraries of its own; AddressSanitizer's runtime has to come first "
                    "in the interpreter and is not forced in front of them")
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    _run("address,undefined", preload=os.path.realpath(libasan))
