"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer -- CPU only.

osc_ref.c is rebuilt with -fsanitize=address,undefined and every CPU test of the oracle runs again in
a child process against that build (the sanitizer runtimes are preloaded there, after whatever the
environment already preloads).  An out-of-bounds access, a misaligned or overflowing operation or a
bad shift anywhere in the oracle ends the child with a report."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    p = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return p if os.path.isabs(p) and os.path.exists(p) else None


def test_oracle_tests_pass_under_asan_and_ubsan():
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    if not asan or not ubsan:
        pytest.skip("gcc's sanitizer runtimes are not installed")
    env = dict(os.environ)
    env["OSC_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = " ".join(x for x in (env.get("LD_PRELOAD", ""), asan, ubsan) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    files = sorted(f for f in glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py"))
                   if not f.endswith("test_oracle_sanitized.py"))
    assert len(files) >= 8
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    out = p.stdout + p.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert p.returncode == 0, out[-4000:]
    assert " passed" in out
