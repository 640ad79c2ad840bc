"""The host code of both sides under AddressSanitizer + UndefinedBehaviorSanitizer.

A second copy of the library (host code of the entry points and of the offline / CPU-side routines
instrumented; device code untouched) and of the C oracle is built with the same clang, and the CPU
test files that drive them are run again in a child interpreter that loads those copies.  Any
report of either sanitizer fails the child (UBSan reports do not recover; ASan aborts)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FILES = ["test_oracle_select.py", "test_oracle_select_equalized.py", "test_oracle_attend.py",
         "test_oracle_index.py", "test_oracle_pool.py", "test_oracle_skew.py", "test_host_library.py",
         "test_host_speculation.py"]


@pytest.mark.skipif(os.environ.get("IG_LIBRARY"), reason="already inside the sanitized run")
def test_cpu_suite_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2406_19707_amd import build as hip_build
    from oracle import ig_oracle
    out = os.path.join(ROOT, "paper_2406_19707_amd", "_build", "san")
    lib = hip_build.build_host_sanitized(out)
    rt = hip_build.sanitizer_runtime()
    clang = os.path.join(os.path.dirname(hip_build.HIPCC), "amdclang")
    olib = ig_oracle.build_sanitized(out, clang)
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join([rt] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else []))
    # the interpreter itself is not instrumented: its own allocations at exit are not the subject
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["IG_LIBRARY"], env["IG_ORACLE_LIBRARY"] = lib, olib
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
           *[os.path.join(ROOT, "tests", f) for f in FILES]]
    r = subprocess.run(cmd, env=env, cwd=ROOT, capture_output=True, text=True, timeout=1500)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, tail
    assert " passed" in r.stdout
