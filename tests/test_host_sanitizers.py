"""The launcher's host code (argument checks, workspace carving, kernel selection: csrc/api.hip) under
AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU: the host-side ABI tests run again in a child
process against a build whose host code is instrumented.  No GPU is involved (every call in those tests
returns from the host checks before a launch)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_abi_host_checks_under_asan_and_ubsan():
    from paper_2509_18085_amd import build
    try:
        lib, rt = build.build_host_sanitized()
    except RuntimeError as e:
        pytest.skip("no sanitizer build: %s" % str(e)[:200])
    if not os.path.exists(rt):
        pytest.skip("no AddressSanitizer runtime to preload")
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join(x for x in (rt, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"          # the interpreter itself is not leak-clean
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["SPIFFY_LIB"] = lib
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_abi_host.py"),
                        os.path.join(ROOT, "tests", "test_zz_no_alloc.py") + "::test_static_head_limits_are_host_checks"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
