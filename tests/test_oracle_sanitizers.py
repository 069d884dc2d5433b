"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): its pins run once more in a child
process against a sanitizer build of the same source; any report ends that process with an error."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_asan_and_ubsan():
    from oracle.build_oracle import asan_runtime, build_sanitized
    try:
        lib = build_sanitized()
        rt = asan_runtime()
    except (OSError, subprocess.CalledProcessError) as e:
        pytest.skip(f"no sanitizer toolchain: {e}")
    if not os.path.isabs(rt) or not os.path.exists(rt):
        pytest.skip("the compiler ships no AddressSanitizer runtime")
    env = dict(os.environ)
    env["DYNORACLE_LIB"] = lib
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"      # the interpreter's own allocations are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
