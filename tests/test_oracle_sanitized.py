"""The oracle pins once more against a build of oracle/lx_oracle.cpp with AddressSanitizer and
UndefinedBehaviorSanitizer (host code on the CPU; never on a GPU machine): an out-of-bounds index, a
read of uninitialised stack, signed overflow or a misaligned access in the oracle aborts the run.
The pins run in a child process because the sanitizer runtime has to be loaded before Python."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_under_address_and_ub_sanitizers():
    from oracle import build
    try:
        build.build_sanitized(force=False)
        asan = build.asan_runtime()
    except (subprocess.CalledProcessError, OSError) as e:      # no sanitizer runtime on this machine
        pytest.skip(f"sanitized oracle build not available: {e}")
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("libasan.so not found")
    env = dict(os.environ)
    # the sanitizer runtime goes first; whatever is preloaded already stays behind it
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"   # the interpreter's own leaks are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["LX_ORACLE_SANITIZED"] = "1"
    files = sorted(os.path.join(ROOT, "tests", f) for f in os.listdir(os.path.join(ROOT, "tests"))
                   if f.startswith("test_oracle_") and f != os.path.basename(__file__))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                        *files], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "failed" not in r.stdout, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
