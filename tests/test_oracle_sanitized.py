"""The oracle's pin tests once more with the oracle built under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only): an out-of-bounds index or signed overflow in the plain
loops would otherwise go unnoticed as long as the numbers still came out right."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_under_asan_ubsan():
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    rt = oracle_build.sanitizer_preload()
    if rt is None:
        pytest.skip("this gcc ships no AddressSanitizer runtime")
    oracle_build.build(force=True, sanitize=True)
    env = dict(os.environ)
    env["MSD_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"   # the interpreter's own allocations are not the subject
    env["OMP_NUM_THREADS"] = "4"
    files = [os.path.join(ROOT, "tests", f) for f in ("test_oracle_int8.py", "test_oracle_mxfp4.py", "test_oracle_attn.py")]
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    assert " passed" in out
