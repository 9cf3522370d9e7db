"""The oracle's pins once more with the C code built under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only; no GPU): an out-of-bounds index, a use after free or
signed overflow in the oracle would pass the numeric pins unnoticed and still taint every parity
claim that rests on it."""
import os
import subprocess
import sys

import pytest

from oracle import mosaic_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    rt = orc.sanitizer_runtime()
    if rt is None:
        pytest.skip("gcc's libasan.so is not installed")
    orc.build(force=True, sanitize=True)
    env = dict(os.environ)
    env["MOSAIC_ORACLE_SANITIZED"] = "1"
    # the sanitizer runtime has to be in the process before the sanitized library is loaded; whatever
    # is preloaded already stays in place
    env["LD_PRELOAD"] = " ".join(x for x in (rt, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_cache_model_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (p.stdout + p.stderr)[-3000:]
    assert p.returncode == 0, tail
    assert "passed" in p.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
