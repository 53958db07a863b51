"""The oracle's pins once more, against a build of the oracle with AddressSanitizer and
UndefinedBehaviorSanitizer (host code only; nothing here touches a GPU): an out-of-bounds
index, a use after free or signed overflow in the oracle would pass silently otherwise."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_score.py", "tests/test_oracle_window.py", "tests/test_oracle_missing.py",
        "tests/test_oracle_severity.py", "tests/test_oracle_sweep.py", "tests/test_oracle_ledger.py"]


def _runtime(name):
    out = subprocess.run(["g++", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


@pytest.mark.skipif(os.environ.get("GUARD_ORACLE_SANITIZE") == "1", reason="already inside the sanitized run")
def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers():
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("no AddressSanitizer runtime beside g++")
    env = dict(os.environ)
    env["GUARD_ORACLE_SANITIZE"] = "1"
    # the interpreter itself is not instrumented, so the runtime is preloaded (behind
    # whatever is preloaded already) and leak checking, which would list CPython's own
    # allocations, is off
    env["LD_PRELOAD"] = ":".join(x for x in (env.get("LD_PRELOAD", ""), asan) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = env.get("OMP_NUM_THREADS", "8")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *PINS],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
