"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle's pins (tests/test_oracle_*.py)
are run once more in a child process that loads a sanitized build of oracle/isd_oracle.c (-O1, -fsanitize=address,
undefined).  An out-of-bounds access, a use after free, a signed overflow or a misaligned access anywhere in the
oracle ends the child with a report.  CPU only: nothing here touches a GPU or the HIP library."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _libasan():
    try:
        path = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    except (OSError, subprocess.CalledProcessError):
        return None
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.mark.skipif(os.environ.get("ISD_ORACLE_SANITIZE", "") not in ("", "0"), reason="already the sanitized child")
def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    asan = _libasan()
    if asan is None:
        pytest.skip("gcc's libasan.so is not installed")
    env = dict(os.environ)
    env["ISD_ORACLE_SANITIZE"] = "1"
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter and numpy are not built for leak checking; errors abort instead of being printed and ignored
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    pins = sorted(p for p in glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py"))
                  if not p.endswith("test_oracle_sanitized.py"))
    assert len(pins) >= 8
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu", *pins],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout[-3000:] + "\n" + res.stderr[-3000:])
    assert "AddressSanitizer" not in res.stderr and "runtime error:" not in res.stderr, tail
    assert res.returncode == 0, tail
    assert " passed" in res.stdout, tail
