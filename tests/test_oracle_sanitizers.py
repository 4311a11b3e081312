"""The oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU involved) must pass
every pin without a report: an out-of-bounds read in the yardstick could otherwise hide behind plausible numbers."""
import os
import subprocess
import sys

import pytest

from oracle import sig_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_oracle_backward_pins.py", "tests/test_oracle_log_pins.py"]


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("this gcc ships no libasan.so")
    lib = orc.compile_copy(str(tmp_path / "libsig_oracle_sanitized.so"),
                           extra=["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                                  "-fno-omit-frame-pointer"])
    env = dict(os.environ)
    env["SIG_ORACLE_LIB"] = lib
    # the sanitizer runtime has to be in the interpreter's initial library list; whatever is preloaded already stays
    env["LD_PRELOAD"] = " ".join(p for p in (asan, env.get("LD_PRELOAD", "")) if p)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:halt_on_error=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider", *PIN_FILES],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert " passed" in res.stdout
