"""The oracle's pins once more, against a build of both oracle sources with AddressSanitizer and
UndefinedBehaviorSanitizer (gcc, host code only): an out-of-bounds read, a shift past the word
size, a signed overflow or a misaligned access inside the checker itself would otherwise go
unnoticed as long as the numbers happen to come out right.  The pins run in a child process whose
dynamic loader brings the sanitizer runtime in first; any report makes that process fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_group_oracle_pins.py", "tests/test_f16_oracle_pins.py",
             "tests/test_repack_oracle_pins.py", "tests/test_quant_oracle_pins.py"]


def test_pins_pass_on_the_sanitised_oracle_build():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not asan or not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    env = dict(os.environ)
    env["ANY4_ORACLE_SANITIZE"] = "1"
    # the sanitizer runtime first, whatever was preloaded already after it
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # (leak checking off: the interpreter itself never frees everything; link order not verified
    # because other preloaded libraries may precede the runtime in the loader's list)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    for lib in ("libany4_oracle_san.so", "libany4_quant_oracle_san.so"):      # always a fresh build
        p = os.path.join(ROOT, "oracle", lib)
        if os.path.exists(p):
            os.remove(p)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
    for lib in ("libany4_oracle_san.so", "libany4_quant_oracle_san.so"):
        assert os.path.exists(os.path.join(ROOT, "oracle", lib)), "the sanitised build was not the one loaded"
