"""The CPU checker built with AddressSanitizer and UndefinedBehaviorSanitizer, under the pins: a checker that
reads or writes one byte outside a buffer, or relies on undefined arithmetic, could still produce the right
bytes in the tests that compare against it; here it cannot pass.  (Host code only: no GPU is involved.)"""

import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
RUNNER = os.path.join(HERE, "pins_runner.py")


def sanitizer_runtime():
    p = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return p if os.path.isabs(p) and os.path.exists(p) else None


def test_pins_hold_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan = sanitizer_runtime()
    if not asan:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    out = str(tmp_path / "libdl_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    os.path.join(ROOT, "oracle", "dl_oracle.c"), "-o", out], check=True)
    # the interpreter is not instrumented: the runtime has to be loaded first, and its leak check would report
    # the interpreter's own allocations
    env = dict(os.environ, LD_PRELOAD=asan, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=23",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([sys.executable, RUNNER, out], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]


def test_the_sanitizers_do_catch_a_planted_overrun(tmp_path):
    """The same build with one planted mistake (the all-gather copies one byte too many into the last slot of
    each receive buffer): the run above must be able to fail."""
    asan = sanitizer_runtime()
    if not asan:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    text = open(os.path.join(ROOT, "oracle", "dl_oracle.c")).read()
    old = "memcpy((char *)out[r] + (size_t)j * B, in[j], B);"
    assert text.count(old) == 1
    src = tmp_path / "overrun.c"
    src.write_text(text.replace(old, "memcpy((char *)out[r] + (size_t)j * B, in[j], B + (j == W - 1));"))
    out = str(tmp_path / "libdl_oracle_overrun.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fsanitize=address,undefined", str(src), "-o", out],
                   check=True)
    env = dict(os.environ, LD_PRELOAD=asan, ASAN_OPTIONS="detect_leaks=0:exitcode=23")
    r = subprocess.run([sys.executable, RUNNER, out], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr
