"""The library's host side (lowering, hazard check, mode table, argument checks) under AddressSanitizer and
UndefinedBehaviorSanitizer: the library is built once more with its HOST pass instrumented (the device code is
untouched and never runs here) and the host-logic tests run against that build in a process of their own."""

import glob
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
sys.path.insert(0, ROOT)


def clang_asan_runtime(hipcc):
    rocm = os.path.dirname(os.path.dirname(os.path.abspath(hipcc)))
    found = sorted(glob.glob(os.path.join(rocm, "lib", "llvm", "lib", "clang", "*", "lib", "linux", "libclang_rt.asan-x86_64.so")))
    return found[-1] if found else None


def test_host_logic_under_sanitizers(tmp_path):
    from paper_2511_06605_amd import build as dl_build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    runtime = clang_asan_runtime(hipcc)
    if not runtime:
        pytest.skip("this ROCm installation has no AddressSanitizer runtime for the host")
    lib = tmp_path / "libdmalatte.so"
    flags = [f for f in dl_build.HIPCC_FLAGS if f != "-O3"]
    cmd = [hipcc, *flags, "-O1", "-g", "-fno-omit-frame-pointer",
           # sanitizers for the host pass only
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-shared-libsan",
           *[os.path.join(dl_build.CSRC, s) for s in dl_build.SOURCES], "-o", str(lib)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, LD_PRELOAD=runtime, DL_LIBRARY=str(lib),
               ASAN_OPTIONS="detect_leaks=0:exitcode=23", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(HERE, "test_host_logic.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, timeout=600, cwd=ROOT)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert " passed" in r.stdout
