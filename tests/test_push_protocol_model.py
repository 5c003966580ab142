"""The order in which a kernel must read a copy table that the host wrote straight into device memory (table,
fence, stamp), checked on a host-thread model of writer and reader: tests/models/push_protocol_model.cpp.

The model is not the device code; it pins the reasoning that the device code follows (dl_pushed_sealed, then the
entry loads): only what is read after the stamp was seen is vouched for by it.  The opposite order, which an
earlier version of the kernels used, pairs a new stamp with the slot's previous table under a forced
interleaving; the order in use never does, forced or free-running (also under ThreadSanitizer where the
compiler has it)."""

import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "models", "push_protocol_model.cpp")


def build(tmp_path, flags):
    exe = tmp_path / "push_protocol_model"
    subprocess.run(["g++", "-O2", "-std=c++17", "-pthread", *flags, SRC, "-o", str(exe)], check=True)
    return str(exe)


def test_stamp_first_never_pairs_a_stamp_with_older_payload(tmp_path):
    exe = build(tmp_path, [])
    r = subprocess.run([exe, "stamp_first"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    assert "STALE" not in r.stdout and "0 stale pairings" in r.stdout


def test_payload_first_is_caught_by_the_forced_interleaving(tmp_path):
    """The planted mistake: the model must be able to tell the two orders apart."""
    exe = build(tmp_path, [])
    r = subprocess.run([exe, "payload_first"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 1, r.stdout
    assert "forced: stamp 2 payload 1  STALE" in r.stdout


def test_stamp_first_is_clean_under_thread_sanitizer(tmp_path):
    try:
        exe = build(tmp_path, ["-fsanitize=thread", "-g"])
    except subprocess.CalledProcessError:
        pytest.skip("this compiler has no ThreadSanitizer runtime")
    r = subprocess.run([exe, "stamp_first"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "WARNING: ThreadSanitizer" not in r.stderr, r.stdout + r.stderr
