"""The protocol of the withdrawn executor that served many requests from one launch (leader workgroup, worker
workgroups, command ring, arrival count), as a host-thread model: tests/models/resident_protocol_model.cpp.
Nothing of that executor is in the library and nothing of it runs on a GPU; the model exists to say whether the
protocol itself holds a race, a deadlock or an index out of range.  It does not: thousands of requests complete
with every tile written exactly once under perturbed schedules, both ways of leaving (quit flag, no doorbell
for too long) end every thread, ThreadSanitizer and AddressSanitizer have nothing to report, and a planted
ordering mistake is caught."""

import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "models", "resident_protocol_model.cpp")


def build(tmp_path, flags, name):
    exe = tmp_path / name
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-pthread", "-Wall", "-Wextra", *flags, SRC, "-o", str(exe)], check=True)
    return str(exe)


@pytest.mark.parametrize("workgroups,seed", [(2, 1), (6, 2), (13, 3)])
def test_protocol_as_built_completes_every_request_and_every_thread_leaves(tmp_path, workgroups, seed):
    exe = build(tmp_path, [], "resident_model")
    r = subprocess.run([exe, "as_built", "3000", str(workgroups), str(seed)], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout
    assert "quit: 3000 of 3000 requests complete and correct, end state 2" in r.stdout
    assert "idle: 751 of 751 requests complete and correct, end state 3" in r.stdout


def test_late_clear_of_the_arrival_counter_is_caught(tmp_path):
    """The planted mistake: arrivals for the next command are wiped out, the leader's bounded wait gives up."""
    exe = build(tmp_path, [], "resident_model")
    r = subprocess.run([exe, "reset_late", "3000", "6", "1"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 1 and "never completed: executor state 4" in r.stdout, r.stdout


def test_protocol_as_built_is_clean_under_thread_sanitizer(tmp_path):
    try:
        exe = build(tmp_path, ["-fsanitize=thread"], "resident_model_tsan")
    except subprocess.CalledProcessError:
        pytest.skip("this compiler has no ThreadSanitizer runtime")
    r = subprocess.run([exe, "as_built", "1500", "6", "5"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "WARNING: ThreadSanitizer" not in r.stderr, r.stdout + r.stderr


def test_protocol_as_built_is_clean_under_address_sanitizer(tmp_path):
    try:
        exe = build(tmp_path, ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"], "resident_model_asan")
    except subprocess.CalledProcessError:
        pytest.skip("this compiler has no AddressSanitizer runtime")
    r = subprocess.run([exe, "as_built", "3000", "8", "4"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stdout + r.stderr
