"""Standby mode on the GPU: the checks of standby_runner.py, in a process of their own (that file says why)."""

import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))


def test_standby_mode_in_a_process_of_its_own():
    p = subprocess.run([sys.executable, "-u", os.path.join(HERE, "standby_runner.py")], stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=100)
    print(p.stdout)
    assert p.returncode == 0, p.stdout[-4000:]
    assert "standby: all ok" in p.stdout
