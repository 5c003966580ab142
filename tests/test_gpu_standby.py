"""Standby mode on the GPU: the checks of standby_runner.py, in a process of their own (that file says why), once
as the library runs by default and once with DL_NO_BAR=1: doorbells, records and tables in host memory, the
placement for devices whose memory the host cannot write directly."""

import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.parametrize("no_bar", ["0", "1"])
def test_standby_mode_in_a_process_of_its_own(no_bar):
    env = dict(os.environ, DL_NO_BAR=no_bar)
    p = subprocess.run([sys.executable, "-u", os.path.join(HERE, "standby_runner.py")], stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=100, env=env)
    print(p.stdout)
    assert p.returncode == 0, p.stdout[-4000:]
    assert "standby: all ok" in p.stdout
