"""The launch-shape overrides (SIRLLM_TUNE=1 plus SIRLLM_SCORE_*, SIRLLM_GATHER_*, SIRLLM_INPLACE_*, SIRLLM_FUSE_SELECT, SIRLLM_LMHEAD_WIDE)
are part of the library: a sweep must be able to trust every setting.  The switch is read at the library's first
launch in a process, so the matrix runs in a child process (tests/tuning_child.py), which checks each setting
against the oracle."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_launch_shape_override_matches_the_oracle():
    env = dict(os.environ, SIRLLM_TUNE="1")
    r = subprocess.run([sys.executable, "-u", os.path.join(ROOT, "tests", "tuning_child.py")], env=env,
                       capture_output=True, text=True, timeout=560)
    tail = "\n".join((r.stdout + "\n" + r.stderr).splitlines()[-15:])
    assert r.returncode == 0, tail
    assert "ALL OK" in r.stdout, tail
