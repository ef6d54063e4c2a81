"""The persistent ("streaming") kernels against the oracle on short vectors: the
cases of streaming_cases.py in a process whose environment makes every eligible
call take the persistent kernels on a twelve-wave grid (the library reads the two
variables once per process, so they cannot be changed inside this one)."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))


def test_streaming_kernels_match_oracle_on_short_vectors():
    env = dict(os.environ, NDQ_STREAM_MIN_TILES_PER_WAVE="0", NDQ_STREAM_MAX_BLOCKS="3")
    res = subprocess.run([sys.executable, "-u", os.path.join(HERE, "streaming_cases.py")], env=env,
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = "\n".join(res.stdout.splitlines()[-15:])
    assert res.returncode == 0, tail
    assert "STREAMING_CASES_OK" in res.stdout, tail
