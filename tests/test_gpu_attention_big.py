"""The attention parity cases again with the large-launch matrix-core kernel pinned (64 query rows
per wave); on its own it is only chosen for launches with hundreds of row tiles, which the
oracle cannot follow.  Runs the cases in a child process because the choice is read once per
process from the environment."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_attention_cases_with_large_launch_kernel():
    env = dict(os.environ, KVS_ATTN_VARIANT="big")
    cmd = [sys.executable, "-u", "-m", "pytest", "-x", "-q", "-m", "gpu", "--timeout", "120",
           "--timeout-method", "thread", "-k", "attention or end_to_end",
           os.path.join(ROOT, "tests", "test_gpu_parity.py")]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    print(r.stdout[-3000:])
    print(r.stderr[-2000:], file=sys.stderr)
    assert r.returncode == 0, "attention parity failed with KVS_ATTN_VARIANT=big"
    assert " passed" in r.stdout
