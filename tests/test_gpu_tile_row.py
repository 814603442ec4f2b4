"""The alternative GEMM tile (128 x 256 x 32, two workgroups per CU; MOE_GEMM_TILE=0 in the environment) is kept
to the same parity bar: the grouped-FFN, whole-layer and random-shape parity tests run once more in a child process that
selects it (the library reads the variable once per process)."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_parity_with_the_two_workgroup_tile():
    env = dict(os.environ, MOE_GEMM_TILE="0")
    cmd = [sys.executable, "-u", "-m", "pytest", "-x", "-q", "-m", "gpu", "--timeout", "170", "--timeout-method", "thread",
           "tests/test_gpu_parity.py", "tests/test_gpu_gather.py", "tests/test_gpu_random_shapes.py", "-k",
           "grouped_ffn or gather_ffn or end_to_end or long_experts or ep_share or dense_swiglu or random_shape"]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = "\n".join((res.stdout + res.stderr).splitlines()[-15:])
    print(tail, flush=True, file=sys.stderr)
    assert res.returncode == 0, tail
    assert " passed" in res.stdout
