"""GPU: the decode tests once more with each of the two decode kernels forced for every launch (the library's own
choice mixes them: the matrix-core kernel for short key ranges and large query groups, the vector kernel elsewhere,
so neither sees every shape of the other tests).  A child pytest per kernel, one at a time; the child's contexts take
the kernel from LT_DECODE_PATH."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FILES = ["tests/test_gpu_decode.py", "tests/test_gpu_ragged.py", "tests/test_gpu_online.py", "tests/test_gpu_graph.py",
         "tests/test_gpu_random.py", "tests/test_gpu_guards.py", "tests/test_gpu_paged.py"]


@pytest.mark.parametrize("path", ["matrix", "vector"])
def test_decode_tests_with_one_kernel_forced(path):
    env = dict(os.environ)
    env["LT_DECODE_PATH"] = path
    print("decode tests on the", path, "kernel", flush=True)
    run = subprocess.run([sys.executable, "-u", "-m", "pytest", "-q", "-x", "-m", "gpu", "-p", "no:cacheprovider", "--timeout", "300",
                          "--timeout-method", "thread"] + FILES, cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    report = run.stdout + run.stderr
    assert run.returncode == 0, report[-6000:]
    assert " passed" in report and " failed" not in report, report[-3000:]
