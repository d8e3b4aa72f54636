"""The one-wave-per-tile STACK / SCORE kernels at d = 128 and d = 256 stay in the library as the fallback
of the two-waves-per-tile kernels (wider query sets, LDS limits) and as their comparison.  With
LONGER_DISABLE_PAIR_KERNELS=1 every launch uses them; the switch is read once per process, so the parity
cases that exercise those shapes run once more in ONE child process with it set."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CASES = ("test_c3_bf16_all_entry_points or test_c5_bf16_serving or test_bf16_other_head_widths "
         "or test_bf16_d256_forward_entry_points or test_parameters_packed_once_equal_packing_per_call")


@pytest.mark.gpu
def test_parity_with_the_pair_kernels_switched_off():
    env = dict(os.environ, LONGER_DISABLE_PAIR_KERNELS="1")
    r = subprocess.run([sys.executable, "-u", "-m", "pytest", os.path.join(ROOT, "tests", "test_gpu_parity.py"),
                        "-x", "-q", "-m", "gpu", "-k", CASES, "--timeout", "300", "--timeout-method", "thread",
                        "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = "\n".join(r.stdout.splitlines()[-25:])
    assert r.returncode == 0, tail
    assert " passed" in tail and "failed" not in tail, tail
