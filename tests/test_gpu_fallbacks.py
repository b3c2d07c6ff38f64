"""The kernels that only special sizes reach (LDS-staged producers: byte offsets past 32 bits; fp32 matrix-op
contraction, single-pass 128-wide kernels and the direct-form kernels for arbitrary widths: kept for comparisons and
as the last resort; the separate feature- and parameter-gradient kernels of a full 64 -> 64 backward call; the planned pooling backward
kernel on clouds below the size it is chosen for) are selected here through the library's
environment switches, which are read once per process: so each setting runs the parity file once in a child process
(one at a time)."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.parametrize("env", [{"FLEX_PRODUCER": "staged"}, {"FLEX_CONTRACT": "f32"}, {"FLEX_SPLIT": "0"},
                                 {"FLEX_PAD": "0"}, {"FLEX_FUSED_BWD": "0"}, {"FLEX_POOL_PLAN": "1"}],
                         ids=["staged_producers", "fp32_contraction", "single_pass_128", "direct_form_kernels",
                              "separate_backward_kernels", "planned_pooling_at_every_size"])
def test_parity_file_under_switch(env):
    child_env = dict(os.environ)
    child_env.update(env)
    files = [os.path.join(HERE, "test_gpu_parity.py")]
    if "FLEX_PAD" in env:
        files.append(os.path.join(HERE, "test_gpu_bwd_pos.py"))     # its direct-form kernel is reached the same way
    if "FLEX_POOL_PLAN" in env:
        # the planned pooling kernel on the small and ragged clouds that it is otherwise not chosen for
        files = [os.path.join(HERE, "test_gpu_pool_plan.py")]
    r = subprocess.run([sys.executable, "-u", "-m", "pytest", *files, "-x", "-q",
                        "-m", "gpu", "--timeout", "120", "--timeout-method", "thread", "-p", "no:cacheprovider"],
                       capture_output=True, text=True, env=child_env, cwd=os.path.dirname(HERE), timeout=600)
    tail = "\n".join((r.stdout + r.stderr).splitlines()[-15:])
    assert r.returncode == 0, tail
    assert " passed" in r.stdout, tail
