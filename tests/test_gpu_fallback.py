"""The comparison switches TSM_IGEMM_RING=0 / TSM_WGRAD_TR=0 route the bf16 convolutions to the register-prefetch and
register-transposing kernels (the ones that otherwise serve channel counts that are not multiples of 64) and the
inference path to its unfused form.  The switches are read once per process, so a child process runs a few of the
parity tests under them."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_parity_holds_on_the_fallback_kernels():
    env = dict(os.environ, TSM_IGEMM_RING="0", TSM_WGRAD_TR="0")
    picks = ["tests/test_gpu_infer.py::test_infer_bf16_against_oracle",
             "tests/test_gpu_block.py::test_config1_bottleneck_reduced",
             "tests/test_gpu_block.py::test_bottleneck_projection_stride2",
             "tests/test_gpu_step.py::test_step_bf16_against_oracle_reduced_size"]
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-m", "gpu", "-p", "no:cacheprovider"] + picks,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
