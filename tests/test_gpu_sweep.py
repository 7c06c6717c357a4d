"""Seeded random shapes through the convolution and block entry points (bf16 MFMA path, channels innermost):
ragged pixel counts, channel counts that are and are not multiples of the 64-channel K step, strides, shift
proportions, single-frame clips.  Every result is compared with the oracle as in the fixed-shape tests."""
import numpy as np
import pytest

import test_gpu_block as TB
import test_gpu_conv as TC

pytestmark = pytest.mark.gpu


def _conv_cases(seed, n):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        k = int(rng.choice([1, 3]))
        s = int(rng.choice([1, 2]))
        Cin = int(rng.choice([64, 128, 192, 256, 320, 72]))
        Cout = int(rng.choice([64, 128, 256, 40, 192, 384]))
        H, W = int(rng.integers(3, 20)), int(rng.integers(3, 20))
        N, T = int(rng.integers(1, 4)), int(rng.integers(1, 6))
        fd = int(rng.choice([0, 8, 4])) if k == 1 else int(rng.choice([0, 8]))
        out.append((N, T, Cin, H, W, Cout, k, s, 1 if k == 3 else 0, fd))
    return out


def _block_cases(seed, n):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        Cmid = int(rng.choice([64, 128, 192]))
        proj = bool(rng.integers(0, 2))
        stride = int(rng.choice([1, 2])) if proj else 1
        Cin = int(rng.choice([Cmid, 2 * Cmid, 4 * Cmid])) if proj else 4 * Cmid
        H, W = int(rng.integers(4, 15)), int(rng.integers(4, 15))
        N, T = int(rng.integers(1, 3)), int(rng.integers(1, 5))
        out.append((N, T, Cin, H, W, Cmid, 4 * Cmid, stride, proj, int(rng.choice([8, 4, 0]))))
    return out


@pytest.mark.parametrize("case", _conv_cases(11, 16))
def test_random_conv_shapes(case):
    TC._run(case, "bf16", "nthwc")


@pytest.mark.parametrize("case", _block_cases(12, 6))
def test_random_bottleneck_shapes(case):
    N, T, Cin, H, W, Cmid, Cout, stride, proj, fd = case
    TB.run_block("bottleneck", N, T, Cin, H, W, Cmid, Cout, stride, proj, fd, "bf16", "nthwc")
