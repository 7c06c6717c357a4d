"""Parity of the HIP temporal shift with the oracle: bit-exact in every layout and
storage type, including ragged channel counts, T = 1, fold_div = 0 and clip isolation."""
import numpy as np
import pytest
import torch

from oracle import tsm_oracle as O
from paper_1910_00932_amd import binding as B
from paper_1910_00932_amd import inputs as I
from gpu_util import CDT, CLAY, empty_act, from_dev, to_dev

pytestmark = pytest.mark.gpu

SHAPES = [  # N,T,C,H,W,fold_div
    (2, 8, 64, 14, 14, 8),      # configs[0]
    (2, 8, 256, 56, 56, 8),     # configs[1] shape at 2 clips
    (1, 8, 1024, 14, 14, 8),    # configs[4] shape at 1 clip
    (3, 5, 20, 7, 5, 8),        # fold 2: ragged everything
    (2, 1, 16, 3, 3, 4),        # T = 1
    (2, 4, 24, 4, 4, 0),        # no shift
    (1, 3, 7, 1, 3, 3),         # odd C
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("layout", ["nthwc", "ntchw"])
def test_shift_fwd_bwd_bit_exact(shape, dtype, layout):
    N, T, C, H, W, fd = shape
    x = I.normal((N, T, C, H, W), seed=0, dtype=dtype)
    xd = to_dev(x, dtype, layout)
    y = empty_act((N, T, C, H, W), dtype, layout)
    g = empty_act((N, T, C, H, W), dtype, layout)
    y.fill_(float("nan"))
    g.fill_(float("nan"))
    B.tsm_shift_fwd(xd, y, N, T, C, H, W, fd, CDT[dtype], CLAY[layout])
    B.tsm_shift_bwd(xd, g, N, T, C, H, W, fd, CDT[dtype], CLAY[layout])
    torch.cuda.synchronize()
    assert np.array_equal(from_dev(y, layout), O.shift(x.astype(np.float64), fd))
    assert np.array_equal(from_dev(g, layout), O.shift_adjoint(x.astype(np.float64), fd))


def test_shift_clip_isolation_on_device():
    N, T, C, H, W = 3, 4, 16, 4, 4
    x = I.normal((N, T, C, H, W), seed=1, dtype="bf16")
    x[1] = np.nan
    xd = to_dev(x, "bf16", "nthwc")
    y = empty_act((N, T, C, H, W), "bf16", "nthwc")
    B.tsm_shift_fwd(xd, y, N, T, C, H, W, 8, B.TSM_BF16, B.TSM_NTHWC)
    out = from_dev(y, "nthwc")
    assert np.isfinite(out[0]).all() and np.isfinite(out[2]).all()


def test_shift_full_size_sampled():
    """configs[1] tensor at full size [8,8,256,56,56] bf16, checked on sampled frames
    against the definition evaluated by the oracle on those clips."""
    N, T, C, H, W = 8, 8, 256, 56, 56
    x = I.normal((N, T, C, H, W), seed=0, dtype="bf16")
    xd = to_dev(x, "bf16", "nthwc")
    y = empty_act((N, T, C, H, W), "bf16", "nthwc")
    B.tsm_shift_fwd(xd, y, N, T, C, H, W, 8, B.TSM_BF16, B.TSM_NTHWC)
    out = from_dev(y, "nthwc")
    for n in (0, 3, 7):
        assert np.array_equal(out[n:n + 1], O.shift(x[n:n + 1].astype(np.float64), 8))
