"""The comparator the GPU parity tests use (gpu_util.compare_local / compare_act), on the CPU: planted errors that
one relative L2 norm over the whole tensor does not see -- a wrong tile edge, a wrong clip-end frame, a wrong ragged
last tile, single wrong elements -- must fail it; rounding-sized differences must pass."""
import numpy as np
import pytest

import gpu_util as G


def _pair(shape=(4, 8, 64, 27, 27), seed=0, noise=2e-3):
    rng = np.random.default_rng(seed)
    b = rng.standard_normal(shape)
    a = b * (1 + noise * rng.standard_normal(shape))
    return a, b


def test_rounding_sized_differences_pass():
    a, b = _pair()
    out = G.compare_act(a, b, 2e-2, "clean", "bf16", rtol=2.0 ** -6, atol_rel=2.0 ** -6)
    assert out["l2"] < 3e-3 and out["tile_max"] < 4e-3 and out["elem_outliers"] == 0


@pytest.mark.parametrize("plant", ["tile_edge_row", "clip_end_frame_group", "ragged_last_tile", "single_elements"])
def test_localised_errors_fail_although_the_whole_tensor_norm_passes(plant):
    a, b = _pair()
    N, T, C, H, W = a.shape
    if plant == "tile_edge_row":            # the last pixel row of one 256-row tile, all channels
        rows = G.act_rows(a)
        rows[255 + 256 * 7] = 0.0
        a = rows.reshape(N, T, H, W, C).transpose(0, 1, 4, 2, 3)
    elif plant == "clip_end_frame_group":   # the shifted channel group of the last frame of one clip left unzeroed
        a[2, T - 1, :8] += 0.3 * b[3, 0, :8]
    elif plant == "ragged_last_tile":       # the rows behind the last whole tile
        rows = G.act_rows(a)
        R = rows.shape[0]
        assert R % 256 == 32
        rows[R - 22:] *= 0.5
        a = rows.reshape(N, T, H, W, C).transpose(0, 1, 4, 2, 3)
    else:
        a[1, 3, 5, 7, 9] += 1.0
        a[0, 0, 63, 26, 26] -= 1.0
    from conftest import rel_l2
    assert rel_l2(a, b) < 2e-2               # invisible to the whole-tensor norm at the bf16 bound
    with pytest.raises(AssertionError):
        G.compare_act(a, b, 2e-2, plant, "bf16", rtol=2.0 ** -6, atol_rel=2.0 ** -6)


def test_weight_gradient_rows():
    rng = np.random.default_rng(1)
    b = rng.standard_normal((256, 64, 3, 3))
    a = b * (1 + 1e-3 * rng.standard_normal(b.shape))
    G.compare_local(a, b, 2e-2, "dw", local_factor=4.0, part_outliers=0.02, part_cap=25.0)
    one = a.copy()
    one[17] *= 1.2                           # one output channel moved by a flipped decision: tolerated
    G.compare_local(one, b, 2e-2, "dw", local_factor=4.0, part_outliers=0.02, part_cap=25.0)
    tile = a.copy()
    tile[64:128, :32] = 0.0                  # a 64 x 32 tile never written
    with pytest.raises(AssertionError):
        G.compare_local(tile, b, 2e-1, "dw", local_factor=0.4, part_outliers=0.02, part_cap=2.5)
    far = a.copy()
    far[3] = -far[3]                         # one channel far out
    with pytest.raises(AssertionError):
        G.compare_local(far, b, 2e-1, "dw", local_factor=0.4, part_outliers=0.02, part_cap=2.5)
