"""Pins for the oracle's temporal shift (paper section 2, Fig. 1): hand-worked
case, zero-FLOP / zero-parameter permutation with zero fill, adjoint identity,
clip isolation, degenerate cases, equivalence to a one-hot temporal conv."""
import os

import numpy as np
import pytest

from oracle import tsm_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "shift_tiny.txt")


def _read_golden():
    out, key = {}, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            key = line.strip("[]")
            out[key] = []
        else:
            out[key].append([float(v) for v in line.split()])
    return {k: np.array(v) for k, v in out.items()}


def _pattern():
    t = np.arange(3)[:, None]
    c = np.arange(8)[None, :]
    return (10.0 * t + c).reshape(1, 3, 8, 1, 1)


def test_hand_worked_case():
    g = _read_golden()
    assert np.array_equal(O.shift(_pattern(), 4)[0, :, :, 0, 0], g["shift"])
    assert np.array_equal(O.shift_adjoint(_pattern(), 4)[0, :, :, 0, 0], g["adjoint"])


@pytest.mark.parametrize("shape,fd", [((2, 8, 64, 3, 5), 8), ((3, 4, 20, 2, 2), 8), ((1, 5, 7, 1, 3), 3)])
def test_values_are_inputs_or_zero_and_static_channels_untouched(shape, fd):
    rng = np.random.default_rng(0)
    x = rng.standard_normal(shape)
    x[x == 0] = 1.0
    y = O.shift(x, fd)
    fold = shape[2] // fd
    assert np.array_equal(y[:, :, 2 * fold:], x[:, :, 2 * fold:])
    # shifted channels come from t+1 / t-1 only, bit-identical, zero at the ends
    assert np.array_equal(y[:, :-1, :fold], x[:, 1:, :fold]) and np.all(y[:, -1, :fold] == 0)
    assert np.array_equal(y[:, 1:, fold:2 * fold], x[:, :-1, fold:2 * fold]) and np.all(y[:, 0, fold:2 * fold] == 0)
    # sum identity: only the frames pushed out of the clip are lost
    lost = x[:, 0, :fold].sum() + x[:, -1, fold:2 * fold].sum()
    assert abs(y.sum() - (x.sum() - lost)) < 1e-9


def test_adjoint_identity_exact_in_integers():
    rng = np.random.default_rng(1)
    x = rng.integers(-50, 50, size=(3, 6, 24, 2, 3)).astype(np.float64)
    y = rng.integers(-50, 50, size=x.shape).astype(np.float64)
    for fd in (0, 3, 4, 8, 12):
        assert (O.shift(x, fd) * y).sum() == (x * O.shift_adjoint(y, fd)).sum()


def test_adjoint_after_shift_zeroes_only_the_lost_frames():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 5, 16, 2, 2))
    r = O.shift_adjoint(O.shift(x, 4), 4)
    e = x.copy()
    e[:, 0, :4] = 0
    e[:, -1, 4:8] = 0
    assert np.array_equal(r, e)


def test_clip_isolation():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 4, 16, 2, 2))
    x[1] = np.nan
    y = O.shift(x, 8)
    assert np.isfinite(y[0]).all() and np.isfinite(y[2]).all()
    d = O.shift_adjoint(x, 8)
    assert np.isfinite(d[0]).all() and np.isfinite(d[2]).all()


def test_degenerate_cases():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 4, 16, 2, 2))
    assert np.array_equal(O.shift(x, 0), x) and np.array_equal(O.shift_adjoint(x, 0), x)
    x1 = rng.standard_normal((2, 1, 16, 2, 2))
    y1 = O.shift(x1, 8)
    assert np.all(y1[:, :, :4] == 0) and np.array_equal(y1[:, :, 4:], x1[:, :, 4:])
    with pytest.raises(ValueError):
        O.shift(x, 1)
    # C not divisible: floor
    x2 = rng.standard_normal((1, 3, 10, 1, 1))
    assert O.fold_of(10, 8) == 1
    y2 = O.shift(x2, 8)
    assert np.array_equal(y2[:, :, 2:], x2[:, :, 2:])


def test_shift_equals_one_hot_temporal_conv():
    """S(x) is the 3x1x1 temporal convolution whose weights are one-hot per
    channel: tap t+1 for group 1, tap t-1 for group 2, centre tap otherwise."""
    rng = np.random.default_rng(5)
    C, fold = 16, 2
    x = rng.standard_normal((2, 5, C, 3, 3))
    w = np.zeros((C, C, 3))
    for c in range(C):
        w[c, c, 2 if c < fold else (0 if c < 2 * fold else 1)] = 1.0
    assert np.allclose(O.tconv_fwd(x, w), O.shift(x, 8), atol=0, rtol=0)
    assert np.allclose(O.tconv_dgrad(x, w, 3, 3), O.shift_adjoint(x, 8), atol=0, rtol=0)


def test_sum_identity_counts_exactly_what_falls_off_the_clip_ends():
    """The shift only moves values and drops those pushed past a clip end: the sum over the output equals the sum
    over the input minus group 1's first frames and group 2's last frames (exact in integers); the adjoint drops
    the mirror-image frames."""
    rng = np.random.default_rng(7)
    N, T, C, H, W, fd = 3, 5, 24, 4, 3, 4
    fold = C // fd
    x = rng.integers(-50, 50, size=(N, T, C, H, W)).astype(np.float64)
    lost = x[:, 0, :fold].sum() + x[:, T - 1, fold:2 * fold].sum()
    assert O.shift(x, fd).sum() == x.sum() - lost
    lost_adj = x[:, T - 1, :fold].sum() + x[:, 0, fold:2 * fold].sum()
    assert O.shift_adjoint(x, fd).sum() == x.sum() - lost_adj
