"""Pins for the oracle's convolution, dgrad and wgrad (per-frame 2-D conv of the
shifted input; paper section 2): library special cases, matmul for 1x1, closed
forms, adjoint identities, finite differences, brute force on integers."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from oracle import tsm_oracle as O

CASES = [  # N,T,Cin,H,W,Cout,k,stride,pad
    (1, 2, 3, 9, 8, 4, 3, 1, 1),
    (2, 2, 5, 7, 7, 6, 3, 2, 1),
    (1, 3, 4, 6, 5, 3, 1, 1, 0),
    (1, 2, 8, 8, 8, 5, 1, 2, 0),
    (1, 1, 3, 16, 16, 4, 7, 2, 3),
]


def _rand(case, seed=0):
    N, T, Cin, H, W, Cout, k, s, p = case
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, T, Cin, H, W))
    w = rng.standard_normal((Cout, Cin, k, k))
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    dy = rng.standard_normal((N, T, Cout, Ho, Wo))
    return x, w, dy


@pytest.mark.parametrize("case", CASES)
def test_no_shift_matches_library_conv2d_and_its_autograd(case):
    N, T, Cin, H, W, Cout, k, s, p = case
    x, w, dy = _rand(case)
    xt = torch.tensor(x.reshape(N * T, Cin, H, W), requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    yt = Fn.conv2d(xt, wt, stride=s, padding=p)
    yt.backward(torch.tensor(dy.reshape(yt.shape)))
    assert np.allclose(O.conv_fwd(x, w, s, p, 0).reshape(yt.shape), yt.detach().numpy(), atol=1e-11)
    assert np.allclose(O.conv_dgrad(dy, w, H, W, s, p, 0).reshape(xt.shape), xt.grad.numpy(), atol=1e-11)
    assert np.allclose(O.conv_wgrad(x, dy, k, k, s, p, 0), wt.grad.numpy(), atol=1e-10)


def test_1x1_is_a_matrix_product():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 3, 10, 4, 5))
    w = rng.standard_normal((7, 10, 1, 1))
    y = O.conv_fwd(x, w)
    ref = np.einsum("oc,ntchw->ntohw", w[:, :, 0, 0], x)
    assert np.allclose(y, ref, atol=1e-12)


def test_closed_forms_ones_and_delta():
    x = np.ones((1, 1, 3, 5, 6))
    w = np.ones((2, 3, 3, 3))
    y = O.conv_fwd(x, w, 1, 1)
    assert np.all(y[0, 0, :, 1:-1, 1:-1] == 27)      # interior: Cin * 9
    assert np.all(y[0, 0, :, 0, 0] == 12)            # corner: Cin * 4 valid taps
    assert np.all(y[0, 0, :, 0, 1:-1] == 18)         # edge: Cin * 6
    rng = np.random.default_rng(2)
    x = rng.standard_normal((1, 2, 1, 6, 6))
    for kh, kw in itertools.product(range(3), range(3)):
        d = np.zeros((1, 1, 3, 3))
        d[0, 0, kh, kw] = 1.0
        y = O.conv_fwd(x, d, 1, 1)
        e = np.zeros_like(x)                         # y[oh,ow] = x[oh+kh-1, ow+kw-1]
        for oh, ow in itertools.product(range(6), range(6)):
            ih, iw = oh + kh - 1, ow + kw - 1
            if 0 <= ih < 6 and 0 <= iw < 6:
                e[0, :, 0, oh, ow] = x[0, :, 0, ih, iw]
        assert np.array_equal(y, e)


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("fd", [0, 2, 4])
def test_adjoint_identities_pin_dgrad_and_wgrad_from_fwd(case, fd):
    N, T, Cin, H, W, Cout, k, s, p = case
    if fd and 2 * (Cin // fd) > Cin:
        pytest.skip("fold too large")
    x, w, dy = _rand(case, 3)
    lhs = (O.conv_fwd(x, w, s, p, fd) * dy).sum()
    assert abs(lhs - (x * O.conv_dgrad(dy, w, H, W, s, p, fd)).sum()) < 1e-9 * max(1, abs(lhs))
    assert abs(lhs - (w * O.conv_wgrad(x, dy, k, k, s, p, fd)).sum()) < 1e-9 * max(1, abs(lhs))


def test_shifted_conv_is_conv_of_explicit_shift():
    case = (2, 4, 8, 5, 5, 6, 3, 1, 1)
    x, w, dy = _rand(case, 4)
    assert np.array_equal(O.conv_fwd(x, w, 1, 1, 4), O.conv_fwd(O.shift(x, 4), w, 1, 1, 0))
    assert np.array_equal(O.conv_dgrad(dy, w, 5, 5, 1, 1, 4),
                          O.shift_adjoint(O.conv_dgrad(dy, w, 5, 5, 1, 1, 0), 4))
    assert np.array_equal(O.conv_wgrad(x, dy, 3, 3, 1, 1, 4), O.conv_wgrad(O.shift(x, 4), dy, 3, 3, 1, 1, 0))
    # and the shift matters: the result differs from the unshifted conv
    assert not np.allclose(O.conv_fwd(x, w, 1, 1, 4), O.conv_fwd(x, w, 1, 1, 0))


def _brute(x, w, s, p, fd):
    """Pure-Python evaluation of the definition on integer data (exact)."""
    N, T, Cin, H, W = x.shape
    Cout, _, KH, KW = w.shape
    fold = Cin // fd if fd else 0
    Ho, Wo = (H + 2 * p - KH) // s + 1, (W + 2 * p - KW) // s + 1
    y = np.zeros((N, T, Cout, Ho, Wo))
    for n, t, co, oh, ow in itertools.product(range(N), range(T), range(Cout), range(Ho), range(Wo)):
        acc = 0
        for ci in range(Cin):
            ts = t + 1 if ci < fold else (t - 1 if ci < 2 * fold else t)
            if not 0 <= ts < T:
                continue
            for kh, kw in itertools.product(range(KH), range(KW)):
                ih, iw = oh * s + kh - p, ow * s + kw - p
                if 0 <= ih < H and 0 <= iw < W:
                    acc += int(w[co, ci, kh, kw]) * int(x[n, ts, ci, ih, iw])
        y[n, t, co, oh, ow] = acc
    return y


@pytest.mark.parametrize("s,p,k,fd", [(1, 1, 3, 4), (2, 1, 3, 4), (1, 0, 1, 2), (2, 0, 1, 0)])
def test_brute_force_integers_exact(s, p, k, fd):
    rng = np.random.default_rng(5)
    x = rng.integers(-4, 5, size=(2, 3, 8, 5, 4)).astype(np.float64)
    w = rng.integers(-3, 4, size=(3, 8, k, k)).astype(np.float64)
    assert np.array_equal(O.conv_fwd(x, w, s, p, fd), _brute(x, w, s, p, fd))


def test_finite_differences_through_shifted_conv():
    case = (1, 3, 4, 4, 4, 3, 3, 2, 1)
    x, w, dy = _rand(case, 6)
    f = lambda xx, ww: (O.conv_fwd(xx, ww, 2, 1, 2) * dy).sum()
    dx, dw = O.conv_dgrad(dy, w, 4, 4, 2, 1, 2), O.conv_wgrad(x, dy, 3, 3, 2, 1, 2)
    rng = np.random.default_rng(7)
    for _ in range(5):
        ex, ew = rng.standard_normal(x.shape), rng.standard_normal(w.shape)
        h = 1e-5
        num = (f(x + h * ex, w + h * ew) - f(x - h * ex, w - h * ew)) / (2 * h)
        assert abs(num - ((dx * ex).sum() + (dw * ew).sum())) < 1e-6 * max(1, abs(num))


def test_temporal_conv_pins():
    """3x1x1 conv: 3x the parameters of the 1x1 it inflates; centre-tap-only
    weights reduce to the 1x1; equals a 1-D correlation along t per pixel; its
    dgrad/wgrad satisfy the adjoint identities."""
    rng = np.random.default_rng(8)
    x = rng.standard_normal((2, 5, 6, 2, 3))
    w = rng.standard_normal((4, 6, 3))
    assert w.size == 3 * w[:, :, 1].size
    w0 = w.copy()
    w0[:, :, 0] = 0
    w0[:, :, 2] = 0
    assert np.allclose(O.tconv_fwd(x, w0), O.conv_fwd(x, w[:, :, 1, None, None]), atol=1e-12)
    y = O.tconv_fwd(x, w)
    ref = np.zeros_like(y)
    for n, h, ww_, co in itertools.product(range(2), range(2), range(3), range(4)):
        for ci in range(6):
            ref[n, :, co, h, ww_] += np.correlate(np.pad(x[n, :, ci, h, ww_], 1), w[co, ci], mode="valid")
    assert np.allclose(y, ref, atol=1e-12)
    dy = rng.standard_normal(y.shape)
    lhs = (y * dy).sum()
    assert abs(lhs - (x * O.tconv_dgrad(dy, w, 2, 3)).sum()) < 1e-10
    assert abs(lhs - (w * O.tconv_wgrad(x, dy)).sum()) < 1e-10
