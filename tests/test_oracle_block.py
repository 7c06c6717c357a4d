"""Pins for the oracle's BatchNorm/ReLU and residual blocks: normalisation
properties, projection property of the BN gradient, finite differences through
whole blocks, the gamma3 = 0 special case, and TSM == 3x1x1 block with one-hot
temporal weights."""
import numpy as np
import pytest

from oracle import tsm_oracle as O


def test_bn_normalises_and_is_affine_invariant():
    rng = np.random.default_rng(0)
    y = rng.standard_normal((2, 3, 5, 4, 4)) * 3 + 2
    g, b = rng.standard_normal(5), rng.standard_normal(5)
    z, (yhat, rstd, mu, var) = O.bn_fwd(y, g, b, eps=0.0)
    assert np.allclose(yhat.mean(axis=(0, 1, 3, 4)), 0, atol=1e-12)
    assert np.allclose(yhat.var(axis=(0, 1, 3, 4)), 1, atol=1e-12)
    assert np.allclose(z, g.reshape(1, 1, 5, 1, 1) * yhat + b.reshape(1, 1, 5, 1, 1))
    a = np.array([2.0, 0.5, 3.0, 1.5, 7.0]).reshape(1, 1, 5, 1, 1)
    z2, _ = O.bn_fwd(a * y + 11.0, g, b, eps=0.0)
    assert np.allclose(z, z2, atol=1e-10)
    # biased variance: matches numpy's population variance
    assert np.allclose(var, y.var(axis=(0, 1, 3, 4)), atol=1e-12)


def test_bn_bwd_projection_and_finite_differences():
    rng = np.random.default_rng(1)
    y = rng.standard_normal((2, 2, 3, 3, 3))
    g, b = rng.standard_normal(3) + 2, rng.standard_normal(3)
    dz = rng.standard_normal(y.shape)
    z, cache = O.bn_fwd(y, g, b, eps=0.0)     # the projection property is exact only at eps = 0
    dy, dg, db = O.bn_bwd(dz, cache, g)
    assert np.allclose(dy.sum(axis=(0, 1, 3, 4)), 0, atol=1e-12)
    assert np.allclose((dy * cache[0]).sum(axis=(0, 1, 3, 4)), 0, atol=1e-10)
    z, cache = O.bn_fwd(y, g, b)
    dy, dg, db = O.bn_bwd(dz, cache, g)
    f = lambda yy, gg, bb: (O.bn_fwd(yy, gg, bb)[0] * dz).sum()
    for _ in range(4):
        ey, eg, eb = rng.standard_normal(y.shape), rng.standard_normal(3), rng.standard_normal(3)
        h = 1e-6
        num = (f(y + h * ey, g + h * eg, b + h * eb) - f(y - h * ey, g - h * eg, b - h * eb)) / (2 * h)
        ana = (dy * ey).sum() + (dg * eg).sum() + (db * eb).sum()
        assert abs(num - ana) < 1e-6 * max(1, abs(num))


def test_relu_gradient_is_zero_at_zero():
    out = np.array([0.0, 1.0, 0.0, 2.0])
    assert np.array_equal(O.relu_bwd(np.ones(4), out), [0, 1, 0, 1])
    assert np.array_equal(O.relu(np.array([-1.0, 0.0, 3.0])), [0, 0, 3])


def _bparams(rng, cin, mid, proj, cout=None, temporal=False):
    cout = cout or cin
    p = {"w1": rng.standard_normal((mid, cin, 3) if temporal else (mid, cin, 1, 1)) * 0.4,
         "w2": rng.standard_normal((mid, mid, 3, 3)) * 0.2, "w3": rng.standard_normal((cout, mid, 1, 1)) * 0.4}
    for i, c in (("1", mid), ("2", mid), ("3", cout)):
        p["g" + i], p["b" + i] = rng.standard_normal(c) * 0.3 + 1, rng.standard_normal(c) * 0.3
    if proj:
        p["wd"] = rng.standard_normal((cout, cin, 1, 1)) * 0.4
        p["gd"], p["bd"] = rng.standard_normal(cout) * 0.3 + 1, rng.standard_normal(cout) * 0.3
    return p


def _fd_check(fwd, bwd, x, p, dout, rng, tol=2e-5):
    out, c = fwd(x, p)
    dx, g = bwd(dout, c, p)
    f = lambda xx, pp: (fwd(xx, pp)[0] * dout).sum()
    for _ in range(4):
        ex = rng.standard_normal(x.shape)
        ep = {k: rng.standard_normal(v.shape) for k, v in p.items()}
        h = 1e-6
        pp = {k: v + h * ep[k] for k, v in p.items()}
        pm = {k: v - h * ep[k] for k, v in p.items()}
        num = (f(x + h * ex, pp) - f(x - h * ex, pm)) / (2 * h)
        ana = (dx * ex).sum() + sum((g[k] * ep[k]).sum() for k in p)
        assert abs(num - ana) < tol * max(1, abs(num)), (num, ana)


def test_basic_block_finite_differences():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((1, 3, 8, 4, 4))
    p = {"w1": rng.standard_normal((8, 8, 3, 3)) * 0.2, "w2": rng.standard_normal((8, 8, 3, 3)) * 0.2,
         "g1": rng.standard_normal(8) * 0.3 + 1, "b1": rng.standard_normal(8) * 0.3,
         "g2": rng.standard_normal(8) * 0.3 + 1, "b2": rng.standard_normal(8) * 0.3}
    dout = rng.standard_normal(x.shape)
    _fd_check(lambda a, b: O.basic_block_fwd(a, b, 4), lambda d, c, b: O.basic_block_bwd(d, c, b, 4), x, p, dout, rng)


@pytest.mark.parametrize("stride,proj,temporal", [(1, False, False), (2, True, False), (1, True, False), (1, False, True)])
def test_bottleneck_finite_differences(stride, proj, temporal):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 3, 8, 4, 4))
    p = _bparams(rng, 8, 4, proj, 8 if not proj else 12, temporal)
    ho = 4 // stride
    dout = rng.standard_normal((2, 3, p["w3"].shape[0], ho, ho))
    _fd_check(lambda a, b: O.bottleneck_fwd(a, b, stride, 4, temporal=temporal),
              lambda d, c, b: O.bottleneck_bwd(d, c, b, stride, 4, temporal=temporal), x, p, dout, rng)


def test_zero_last_gamma_leaves_only_the_shortcut():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 3, 8, 4, 4))
    p = _bparams(rng, 8, 4, False)
    p["g3"][:] = 0
    p["b3"][:] = 0
    out, c = O.bottleneck_fwd(x, p, 1, 4)
    assert np.array_equal(out, np.maximum(x, 0))
    dout = rng.standard_normal(x.shape)
    dx, g = O.bottleneck_bwd(dout, c, p, 1, 4)
    assert np.allclose(dx, dout * (x > 0), atol=1e-12)
    assert np.allclose(g["w1"], 0) and np.allclose(g["w2"], 0) and np.allclose(g["w3"], 0)


def test_shift_is_on_the_residual_branch_only():
    """With the residual branch silenced the block must not move anything in time."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 4, 8, 2, 2))
    p = _bparams(rng, 8, 4, False)
    p["g3"][:] = 0
    p["b3"][:] = 0
    out, _ = O.bottleneck_fwd(x, p, 1, 4)
    assert np.array_equal(out, np.maximum(x, 0))   # shortcut sees the unshifted input
    p["g3"][:] = 1
    a, _ = O.bottleneck_fwd(x, p, 1, 4)
    b, _ = O.bottleneck_fwd(x, p, 1, 0)
    assert not np.allclose(a, b)                     # and the residual branch does shift


def test_tsm_block_equals_temporal_block_with_one_hot_weights():
    rng = np.random.default_rng(6)
    C, mid, fold = 16, 4, 2
    x = rng.standard_normal((2, 5, C, 3, 3))
    p = _bparams(rng, C, mid, False)
    wt = np.zeros((mid, C, 3))
    w = p["w1"][:, :, 0, 0]
    wt[:, :fold, 2] = w[:, :fold]                 # group 1 reads t+1
    wt[:, fold:2 * fold, 0] = w[:, fold:2 * fold]  # group 2 reads t-1
    wt[:, 2 * fold:, 1] = w[:, 2 * fold:]
    pt = dict(p, w1=wt)
    a, ca = O.bottleneck_fwd(x, p, 1, 8)
    b, cb = O.bottleneck_fwd(x, pt, 1, 0, temporal=True)
    assert np.allclose(a, b, atol=1e-12)
    dout = rng.standard_normal(a.shape)
    dxa, ga = O.bottleneck_bwd(dout, ca, p, 1, 8)
    dxb, gb = O.bottleneck_bwd(dout, cb, pt, 1, 0, temporal=True)
    assert np.allclose(dxa, dxb, atol=1e-11)
    assert np.allclose(ga["w1"][:, :fold, 0, 0], gb["w1"][:, :fold, 2], atol=1e-11)
    assert np.allclose(ga["w1"][:, 2 * fold:, 0, 0], gb["w1"][:, 2 * fold:, 1], atol=1e-11)


# ---- Gates: decisions recorded in one pass, imposed on another -----------------------------------------------
def test_gates_replaying_own_decisions_changes_nothing():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 3, 8, 4, 4))
    p = _bparams(rng, 8, 4, True, 12)
    dout = rng.standard_normal((2, 3, 12, 2, 2))
    out0, c0 = O.bottleneck_fwd(x, p, 2, 4)
    dx0, g0 = O.bottleneck_bwd(dout, c0, p, 2, 4)
    gates = O.Gates()
    out1, c1 = O.bottleneck_fwd(x, p, 2, 4, gates=gates, pre="b.")      # recording pass: arithmetic untouched
    dx1, g1 = O.bottleneck_bwd(dout, c1, p, 2, 4, gates=gates, pre="b.")
    assert np.array_equal(out0, out1) and np.array_equal(dx0, dx1)
    assert sorted(gates.store) == ["b.out", "b.z1", "b.z2"]
    assert np.array_equal(gates.store["b.out"], out0 > 0)
    gates.record = False
    out2, c2 = O.bottleneck_fwd(x, p, 2, 4, gates=gates, pre="b.")
    dx2, g2 = O.bottleneck_bwd(dout, c2, p, 2, 4, gates=gates, pre="b.")
    assert np.array_equal(out0, out2) and np.array_equal(dx0, dx2)
    assert all(np.array_equal(g0[k], g2[k]) for k in g0)
    assert gates.flips(gates) == (0, sum(m.size for m in gates.store.values()))


@pytest.mark.parametrize("kind", ["bottleneck", "basic"])
def test_gated_pass_is_the_derivative_of_the_gate_frozen_block(kind):
    """Decisions recorded from the bf16-storage pass and imposed on the plain pass: the block is then a smooth
    function of its inputs (no ReLU kinks left), its value differs from the ungated plain pass only at the few
    units the two passes decide differently, and its backward pass is exactly its derivative."""
    rng = np.random.default_rng(8)
    if kind == "bottleneck":
        x = rng.standard_normal((2, 3, 8, 5, 5))
        p = _bparams(rng, 8, 4, False)
        fwd = lambda a, b, **kw: O.bottleneck_fwd(a, b, 1, 4, **kw)
        bwd = lambda d, c, b, **kw: O.bottleneck_bwd(d, c, b, 1, 4, **kw)
    else:
        x = rng.standard_normal((1, 3, 8, 4, 4))
        p = {"w1": rng.standard_normal((8, 8, 3, 3)) * 0.2, "w2": rng.standard_normal((8, 8, 3, 3)) * 0.2,
             "g1": rng.standard_normal(8) * 0.3 + 1, "b1": rng.standard_normal(8) * 0.3,
             "g2": rng.standard_normal(8) * 0.3 + 1, "b2": rng.standard_normal(8) * 0.3}
        fwd = lambda a, b, **kw: O.basic_block_fwd(a, b, 4, **kw)
        bwd = lambda d, c, b, **kw: O.basic_block_bwd(d, c, b, 4, **kw)
    dout = rng.standard_normal(x.shape)
    gates = O.Gates()
    outq, _ = fwd(x, p, q=O.round_bf16, gates=gates, pre="")
    gates.record = False
    plain, _ = fwd(x, p)
    own = O.Gates()
    fwd(x, p, gates=own, pre="")
    nflip, ntot = gates.flips(own)
    assert nflip < 0.05 * ntot
    gated, _ = fwd(x, p, gates=gates, pre="")
    # the gated value and the plain value agree wherever no decision on the way differs; overall they are close
    assert np.linalg.norm(gated - plain) <= 0.2 * np.linalg.norm(plain)
    assert np.linalg.norm(gated - outq) < 2e-2 * np.linalg.norm(outq)
    _fd_check(lambda a, b: fwd(a, b, gates=gates, pre=""), lambda d, c, b: bwd(d, c, b, gates=gates, pre=""),
              x, p, dout, rng)


def test_maxpool_with_given_positions():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((1, 2, 3, 6, 6))
    best, arg = O.maxpool_fwd(x)
    again, arg2 = O.maxpool_fwd(x, arg)
    assert np.array_equal(best, again) and arg2 is arg
    y = x + 0.01 * rng.standard_normal(x.shape)
    picked, _ = O.maxpool_fwd(y, arg)
    flat = y.reshape(6, 36)
    assert np.array_equal(picked.reshape(6, -1), np.take_along_axis(flat, arg.reshape(6, -1), axis=1))
    assert np.all(picked <= O.maxpool_fwd(y)[0])
