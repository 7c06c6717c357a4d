"""CPU ORACLE for the TSM training hot path -- test infrastructure only.

Nothing in the product path may import this module; only the tests, the smoke
check and the CPU-baseline leg of the benchmark do.  It shares no code with
the HIP path.

Everything is float64 numpy on tensors laid out as the paper's five-dimensional
activation ``[N, T, C, H, W]`` (section 2, "Preliminary").  The only compiled
piece is the direct-summation 2-D convolution in ``conv_direct.c``.

What each function follows:

* ``shift`` / ``shift_adjoint`` -- the Temporal Shift Module of section 2
  ("Temporal modeling unit") and Fig. 1: part of the channels move along the
  temporal axis between consecutive frames, with no arithmetic and no
  parameters.  The paper leaves the proportion and the direction per channel
  group open; the reading used here: ``fold = C // fold_div`` channels
  ``[0, fold)`` take their value from frame ``t+1``, channels
  ``[fold, 2*fold)`` from frame ``t-1``, all others stay; frames outside the
  clip read as zero; nothing crosses from one clip to the next.
* ``conv_*`` -- per-frame 2-D convolution ("pure 2D CNN", section 2) of the
  explicitly shifted input, plus its two adjoints.
* ``bn_*``, ``relu*`` -- training-mode batch normalisation over all N*T frames
  and ReLU; the paper names BatchNorm only in its training setting (section
  4.1); the standard definitions are used (biased batch variance, eps 1e-5).
* block / network functions -- ResNet-50 with the shift "inserted into every
  ResBlock" (section 3, model (3)), 8 frames, no temporal pooling (Table 2),
  400 classes (section 4.1), SGD with weight decay 1e-4 that skips BatchNorm
  and bias parameters (section 4.1).
* ``Gates`` -- not arithmetic of the method: a way to take the 0/1 decisions of
  ReLU and max-pooling in the precision of the implementation under test while
  all arithmetic stays plain fp64.

Parity status: every function below is pinned by ``tests/test_oracle_*.py``
(closed forms, adjoint identities, library special cases, finite differences,
the paper's Table 1 parameter and FLOP counts).  The paper's accuracy figures
need the Kinetics data and are "parity unpinned".
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.build()
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ints = [ctypes.c_int] * 9
        for name in ("oracle_conv2d_fwd", "oracle_conv2d_dgrad", "oracle_conv2d_wgrad"):
            fn = getattr(lib, name)
            fn.argtypes = [dp, dp, dp] + ints
            fn.restype = None
        lib.oracle_max_threads.restype = ctypes.c_int
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        _LIB = lib
    return _LIB


def max_threads():
    return int(_lib().oracle_max_threads())


def set_threads(n):
    _lib().oracle_set_threads(int(n))


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _c64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------
# Temporal shift (section 2, Fig. 1)
# ----------------------------------------------------------------------------

def fold_of(C, fold_div):
    """Number of channels moved in each direction; fold_div == 0 means no shift."""
    if fold_div == 0:
        return 0
    if fold_div < 0:
        raise ValueError("fold_div must be >= 0")
    fold = C // fold_div
    if 2 * fold > C:
        raise ValueError("fold_div leaves no room for two shifted groups")
    return fold


def shift(x, fold_div):
    """S(x): group 1 reads frame t+1, group 2 reads frame t-1, zero at clip ends."""
    N, T, C, H, W = x.shape
    fold = fold_of(C, fold_div)
    y = np.zeros_like(x)
    for t in range(T):
        if t + 1 < T:
            y[:, t, :fold] = x[:, t + 1, :fold]
        if t - 1 >= 0:
            y[:, t, fold:2 * fold] = x[:, t - 1, fold:2 * fold]
        y[:, t, 2 * fold:] = x[:, t, 2 * fold:]
    return y


def shift_adjoint(g, fold_div):
    """S^T(g): the opposite shift (group 1 reads t-1, group 2 reads t+1)."""
    N, T, C, H, W = g.shape
    fold = fold_of(C, fold_div)
    d = np.zeros_like(g)
    for t in range(T):
        if t - 1 >= 0:
            d[:, t, :fold] = g[:, t - 1, :fold]
        if t + 1 < T:
            d[:, t, fold:2 * fold] = g[:, t + 1, fold:2 * fold]
        d[:, t, 2 * fold:] = g[:, t, 2 * fold:]
    return d


# ----------------------------------------------------------------------------
# Per-frame 2-D convolution and adjoints (section 2: "pure 2D CNN")
# ----------------------------------------------------------------------------

def _out_hw(H, W, KH, KW, stride, pad):
    return (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1


def conv2d_frames_fwd(x, w, stride, pad):
    """x [F,Cin,H,W], w [Cout,Cin,KH,KW] -> y [F,Cout,Ho,Wo]; no shift."""
    x = _c64(x)
    w = _c64(w)
    F, Cin, H, W = x.shape
    Cout, Cin2, KH, KW = w.shape
    assert Cin == Cin2
    Ho, Wo = _out_hw(H, W, KH, KW, stride, pad)
    y = np.empty((F, Cout, Ho, Wo), dtype=np.float64)
    _lib().oracle_conv2d_fwd(_dptr(x), _dptr(w), _dptr(y), F, Cin, H, W, Cout, KH, KW, stride, pad)
    return y


def conv2d_frames_dgrad(dy, w, H, W, stride, pad):
    dy = _c64(dy)
    w = _c64(w)
    F, Cout, Ho, Wo = dy.shape
    Cout2, Cin, KH, KW = w.shape
    assert Cout == Cout2 and (Ho, Wo) == _out_hw(H, W, KH, KW, stride, pad)
    dx = np.empty((F, Cin, H, W), dtype=np.float64)
    _lib().oracle_conv2d_dgrad(_dptr(dy), _dptr(w), _dptr(dx), F, Cin, H, W, Cout, KH, KW, stride, pad)
    return dx


def conv2d_frames_wgrad(x, dy, KH, KW, stride, pad):
    x = _c64(x)
    dy = _c64(dy)
    F, Cin, H, W = x.shape
    F2, Cout, Ho, Wo = dy.shape
    assert F == F2 and (Ho, Wo) == _out_hw(H, W, KH, KW, stride, pad)
    dw = np.empty((Cout, Cin, KH, KW), dtype=np.float64)
    _lib().oracle_conv2d_wgrad(_dptr(x), _dptr(dy), _dptr(dw), F, Cin, H, W, Cout, KH, KW, stride, pad)
    return dw


def _frames(x):
    N, T = x.shape[:2]
    return x.reshape((N * T,) + x.shape[2:])


def conv_fwd(x, w, stride=1, pad=0, fold_div=0):
    """y = conv2d(S(x), w) per frame.  x [N,T,Cin,H,W] -> y [N,T,Cout,Ho,Wo]."""
    N, T = x.shape[:2]
    xs = shift(x, fold_div) if fold_div else x
    y = conv2d_frames_fwd(_frames(xs), w, stride, pad)
    return y.reshape((N, T) + y.shape[1:])


def conv_dgrad(dy, w, H, W, stride=1, pad=0, fold_div=0):
    """dx = S^T(conv2d^T(dy, w)).  dy [N,T,Cout,Ho,Wo] -> dx [N,T,Cin,H,W]."""
    N, T = dy.shape[:2]
    dxs = conv2d_frames_dgrad(_frames(dy), w, H, W, stride, pad)
    dxs = dxs.reshape((N, T) + dxs.shape[1:])
    return shift_adjoint(dxs, fold_div) if fold_div else dxs


def conv_wgrad(x, dy, KH, KW, stride=1, pad=0, fold_div=0):
    """dw = sum over frames and pixels of dy (x) S(x)."""
    xs = shift(x, fold_div) if fold_div else x
    return conv2d_frames_wgrad(_frames(xs), _frames(dy), KH, KW, stride, pad)


# 3x1x1 temporal convolution: the I3D-style inflation of a 1x1 convolution by
# k=3 along time (section 2: inflating by k multiplies computation and model
# size by k; section 3, model (2): the first 1x1 of a ResBlock is inflated).
# w [Cout, Cin, 3]; tap dt reads frame t + dt - 1; zero padding of one frame.

def _time_tap(x, dt):
    N, T = x.shape[:2]
    xt = np.zeros_like(x)
    for t in range(T):
        s = t + dt - 1
        if 0 <= s < T:
            xt[:, t] = x[:, s]
    return xt


def tconv_fwd(x, w):
    y = None
    for dt in range(3):
        part = conv_fwd(_time_tap(x, dt), w[:, :, dt, None, None])
        y = part if y is None else y + part
    return y


def tconv_dgrad(dy, w, H, W):
    N, T = dy.shape[:2]
    dx = None
    for dt in range(3):
        d = conv_dgrad(dy, w[:, :, dt, None, None], H, W)  # gradient w.r.t. the tapped view
        back = np.zeros_like(d)
        for t in range(T):
            s = t + dt - 1
            if 0 <= s < T:
                back[:, s] += d[:, t]
        dx = back if dx is None else dx + back
    return dx


def tconv_wgrad(x, dy):
    parts = [conv_wgrad(_time_tap(x, dt), dy, 1, 1)[:, :, 0, 0] for dt in range(3)]
    return np.stack(parts, axis=2)


# ----------------------------------------------------------------------------
# BatchNorm (training mode) and ReLU
# ----------------------------------------------------------------------------

_BN_AXES = (0, 1, 3, 4)


def _bc(v):
    return v.reshape(1, 1, -1, 1, 1)


def bn_fwd(y, gamma, beta, eps=1e-5):
    """Returns z = gamma * yhat + beta and the cache (yhat, rstd)."""
    mu = y.mean(axis=_BN_AXES)
    var = ((y - _bc(mu)) ** 2).mean(axis=_BN_AXES)
    rstd = 1.0 / np.sqrt(var + eps)
    yhat = (y - _bc(mu)) * _bc(rstd)
    return _bc(gamma) * yhat + _bc(beta), (yhat, rstd, mu, var)


def bn_bwd(dz, cache, gamma):
    yhat, rstd = cache[0], cache[1]
    m = dz.size // dz.shape[2]
    dbeta = dz.sum(axis=_BN_AXES)
    dgamma = (dz * yhat).sum(axis=_BN_AXES)
    dy = _bc(gamma * rstd) * (dz - _bc(dbeta) / m - yhat * _bc(dgamma) / m)
    return dy, dgamma, dbeta


def relu(z):
    return np.maximum(z, 0.0)


def relu_bwd(dout, out):
    """Gradient 1 where the output is strictly positive, else 0."""
    return dout * (out > 0)


class Gates:
    """The 0/1 decisions of a pass (which units a ReLU lets through, which window position a max-pool picks),
    recorded in one pass and imposed on another.

    A ReLU network's gradients are discontinuous in the forward values: an implementation that stores
    activations in bf16 takes a few of these decisions differently from fp64 arithmetic, and every such unit
    moves gradient entries by O(1).  Where floating point decides an integer, both sides of a comparison have to
    take the decision in the same precision -- the kernel's.  So the block and network functions below accept a
    `gates` object: with `record` set, the pass (typically the storage-emulating one, `q = round_bf16`) stores
    its decisions under the names of the tensors; with `record` cleared, a pass (typically the plain fp64 one)
    uses the stored decisions in place of its own comparisons: z = a * gate instead of max(a, 0), gradient
    dout * gate, pooled value / routing at the recorded window position.  With gates=None nothing changes.
    A pass that replays the decisions it would have taken itself reproduces the ungated pass bit for bit."""

    def __init__(self):
        self.store = {}
        self.record = True

    def flips(self, other):
        """(decisions that differ, decisions) against another recorded set of the same network."""
        diff = total = 0
        for k, m in self.store.items():
            diff += int((m != other.store[k]).sum())
            total += m.size
        return diff, total


def _relu_g(a, gates, key):
    """ReLU of `a`; records or replays the unit decisions under `key`."""
    if gates is None:
        return relu(a)
    if gates.record:
        gates.store[key] = a > 0
        return relu(a)
    return a * gates.store[key]


def _relu_bwd_g(dout, out, gates, key):
    if gates is None or gates.record:
        return relu_bwd(dout, out)
    return dout * gates.store[key]


def _ident(a):
    return a


# ----------------------------------------------------------------------------
# Residual blocks.  The shift sits on the residual branch, in front of its
# first convolution; the shortcut carries the unshifted input.
# `q` is applied to every tensor the HIP path materialises in its storage type
# (identity for the pure fp64 oracle; bf16 rounding for the storage-emulating
# mode used to separate rounding drift from bugs).
# ----------------------------------------------------------------------------

def basic_block_fwd(x, p, fold_div=8, eps=1e-5, q=_ident, gates=None, pre=""):
    """ReLU(BN(conv3x3(ReLU(BN(conv3x3(S(x)))))) + x); p: w1,g1,b1,w2,g2,b2."""
    c = {"x": x}
    c["y1"] = q(conv_fwd(x, p["w1"], 1, 1, fold_div))
    a1, c["bn1"] = bn_fwd(c["y1"], p["g1"], p["b1"], eps)
    c["z1"] = q(_relu_g(a1, gates, pre + "z1"))
    c["y2"] = q(conv_fwd(c["z1"], p["w2"], 1, 1, 0))
    a2, c["bn2"] = bn_fwd(c["y2"], p["g2"], p["b2"], eps)
    c["out"] = q(_relu_g(a2 + x, gates, pre + "out"))
    return c["out"], c


def basic_block_bwd(dout, c, p, fold_div=8, q=_ident, gates=None, pre=""):
    g = {}
    H, W = c["x"].shape[3:]
    da2 = q(_relu_bwd_g(dout, c["out"], gates, pre + "out"))
    dy2, g["g2"], g["b2"] = bn_bwd(da2, c["bn2"], p["g2"])
    dy2 = q(dy2)
    g["w2"] = conv_wgrad(c["z1"], dy2, 3, 3, 1, 1, 0)
    dz1 = q(conv_dgrad(dy2, p["w2"], H, W, 1, 1, 0))
    da1 = q(_relu_bwd_g(dz1, c["z1"], gates, pre + "z1"))
    dy1, g["g1"], g["b1"] = bn_bwd(da1, c["bn1"], p["g1"])
    dy1 = q(dy1)
    g["w1"] = conv_wgrad(c["x"], dy1, 3, 3, 1, 1, fold_div)
    dx = q(da2 + conv_dgrad(dy1, p["w1"], H, W, 1, 1, fold_div))
    return dx, g


def bottleneck_fwd(x, p, stride=1, fold_div=8, eps=1e-5, q=_ident, temporal=False, gates=None, pre=""):
    """1x1 -> 3x3(stride) -> 1x1, BN after each, ReLU after the first two, then
    ReLU(residual + shortcut).  p: w1,g1,b1,w2,g2,b2,w3,g3,b3 and, for a
    projection shortcut, wd,gd,bd (1x1 conv with the block's stride + BN).
    temporal=True replaces the shifted 1x1 by a 3x1x1 temporal convolution
    (w1 [Cmid,Cin,3]) with no shift: the I3D-style comparison block."""
    c = {"x": x}
    if temporal:
        c["y1"] = q(tconv_fwd(x, p["w1"]))
    else:
        c["y1"] = q(conv_fwd(x, p["w1"], 1, 0, fold_div))
    a1, c["bn1"] = bn_fwd(c["y1"], p["g1"], p["b1"], eps)
    c["z1"] = q(_relu_g(a1, gates, pre + "z1"))
    c["y2"] = q(conv_fwd(c["z1"], p["w2"], stride, 1, 0))
    a2, c["bn2"] = bn_fwd(c["y2"], p["g2"], p["b2"], eps)
    c["z2"] = q(_relu_g(a2, gates, pre + "z2"))
    c["y3"] = q(conv_fwd(c["z2"], p["w3"], 1, 0, 0))
    a3, c["bn3"] = bn_fwd(c["y3"], p["g3"], p["b3"], eps)
    if "wd" in p:
        c["yd"] = q(conv_fwd(x, p["wd"], stride, 0, 0))
        sc, c["bnd"] = bn_fwd(c["yd"], p["gd"], p["bd"], eps)
    else:
        sc = x
    c["out"] = q(_relu_g(a3 + sc, gates, pre + "out"))
    return c["out"], c


def bottleneck_bwd(dout, c, p, stride=1, fold_div=8, q=_ident, temporal=False, gates=None, pre=""):
    g = {}
    H, W = c["x"].shape[3:]
    Hm, Wm = c["z1"].shape[3:]
    Ho, Wo = c["z2"].shape[3:]
    da3 = q(_relu_bwd_g(dout, c["out"], gates, pre + "out"))
    dy3, g["g3"], g["b3"] = bn_bwd(da3, c["bn3"], p["g3"])
    dy3 = q(dy3)
    g["w3"] = conv_wgrad(c["z2"], dy3, 1, 1, 1, 0, 0)
    dz2 = q(conv_dgrad(dy3, p["w3"], Ho, Wo, 1, 0, 0))
    da2 = q(_relu_bwd_g(dz2, c["z2"], gates, pre + "z2"))
    dy2, g["g2"], g["b2"] = bn_bwd(da2, c["bn2"], p["g2"])
    dy2 = q(dy2)
    g["w2"] = conv_wgrad(c["z1"], dy2, 3, 3, stride, 1, 0)
    dz1 = q(conv_dgrad(dy2, p["w2"], Hm, Wm, stride, 1, 0))
    da1 = q(_relu_bwd_g(dz1, c["z1"], gates, pre + "z1"))
    dy1, g["g1"], g["b1"] = bn_bwd(da1, c["bn1"], p["g1"])
    dy1 = q(dy1)
    if temporal:
        g["w1"] = tconv_wgrad(c["x"], dy1)
        dres = tconv_dgrad(dy1, p["w1"], H, W)
    else:
        g["w1"] = conv_wgrad(c["x"], dy1, 1, 1, 1, 0, fold_div)
        dres = conv_dgrad(dy1, p["w1"], H, W, 1, 0, fold_div)
    if "wd" in p:
        dyd, g["gd"], g["bd"] = bn_bwd(da3, c["bnd"], p["gd"])
        dyd = q(dyd)
        g["wd"] = conv_wgrad(c["x"], dyd, 1, 1, stride, 0, 0)
        dsc = conv_dgrad(dyd, p["wd"], H, W, stride, 0, 0)
    else:
        dsc = da3
    return q(dres + dsc), g


# ----------------------------------------------------------------------------
# The rest of ResNet-50: stem, pooling, head, loss, update
# ----------------------------------------------------------------------------

def maxpool_fwd(x, arg=None):
    """3x3 window, stride 2, padding 1 (padding never wins).  Returns the pooled
    tensor and, per output, the flat input index (ih*W+iw) of the first maximum
    in row-major window order.  With `arg` given (positions decided by another pass, see Gates) the
    values at those positions are returned instead of the maxima."""
    N, T, C, H, W = x.shape
    if arg is not None:
        flat = x.reshape(N * T * C, H * W)
        picked = np.take_along_axis(flat, arg.reshape(N * T * C, -1), axis=1)
        return picked.reshape(arg.shape), arg
    Ho, Wo = (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1
    best = np.full((N, T, C, Ho, Wo), -np.inf)
    arg = np.full((N, T, C, Ho, Wo), -1, dtype=np.int64)
    oh = np.arange(Ho)[:, None]
    ow = np.arange(Wo)[None, :]
    for kh in range(3):
        for kw in range(3):
            ih = oh * 2 + kh - 1
            iw = ow * 2 + kw - 1
            ok = (ih >= 0) & (ih < H) & (iw >= 0) & (iw < W)
            ihc = np.clip(ih, 0, H - 1) + 0 * iw
            iwc = np.clip(iw, 0, W - 1) + 0 * ih
            v = np.where(ok, x[:, :, :, ihc, iwc], -np.inf)
            better = v > best           # strict: the first maximum is kept
            best = np.where(better, v, best)
            arg = np.where(better, ihc * W + iwc, arg)
    return best, arg


def maxpool_bwd(dout, arg, H, W):
    N, T, C, Ho, Wo = dout.shape
    dx = np.zeros((N * T * C, H * W))
    flat_arg = arg.reshape(N * T * C, Ho * Wo)
    rows = np.repeat(np.arange(N * T * C), Ho * Wo)
    np.add.at(dx, (rows, flat_arg.ravel()), dout.reshape(-1))
    return dx.reshape(N, T, C, H, W)


def head_fwd(feat, wfc, bfc, labels):
    """feat [N,T,C,H,W] -> global average pool -> fc per frame -> mean over T
    (temporal consensus) -> softmax cross-entropy, mean over clips."""
    pooled = feat.mean(axis=(3, 4))                       # [N,T,C]
    frame_logits = pooled @ wfc.T + bfc                   # [N,T,K]
    logits = frame_logits.mean(axis=1)                    # [N,K]
    zmax = logits.max(axis=1, keepdims=True)
    logp = logits - zmax - np.log(np.exp(logits - zmax).sum(axis=1, keepdims=True))
    N = logits.shape[0]
    loss = -logp[np.arange(N), labels].mean()
    return loss, logits, (pooled, logp)


def head_bwd(cache, feat_shape, wfc, labels):
    pooled, logp = cache
    N, T, C, H, W = feat_shape
    dlogits = np.exp(logp)
    dlogits[np.arange(N), labels] -= 1.0
    dlogits /= N
    dframe = np.repeat(dlogits[:, None, :], T, axis=1) / T     # [N,T,K]
    dwfc = np.einsum("ntk,ntc->kc", dframe, pooled)
    dbfc = dframe.sum(axis=(0, 1))
    dpooled = dframe @ wfc                                      # [N,T,C]
    dfeat = np.broadcast_to(dpooled[:, :, :, None, None] / (H * W), feat_shape).copy()
    return dfeat, dwfc, dbfc, dlogits


STAGES = (("res2", 3, 64, 1), ("res3", 4, 128, 2), ("res4", 6, 256, 2), ("res5", 3, 512, 2))


def resnet50_param_table(num_classes=400):
    """Ordered (name, shape, decays) list for TSM-ResNet-50; stride sits on the
    3x3 convolution, which reproduces the FLOP count of Table 1."""
    t = [("conv1.w", (64, 3, 7, 7), True), ("bn1.g", (64,), False), ("bn1.b", (64,), False)]
    cin = 64
    for name, blocks, mid, _ in STAGES:
        for b in range(blocks):
            pre = "%s.%d." % (name, b)
            t += [(pre + "c1.w", (mid, cin, 1, 1), True), (pre + "bn1.g", (mid,), False), (pre + "bn1.b", (mid,), False),
                  (pre + "c2.w", (mid, mid, 3, 3), True), (pre + "bn2.g", (mid,), False), (pre + "bn2.b", (mid,), False),
                  (pre + "c3.w", (4 * mid, mid, 1, 1), True), (pre + "bn3.g", (4 * mid,), False), (pre + "bn3.b", (4 * mid,), False)]
            if b == 0:
                t += [(pre + "ds.w", (4 * mid, cin, 1, 1), True), (pre + "dsbn.g", (4 * mid,), False), (pre + "dsbn.b", (4 * mid,), False)]
            cin = 4 * mid
    t += [("fc.w", (num_classes, 2048), True), ("fc.b", (num_classes,), False)]
    return t


def resnet50_param_count(num_classes=400):
    return sum(int(np.prod(s)) for _, s, _ in resnet50_param_table(num_classes))


def resnet50_macs_per_frame(size=224, num_classes=400):
    """Multiply-accumulates of one frame's forward pass (convolutions + fc)."""
    h = (size + 6 - 7) // 2 + 1
    macs = 64 * 3 * 49 * h * h
    h = (h + 2 - 3) // 2 + 1
    cin = 64
    for _, blocks, mid, stride in STAGES:
        for b in range(blocks):
            s = stride if b == 0 else 1
            ho = (h + 2 - 3) // s + 1
            macs += mid * cin * h * h + mid * mid * 9 * ho * ho + 4 * mid * mid * ho * ho
            if b == 0:
                macs += 4 * mid * cin * ho * ho
            cin, h = 4 * mid, ho
    return macs + num_classes * 2048


def unflatten_params(flat, num_classes=400):
    out, off = {}, 0
    for name, shape, _ in resnet50_param_table(num_classes):
        n = int(np.prod(shape))
        out[name] = np.asarray(flat[off:off + n], dtype=np.float64).reshape(shape)
        off += n
    assert off == len(flat)
    return out


def flatten_params(d, num_classes=400):
    return np.concatenate([np.asarray(d[name], dtype=np.float64).ravel()
                           for name, _, _ in resnet50_param_table(num_classes)])


def _block_params(P, pre, proj):
    p = {"w1": P[pre + "c1.w"], "g1": P[pre + "bn1.g"], "b1": P[pre + "bn1.b"],
         "w2": P[pre + "c2.w"], "g2": P[pre + "bn2.g"], "b2": P[pre + "bn2.b"],
         "w3": P[pre + "c3.w"], "g3": P[pre + "bn3.g"], "b3": P[pre + "bn3.b"]}
    if proj:
        p.update({"wd": P[pre + "ds.w"], "gd": P[pre + "dsbn.g"], "bd": P[pre + "dsbn.b"]})
    return p


_BLOCK_KEYS = {"w1": "c1.w", "g1": "bn1.g", "b1": "bn1.b", "w2": "c2.w", "g2": "bn2.g", "b2": "bn2.b",
               "w3": "c3.w", "g3": "bn3.g", "b3": "bn3.b", "wd": "ds.w", "gd": "dsbn.g", "bd": "dsbn.b"}


def resnet50_fwd_bwd(P, clips, labels, fold_div=8, eps=1e-5, q=_ident, wq=_ident, gates=None):
    """One forward + backward pass of TSM-ResNet-50.
    P: dict name -> float64 array; clips [N,T,3,S,S]; labels [N] ints.
    `wq` is applied to the convolution weights before use (the HIP path keeps a
    bf16 working copy of them); `q` as in the block functions; `gates` records or
    imposes the ReLU / max-pool decisions (see Gates).
    Returns loss, logits [N,K], grads dict (same names as P)."""
    num_classes = P["fc.w"].shape[0]
    G = {}
    w0 = wq(P["conv1.w"])
    y0 = q(conv_fwd(clips, w0, 2, 3, 0))
    a0, bn0 = bn_fwd(y0, P["bn1.g"], P["bn1.b"], eps)
    z0 = q(_relu_g(a0, gates, "stem.z"))
    if gates is not None and not gates.record:
        x, pool_arg = maxpool_fwd(z0, gates.store["stem.pool"])
    else:
        x, pool_arg = maxpool_fwd(z0)
        if gates is not None:
            gates.store["stem.pool"] = pool_arg
    caches = []
    for name, blocks, mid, stride in STAGES:
        for b in range(blocks):
            pre = "%s.%d." % (name, b)
            p = _block_params(P, pre, b == 0)
            for k in ("w1", "w2", "w3", "wd"):
                if k in p:
                    p[k] = wq(p[k])
            s = stride if b == 0 else 1
            x, c = bottleneck_fwd(x, p, s, fold_div, eps, q, gates=gates, pre=pre)
            caches.append((pre, p, s, c))
    loss, logits, hc = head_fwd(x, P["fc.w"], P["fc.b"], labels)
    dx, G["fc.w"], G["fc.b"], _ = head_bwd(hc, x.shape, P["fc.w"], labels)
    dx = q(dx)
    for pre, p, s, c in reversed(caches):
        dx, g = bottleneck_bwd(dx, c, p, s, fold_div, q, gates=gates, pre=pre)
        for k, v in g.items():
            G[pre + _BLOCK_KEYS[k]] = v
    dz0 = maxpool_bwd(dx, pool_arg, z0.shape[3], z0.shape[4])
    da0 = q(_relu_bwd_g(dz0, z0, gates, "stem.z"))
    dy0, G["bn1.g"], G["bn1.b"] = bn_bwd(da0, bn0, P["bn1.g"])
    dy0 = q(dy0)
    G["conv1.w"] = conv_wgrad(clips, dy0, 7, 7, 2, 3, 0)
    assert set(G) == set(P) and num_classes == logits.shape[1]
    return loss, logits, G


# ----------------------------------------------------------------------------
# Forward-only (inference) path: BatchNorm with given statistics.  The paper measures single-GPU
# throughput of the models this way (section 3a, Table 1: videos per second, forward only, batch 16).
# ----------------------------------------------------------------------------

def bn_eval(y, gamma, beta, mean, var, eps=1e-5):
    """BatchNorm in inference mode: the per-channel affine map gamma*(y-mean)/sqrt(var+eps)+beta with
    statistics supplied by the caller (running averages) instead of computed from the batch."""
    return (y - _bc(mean)) / np.sqrt(_bc(var) + eps) * _bc(gamma) + _bc(beta)


def bn_state_slots():
    """Ordered (BatchNorm parameter prefix, channels) of the running-statistics vector: per BatchNorm its
    mean [C] then its variance [C], BatchNorms in the order of the parameter table."""
    return [(n[:-2], shp[0]) for n, shp, _ in resnet50_param_table() if n.endswith(".g")]


def bn_state_count():
    return sum(2 * c for _, c in bn_state_slots())


def unflatten_bn_state(flat):
    out, off = {}, 0
    for name, c in bn_state_slots():
        out[name] = (np.asarray(flat[off:off + c], dtype=np.float64), np.asarray(flat[off + c:off + 2 * c], dtype=np.float64))
        off += 2 * c
    assert off == len(flat)
    return out


def bottleneck_infer(x, p, stats, stride=1, fold_div=8, eps=1e-5, q=_ident):
    """bottleneck_fwd with every BatchNorm in inference mode.  stats: "1","2","3" (and "d") -> (mean, var)."""
    z1 = q(relu(bn_eval(q(conv_fwd(x, p["w1"], 1, 0, fold_div)), p["g1"], p["b1"], *stats["1"], eps=eps)))
    z2 = q(relu(bn_eval(q(conv_fwd(z1, p["w2"], stride, 1, 0)), p["g2"], p["b2"], *stats["2"], eps=eps)))
    a3 = bn_eval(q(conv_fwd(z2, p["w3"], 1, 0, 0)), p["g3"], p["b3"], *stats["3"], eps=eps)
    if "wd" in p:
        sc = q(bn_eval(q(conv_fwd(x, p["wd"], stride, 0, 0)), p["gd"], p["bd"], *stats["d"], eps=eps))
    else:
        sc = x
    return q(relu(a3 + sc))


def resnet50_infer(P, bn_state, clips, fold_div=8, eps=1e-5, q=_ident, wq=_ident):
    """Forward pass of TSM-ResNet-50 in inference mode: logits [N,K] (mean over the T per-frame predictions).
    bn_state: flat running-statistics vector (see bn_state_slots)."""
    S = unflatten_bn_state(bn_state)
    y0 = q(conv_fwd(clips, wq(P["conv1.w"]), 2, 3, 0))
    z0 = q(relu(bn_eval(y0, P["bn1.g"], P["bn1.b"], *S["bn1"], eps=eps)))
    x, _ = maxpool_fwd(z0)
    for name, blocks, mid, stride in STAGES:
        for b in range(blocks):
            pre = "%s.%d." % (name, b)
            p = _block_params(P, pre, b == 0)
            for k in ("w1", "w2", "w3", "wd"):
                if k in p:
                    p[k] = wq(p[k])
            st = {"1": S[pre + "bn1"], "2": S[pre + "bn2"], "3": S[pre + "bn3"]}
            if b == 0:
                st["d"] = S[pre + "dsbn"]
            x = bottleneck_infer(x, p, st, stride if b == 0 else 1, fold_div, eps, q)
    pooled = x.mean(axis=(3, 4))
    return (pooled @ P["fc.w"].T + P["fc.b"]).mean(axis=1)


def resnet50_batch_stats(P, clips, fold_div=8, eps=1e-5, q=_ident, wq=_ident):
    """Training-mode forward pass that records, per BatchNorm, the batch mean and (biased) variance it
    normalised with, as a flat vector in the bn_state layout: statistics of the kind the running averages
    converge to, used to give the inference path realistic inputs."""
    S = {}
    y0 = q(conv_fwd(clips, wq(P["conv1.w"]), 2, 3, 0))
    a0, bn0 = bn_fwd(y0, P["bn1.g"], P["bn1.b"], eps)
    S["bn1"] = (bn0[2], bn0[3])
    x, _ = maxpool_fwd(q(relu(a0)))
    for name, blocks, mid, stride in STAGES:
        for b in range(blocks):
            pre = "%s.%d." % (name, b)
            p = _block_params(P, pre, b == 0)
            for k in ("w1", "w2", "w3", "wd"):
                if k in p:
                    p[k] = wq(p[k])
            x, c = bottleneck_fwd(x, p, stride if b == 0 else 1, fold_div, eps, q)
            for k, slot in (("bn1", "bn1"), ("bn2", "bn2"), ("bn3", "bn3"), ("bnd", "dsbn")):
                if k in c:
                    S[pre + slot] = (c[k][2], c[k][3])
    return np.concatenate([np.concatenate([np.ravel(S[n][0]), np.ravel(S[n][1])]) for n, _ in bn_state_slots()])


def sgd_update(P, V, G, lr, momentum=0.9, weight_decay=1e-4, num_classes=400):
    """g <- g + wd*w on convolution and fc weights only (no decay on BatchNorm
    and bias, section 4.1); v <- momentum*v + g; w <- w - lr*v."""
    P2, V2 = {}, {}
    for name, _, decays in resnet50_param_table(num_classes):
        g = G[name] + (weight_decay * P[name] if decays else 0.0)
        V2[name] = momentum * V[name] + g
        P2[name] = P[name] - lr * V2[name]
    return P2, V2


def resnet50_step(P, V, clips, labels, lr, momentum=0.9, weight_decay=1e-4,
                  fold_div=8, eps=1e-5, q=_ident, wq=_ident, gates=None):
    loss, logits, G = resnet50_fwd_bwd(P, clips, labels, fold_div, eps, q, wq, gates)
    P2, V2 = sgd_update(P, V, G, lr, momentum, weight_decay, P["fc.w"].shape[0])
    return loss, logits, G, P2, V2


def resnet50_accum_step(P, V, micro_batches, lr, momentum=0.9, weight_decay=1e-4,
                        fold_div=8, eps=1e-5, q=_ident, wq=_ident):
    """One update from k micro-batches (gradient accumulation, the way the paper simulates node counts it
    could not run, section 4.2): every micro-batch (clips, labels) goes through forward + backward on its own
    (its BatchNorms see only its own frames), the k gradients are averaged, and one SGD update is applied.
    Returns the list of micro-batch losses, the averaged gradients, and the updated P, V."""
    k = len(micro_batches)
    losses, acc = [], None
    for clips, labels in micro_batches:
        loss, _, G = resnet50_fwd_bwd(P, clips, labels, fold_div, eps, q, wq)
        losses.append(loss)
        acc = dict(G) if acc is None else {n: acc[n] + G[n] for n in acc}
    G = {n: v / k for n, v in acc.items()}
    P2, V2 = sgd_update(P, V, G, lr, momentum, weight_decay, P["fc.w"].shape[0])
    return losses, G, P2, V2


def lr_schedule(epoch, total_batch, warm_batch=8, warmup_epochs=5.0, total_epochs=100.0, base_lr=0.00125, base_batch=8):
    """Learning rate at (fractional) `epoch` of the paper's recipe (section 4.1): base_lr per base_batch samples
    scaled linearly with the total batch (eta = 0.00125 k for k GPUs of 8 clips); gradual warm-up over the first
    warmup_epochs, rising linearly from the rate of `warm_batch` samples (one GPU's batch) to the full rate;
    then cosine decay that reaches zero at total_epochs."""
    peak = base_lr * total_batch / base_batch
    start = base_lr * min(warm_batch, total_batch) / base_batch
    if epoch < warmup_epochs:
        return start + (peak - start) * epoch / warmup_epochs
    if epoch >= total_epochs:
        return 0.0
    return 0.5 * peak * (1.0 + np.cos(np.pi * (epoch - warmup_epochs) / (total_epochs - warmup_epochs)))


# ----------------------------------------------------------------------------
# bf16 storage emulation (round-to-nearest-even on the upper 16 bits of fp32)
# ----------------------------------------------------------------------------

def round_bf16(a):
    f = np.asarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    out = r.view(np.float32).astype(np.float64)
    return np.where(np.isfinite(f), out, f.astype(np.float64)).reshape(np.shape(a))
