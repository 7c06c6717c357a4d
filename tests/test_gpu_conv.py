"""Parity of the HIP shift-fused convolution, its data gradient (adjoint shift)
and weight gradient with the fp64 oracle, element by element, for the plain fp32
kernels and the bf16 MFMA kernels, in both memory orders.  Sizes span several
128-row tiles with ragged tails; tolerances are the spec ones (relative L2
1e-4 for fp32, 2e-2 for bf16)."""
import numpy as np
import pytest
import torch

from oracle import tsm_oracle as O
from paper_1910_00932_amd import binding as B
from paper_1910_00932_amd import inputs as I
from conftest import rel_l2
from gpu_util import CDT, CLAY, TDT, TOL, compare_act, compare_local, dev_vec, empty_act, from_dev, to_dev, workspace

pytestmark = pytest.mark.gpu

CASES = [  # N,T,Cin,H,W,Cout,k,stride,pad,fold_div
    (2, 8, 64, 14, 14, 64, 3, 1, 1, 8),     # configs[0] first conv
    (2, 4, 64, 14, 14, 64, 3, 1, 1, 0),     # second conv (no shift)
    (1, 4, 256, 20, 20, 64, 1, 1, 0, 8),    # bottleneck c1 (shifted 1x1), ragged M
    (1, 3, 64, 12, 12, 256, 1, 1, 0, 0),    # c3, two N tiles
    (1, 4, 128, 13, 13, 128, 3, 2, 1, 0),   # strided 3x3
    (1, 2, 256, 9, 9, 512, 1, 2, 0, 0),     # strided projection
    (2, 3, 24, 5, 6, 40, 3, 1, 1, 3),       # ragged channels, fold = 8
    (1, 2, 20, 5, 5, 12, 3, 1, 1, 8),       # channels not multiple of 8 -> plain kernels
    (1, 1, 16, 6, 6, 16, 1, 1, 0, 4),       # T = 1: both shifted groups read zeros
    (1, 1, 64, 6, 6, 64, 3, 1, 1, 0),       # fewer pixels than one 256-row tile (most blocks of the grid idle)
    (1, 4, 64, 10, 10, 64, 1, 1, 0, 8),     # 64 -> 64 1x1 with shift: 256x64 tile, 64x64 weight-gradient tile
    (2, 2, 128, 9, 9, 320, 1, 1, 0, 0),     # output channels not a multiple of the 128-column tile
    (1, 2, 192, 7, 7, 64, 3, 1, 1, 8),      # three 64-channel steps per tap, shift inside the first step only
]


def _run(case, dtype, layout):
    N, T, Cin, H, W, Cout, k, s, p, fd = case
    x = I.normal((N, T, Cin, H, W), 0, dtype)
    w = I.kaiming_conv((Cout, Cin, k, k), 1, dtype)
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    dy = I.normal((N, T, Cout, Ho, Wo), 3, dtype)
    d = B.ConvDesc(N=N, T=T, Cin=Cin, H=H, W=W, Cout=Cout, kh=k, kw=k, stride=s, pad=p, fold_div=fd,
                   dtype=CDT[dtype], layout=CLAY[layout])
    ws = workspace(B.tsm_conv_workspace_bytes(d))
    xd, wd, dyd = to_dev(x, dtype, layout), dev_vec(w, dtype), to_dev(dy, dtype, layout)
    y = empty_act((N, T, Cout, Ho, Wo), dtype, layout)
    dx = empty_act((N, T, Cin, H, W), dtype, layout)
    dw = torch.empty((Cout, Cin, k, k), dtype=torch.float32, device="cuda")
    s1 = torch.empty(Cout, dtype=torch.float32, device="cuda")
    s2 = torch.empty(Cout, dtype=torch.float32, device="cuda")
    B.tsm_conv_fwd(d, xd, wd, y, s1, s2, ws)
    B.tsm_conv_dgrad(d, dyd, wd, dx, ws)
    B.tsm_conv_wgrad(d, xd, dyd, dw, 0, ws)
    torch.cuda.synchronize()
    x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    tol = TOL[dtype]
    # whole tensor, every frame, every 256-row tile and every element (a wrong tile edge, clip-end frame or ragged
    # last tile is a fraction of a per cent of a tensor's energy)
    yo = O.conv_fwd(x64, w64, s, p, fd)
    yg = from_dev(y, layout)
    compare_act(yg, yo, tol, "fwd %s" % (case,), dtype)
    compare_act(from_dev(dx, layout), O.conv_dgrad(dy64, w64, H, W, s, p, fd), tol, "dgrad %s" % (case,), dtype)
    # the weight gradient is an fp32 sum of exact products on both storage types: per output channel, per element
    compare_local(dw.cpu().numpy(), O.conv_wgrad(x64, dy64, k, k, s, p, fd), tol, "wgrad %s" % (case,),
                  rtol=1e-3, atol_rel=1e-3)
    # statistics epilogue: the sums the oracle takes of its own output (the stored values differ from it by one
    # rounding each), and exactly the sums of the stored output
    m = N * T * Ho * Wo
    assert np.allclose(s1.cpu().numpy(), yo.sum(axis=(0, 1, 3, 4)), rtol=0, atol=(8e-3 if dtype == "bf16" else 1e-4) * np.sqrt(m) * yo.std() + 1e-12)
    # (a stored value is off by up to 2^-8 relative, its square by twice that; the sum over m values averages it down)
    assert np.allclose(s2.cpu().numpy(), (yo ** 2).sum(axis=(0, 1, 3, 4)), rtol=1e-3 + 8 * 2.0 ** -8 / np.sqrt(m) if dtype == "bf16" else 1e-4)
    assert np.allclose(s1.cpu().numpy(), yg.sum(axis=(0, 1, 3, 4)), rtol=1e-3, atol=1e-2 * np.sqrt(yg[0, 0, 0].size * N * T))
    assert np.allclose(s2.cpu().numpy(), (yg ** 2).sum(axis=(0, 1, 3, 4)), rtol=1e-3)
    return d, xd, dyd, dw, ws


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_conv_parity_channels_innermost(case, dtype):
    _run(case, dtype, "nthwc")


@pytest.mark.parametrize("case", [CASES[0], CASES[2], CASES[4], CASES[7]])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_conv_parity_paper_order(case, dtype):
    _run(case, dtype, "ntchw")


def test_wgrad_accumulate_adds():
    d, xd, dyd, dw, ws = _run(CASES[2], "bf16", "nthwc")
    first = dw.clone()
    B.tsm_conv_wgrad(d, xd, dyd, dw, 1, ws)
    torch.cuda.synchronize()
    assert rel_l2(dw.cpu().numpy(), 2 * first.cpu().numpy()) < 1e-5


def test_fold_zero_equals_unshifted_and_shift_matters():
    case = (1, 4, 64, 8, 8, 64, 1, 1, 0, 8)
    N, T, Cin, H, W, Cout, k, s, p, fd = case
    x = I.normal((N, T, Cin, H, W), 0, "bf16")
    w = I.kaiming_conv((Cout, Cin, k, k), 1, "bf16")
    outs = []
    for f in (8, 0):
        d = B.ConvDesc(N=N, T=T, Cin=Cin, H=H, W=W, Cout=Cout, kh=k, kw=k, stride=s, pad=p, fold_div=f,
                       dtype=B.TSM_BF16, layout=B.TSM_NTHWC)
        y = empty_act((N, T, Cout, H, W), "bf16", "nthwc")
        B.tsm_conv_fwd(d, to_dev(x, "bf16", "nthwc"), dev_vec(w, "bf16"), y, None, None, workspace(B.tsm_conv_workspace_bytes(d)))
        outs.append(from_dev(y, "nthwc"))
    assert rel_l2(outs[1], O.conv_fwd(x.astype(np.float64), w.astype(np.float64), s, p, 0)) < 2e-2
    assert rel_l2(outs[0], outs[1]) > 0.1


@pytest.mark.parametrize("case", [
    (8, 8, 256, 56, 56, 64, 1, 1, 0, 8),     # configs[1] first conv (shifted 1x1) at full size
    (8, 8, 64, 56, 56, 64, 3, 1, 1, 0),      # configs[1] 3x3 at full size
    (8, 8, 512, 14, 14, 512, 3, 2, 1, 0),    # strided 3x3 of the last stage's first block (parity-class dgrad)
])
def test_conv_full_size_layers(case):
    """Full-size layers in the launch configuration of the benchmark, every element against the oracle."""
    _run(case, "bf16", "nthwc")


@pytest.mark.parametrize("case", [
    (2, 8, 64, 55, 57, 64, 3, 1, 1, 0),      # widest map the kernel takes, H != W, ragged last tile
    (16, 8, 64, 20, 20, 64, 3, 1, 1, 0),     # tiles that straddle frames (400 pixels per frame)
])
def test_conv3x3_c64_kernel_every_element(case, monkeypatch):
    """The 64 -> 64 channel 3x3 kernel (forward with the statistics epilogue, data gradient) on sizes the oracle
    covers element by element; the library would leave so few tiles to the general kernel, the threshold is moved."""
    monkeypatch.setenv("TSM_CONV3X3_C64_MIN_TILES", "1")
    B.tsm_profile_begin()
    _run(case, "bf16", "nthwc")
    classes = B.tsm_profile_end()
    assert "igemm_fwd_c64" in classes and "igemm_dgrad_c64" in classes, sorted(classes)


@pytest.mark.parametrize("case", [
    (2, 8, 64, 40, 40, 256, 3, 1, 1, 0),     # 3x3, 64 -> 256 channels: one column tile, nine K steps
    (2, 8, 512, 40, 40, 256, 1, 1, 0, 8),    # shifted 1x1, 512 -> 256 channels: eight K steps
    (4, 8, 128, 57, 57, 256, 3, 2, 1, 0),    # strided 3x3, 26912 pixels: a ragged last tile, an odd number of K steps
    (2, 8, 512, 31, 31, 512, 1, 1, 0, 8),    # two column tiles
])
def test_forward_with_256_column_tiles_every_element(case, monkeypatch):
    """Forward layers whose result is a multiple of 256 channels wide on 256 x 256 tiles (the staging tile of the
    epilogue lies in the operand stage that the last K step has left; statistics epilogue), on sizes the oracle covers
    element by element; the library would give so few tiles to 128-column tiles, the threshold is moved."""
    monkeypatch.setenv("TSM_IGEMM_WIDE_MIN_TILES", "1")
    B.tsm_profile_begin()
    _run(case, "bf16", "nthwc")
    classes = B.tsm_profile_end()
    assert "igemm_fwd_256x256" in classes, sorted(classes)


@pytest.mark.parametrize("case", [
    (2, 4, 64, 57, 57, 256, 1, 1, 0, 0),     # 25992 pixels: a ragged last pass of 8 pixels
    (3, 8, 64, 33, 35, 256, 1, 1, 0, 0),     # 27720 pixels, H != W; some wavefronts get one pass more than others
    (2, 8, 128, 28, 28, 512, 1, 1, 0, 0),    # 128 -> 512 channels: the result is split over pairs of blocks
    (2, 8, 128, 41, 41, 256, 1, 1, 0, 0),    # 128 -> 256 channels, ragged last pass
    (2, 8, 64, 30, 30, 512, 1, 1, 0, 0),     # 64 -> 512 channels
    (2, 8, 256, 27, 29, 1024, 1, 1, 0, 0),   # 256 -> 1024 channels: blocks of 128 result channels, eight per stream
    (2, 8, 256, 31, 31, 512, 1, 1, 0, 0),    # 256 -> 512 channels
])
def test_pointwise_forward_kernel_every_element(case, monkeypatch):
    """The short-K, wide-result 1x1 forward kernel (statistics epilogue; one wavefront per 32 pixels, nothing shared but
    the weights) on sizes the oracle covers element by element; the library would leave so few pixels to the general
    kernel, the threshold is moved.  (The weight gradient of the case runs on the general kernels as usual.)"""
    monkeypatch.setenv("TSM_PW_MIN_ROWS", "1")
    B.tsm_profile_begin()
    _run(case, "bf16", "nthwc")
    classes = B.tsm_profile_end()
    assert "igemm_fwd_pw" in classes, sorted(classes)


@pytest.mark.parametrize("case", [
    (2, 4, 256, 57, 57, 64, 1, 1, 0, 8),     # 64 -> 256 channels of dx, shifted; 25992 pixels: a ragged last pass
    (3, 8, 256, 33, 35, 64, 1, 1, 0, 8),     # H != W, clips of 8 frames: both clip ends inside the tensor
    (2, 8, 512, 28, 28, 128, 1, 1, 0, 8),    # 128 -> 512 channels: the result is split over pairs of blocks
    (2, 8, 256, 40, 40, 128, 1, 1, 0, 8),    # 128 -> 256 channels
    (2, 8, 256, 57, 57, 64, 1, 1, 0, 0),     # no shift
    (2, 8, 1024, 27, 29, 256, 1, 1, 0, 8),   # 256 -> 1024 channels of dx: blocks of 128 result channels
    (2, 8, 512, 31, 31, 256, 1, 1, 0, 8),    # 256 -> 512 channels of dx
])
def test_pointwise_data_gradient_kernel_every_element(case, monkeypatch):
    """The short-K, wide-result 1x1 data-gradient kernel (adjoint shift on the store, zero rows at the clip ends) on
    sizes the oracle covers element by element; the threshold is moved as above.  Its fused epilogue (shortcut
    gradient, mask bits, BatchNorm sums) runs inside the block and step tests."""
    monkeypatch.setenv("TSM_PW_MIN_ROWS", "1")
    B.tsm_profile_begin()
    _run(case, "bf16", "nthwc")
    classes = B.tsm_profile_end()
    assert "igemm_dgrad_pw" in classes, sorted(classes)


def test_conv3x3_c64_kernel_where_the_library_picks_it():
    """112 frames of 56x56 (1372 tiles: the default dispatch takes the 64-channel kernel) against the oracle on the
    first, a middle and the last frame; without shift the frames are independent."""
    N, T, C, H = 14, 8, 64, 56
    x = I.normal((N, T, C, H, H), 0, "bf16")
    w = I.kaiming_conv((C, C, 3, 3), 1, "bf16")
    dy = I.normal((N, T, C, H, H), 3, "bf16")
    d = B.ConvDesc(N=N, T=T, Cin=C, H=H, W=H, Cout=C, kh=3, kw=3, stride=1, pad=1, fold_div=0, dtype=B.TSM_BF16,
                   layout=B.TSM_NTHWC)
    ws = workspace(B.tsm_conv_workspace_bytes(d))
    y, dx = empty_act((N, T, C, H, H), "bf16", "nthwc"), empty_act((N, T, C, H, H), "bf16", "nthwc")
    s1 = torch.empty(C, dtype=torch.float32, device="cuda")
    s2 = torch.empty(C, dtype=torch.float32, device="cuda")
    xd, wd, dyd = to_dev(x, "bf16", "nthwc"), dev_vec(w, "bf16"), to_dev(dy, "bf16", "nthwc")
    B.tsm_profile_begin()
    B.tsm_conv_fwd(d, xd, wd, y, s1, s2, ws)
    B.tsm_conv_dgrad(d, dyd, wd, dx, ws)
    classes = B.tsm_profile_end()
    assert "igemm_fwd_c64" in classes and "igemm_dgrad_c64" in classes, sorted(classes)
    yg, dxg = from_dev(y, "nthwc"), from_dev(dx, "nthwc")
    w64 = w.astype(np.float64)
    for f in (0, 57, N * T - 1):
        n, t = divmod(f, T)
        yo = O.conv_fwd(x[n:n + 1, t:t + 1].astype(np.float64), w64, 1, 1, 0)
        compare_act(yg[n:n + 1, t:t + 1], yo, 2e-2, "fwd frame %d" % f, "bf16", tile=64)
        dxo = O.conv_dgrad(dy[n:n + 1, t:t + 1].astype(np.float64), w64, H, H, 1, 1, 0)
        compare_act(dxg[n:n + 1, t:t + 1], dxo, 2e-2, "dgrad frame %d" % f, "bf16", tile=64)
    assert np.allclose(s1.cpu().numpy(), yg.sum(axis=(0, 1, 3, 4)), rtol=1e-3, atol=1e-2 * np.sqrt(N * T * H * H))
    assert np.allclose(s2.cpu().numpy(), (yg ** 2).sum(axis=(0, 1, 3, 4)), rtol=1e-3)


def test_conv_of_2_gib_and_more_on_the_fallback_kernels():
    """A shifted 1x1 convolution whose input exceeds the 2 GiB that the general kernels address (168 clips of
    8 frames of 112x112x64 bf16): the library routes forward and data gradient to the register-prefetch kernels
    and the weight gradient to the register-transposing one.  The tensors are drawn on the device (seeded); the
    oracle checks sampled clips -- the first, the last and the one holding byte offset 2^31 -- which is the whole
    answer for them, since neither the convolution nor the shift ever crosses from one clip to the next."""
    N, T, C, H, Co = 168, 8, 64, 112, 64
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    x = torch.randn((N, T, H, H, C), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    assert x.numel() * 2 >= 0x7ff00000
    w = I.kaiming_conv((Co, C, 1, 1), 1, "bf16")
    d = B.ConvDesc(N=N, T=T, Cin=C, H=H, W=H, Cout=Co, kh=1, kw=1, stride=1, pad=0, fold_div=8, dtype=B.TSM_BF16,
                   layout=B.TSM_NTHWC)
    ws = workspace(B.tsm_conv_workspace_bytes(d))
    y = torch.empty((N, T, H, H, Co), dtype=torch.bfloat16, device="cuda")
    s1 = torch.empty(Co, dtype=torch.float32, device="cuda")
    s2 = torch.empty(Co, dtype=torch.float32, device="cuda")
    wd = dev_vec(w, "bf16")
    B.tsm_profile_begin()
    B.tsm_conv_fwd(d, x, wd, y, s1, s2, ws)
    classes = B.tsm_profile_end()
    assert "igemm_fwd_128x64" in classes, sorted(classes)
    dx = torch.empty_like(x)
    B.tsm_profile_begin()
    B.tsm_conv_dgrad(d, y, wd, dx, ws)          # the forward result serves as the upstream gradient
    classes = B.tsm_profile_end()
    assert "igemm_dgrad_128x64" in classes, sorted(classes)
    torch.cuda.synchronize()
    w64 = w.astype(np.float64)
    n_mid = (1 << 31) // (T * H * H * C * 2)
    for n in (0, n_mid, N - 1):
        xo = from_dev(x[n:n + 1], "nthwc")
        yg = from_dev(y[n:n + 1], "nthwc")
        compare_act(yg, O.conv_fwd(xo, w64, 1, 0, 8), 2e-2, "fwd clip %d" % n, "bf16")
        compare_act(from_dev(dx[n:n + 1], "nthwc"), O.conv_dgrad(yg, w64, H, H, 1, 0, 8), 2e-2, "dgrad clip %d" % n, "bf16")
    yf = y.float()
    assert np.allclose(s1.cpu().numpy(), yf.sum(dim=(0, 1, 2, 3)).cpu().numpy(), rtol=1e-3, atol=1e-2 * np.sqrt(N * T * H * H))
    assert np.allclose(s2.cpu().numpy(), (yf * yf).sum(dim=(0, 1, 2, 3)).cpu().numpy(), rtol=1e-3)
