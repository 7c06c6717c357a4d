"""tsm_block_infer (forward pass of one block, BatchNorm with running statistics) against the oracle's
bottleneck_infer: the kernel that runs the 3x3 and the last 1x1 convolution of a bottleneck in one launch, with the
tensor between them kept on the chip, element by element on ragged shapes, strides and both shortcut kinds; the
same blocks on one kernel per convolution; the plain fp32 path."""
import numpy as np
import pytest
import torch

from oracle import tsm_oracle as O
from paper_1910_00932_amd import binding as B
from paper_1910_00932_amd import inputs as I
from conftest import rel_l2
from gpu_util import CDT, CLAY, TOL, compare_act, dev_vec, empty_act, from_dev, to_dev, workspace
from test_gpu_block import make_params

pytestmark = pytest.mark.gpu


def run_infer_block(N, T, Cin, H, W, Cmid, Cout, stride, proj, fd, dtype, layout, eps=1e-5):
    p = make_params("bottleneck", Cin, Cmid, Cout, proj, dtype)
    x = I.normal((N, T, Cin, H, W), 0, dtype)
    rng = np.random.default_rng(21)
    stats, sdev = {}, {}
    for k, c in (("1", Cmid), ("2", Cmid), ("3", Cout)) + ((("d", Cout),) if proj else ()):
        m, v = (0.3 * rng.standard_normal(c)).astype(np.float32), (0.5 + rng.random(c)).astype(np.float32)
        stats[k] = (m.astype(np.float64), v.astype(np.float64))
        sdev["m" + k], sdev["v" + k] = dev_vec(m), dev_vec(v)
    Ho, Wo = (H + 2 - 3) // stride + 1, (W + 2 - 3) // stride + 1
    d = B.BlockDesc(kind=B.TSM_BLOCK_BOTTLENECK, N=N, T=T, Cin=Cin, H=H, W=W, Cmid=Cmid, Cout=Cout, stride=stride,
                    has_projection=int(proj), fold_div=fd, dtype=CDT[dtype], layout=CLAY[layout], bn_eps=eps)
    ws = workspace(B.tsm_block_infer_workspace_bytes(d))
    dp = {k: dev_vec(v, dtype if k.startswith("w") else "f32") for k, v in p.items()}
    out = empty_act((N, T, Cout, Ho, Wo), dtype, layout)
    out.fill_(float("nan"))
    B.tsm_profile_begin()
    B.tsm_block_infer(d, to_dev(x, dtype, layout), dp, sdev, out, ws)
    classes = B.tsm_profile_end()
    p64 = {k: v.astype(np.float64) for k, v in p.items()}
    x64 = x.astype(np.float64)
    ref = O.bottleneck_infer(x64, p64, stats, stride, fd, eps)
    refq = O.bottleneck_infer(x64, p64, stats, stride, fd, eps, q=O.round_bf16) if dtype == "bf16" else ref
    return from_dev(out, layout), ref, refq, classes


FUSED_CASES = [  # N,T,Cin,H,W,Cmid,stride,proj,fold_div
    (2, 3, 256, 13, 11, 64, 1, False, 8),     # 64 middle channels, ragged last tile, tiles straddle frames
    (1, 4, 512, 9, 9, 128, 1, False, 8),      # 128 middle channels: the intermediate tile fills both stages
    (1, 4, 256, 14, 14, 128, 2, True, 8),     # first block of a stage: stride 2 on the 3x3, projection shortcut
    (1, 2, 64, 10, 10, 64, 1, True, 4),       # first block of the first stage: projection at stride 1
    (3, 1, 256, 17, 5, 64, 2, True, 0),       # single-frame clips, stride 2 on an odd map, no shift
]


@pytest.mark.parametrize("case", FUSED_CASES)
def test_two_convolutions_in_one_kernel_every_element(case, monkeypatch):
    N, T, Cin, H, W, Cmid, stride, proj, fd = case
    monkeypatch.setenv("TSM_FUSED_TAIL_MIN_TILES", "1")
    got, ref, refq, classes = run_infer_block(N, T, Cin, H, W, Cmid, 4 * Cmid, stride, proj, fd, "bf16", "nthwc")
    assert ("fused_tail_%d" % Cmid) in classes, sorted(classes)
    assert np.all(np.isfinite(got))
    # frames, 256-row tiles and the whole tensor at 2e-2 against the bf16-storage oracle and the plain fp64 oracle;
    # elements as a gross-error guard (three roundings and two affine maps lie between input and output)
    compare_act(got, refq, 2e-2, "fused tail %s vs bf16-storage oracle" % (case,), "bf16", rtol=2.0 ** -5, atol_rel=2.0 ** -5)
    compare_act(got, ref, 2e-2, "fused tail %s vs fp64 oracle" % (case,), "bf16", rtol=2.0 ** -5, atol_rel=2.0 ** -5)
    # the same block on one kernel per convolution
    monkeypatch.setenv("TSM_FUSED_TAIL", "0")
    two, _, _, classes2 = run_infer_block(N, T, Cin, H, W, Cmid, 4 * Cmid, stride, proj, fd, "bf16", "nthwc")
    assert not any(k.startswith("fused_tail") for k in classes2), sorted(classes2)
    compare_act(two, refq, 2e-2, "two kernels %s vs bf16-storage oracle" % (case,), "bf16", rtol=2.0 ** -5, atol_rel=2.0 ** -5)
    assert rel_l2(got, two) < 5e-3, rel_l2(got, two)


def test_config1_block_at_full_size_takes_the_fused_kernel():
    """configs[1]'s bottleneck (256 -> 64 -> 64 -> 256 at 56x56, 8 clips x 8 frames) in inference mode on the default
    dispatch: 784 tiles, the library picks the one-kernel path."""
    got, ref, refq, classes = run_infer_block(8, 8, 256, 56, 56, 64, 256, 1, False, 8, "bf16", "nthwc")
    assert "fused_tail_64" in classes, sorted(classes)
    compare_act(got, refq, 2e-2, "configs[1] block, inference, vs bf16-storage oracle", "bf16", rtol=2.0 ** -5, atol_rel=2.0 ** -5)
    compare_act(got, ref, 2e-2, "configs[1] block, inference, vs fp64 oracle", "bf16", rtol=2.0 ** -5, atol_rel=2.0 ** -5)


def test_res3_block_at_benchmark_batch_takes_the_fused_kernel():
    """A block of the second stage (512 -> 128 -> 128 -> 512 at 28x28) at the inference benchmark's 16 clips x 8 frames."""
    got, ref, refq, classes = run_infer_block(16, 8, 512, 28, 28, 128, 512, 1, False, 8, "bf16", "nthwc")
    assert "fused_tail_128" in classes, sorted(classes)
    compare_act(got, refq, 2e-2, "res3 block, inference, vs bf16-storage oracle", "bf16", rtol=2.0 ** -5, atol_rel=2.0 ** -5)


@pytest.mark.parametrize("layout", ["nthwc", "ntchw"])
def test_block_infer_fp32(layout):
    for case in ((2, 3, 32, 6, 6, 8, 1, False, 8), (2, 2, 16, 7, 7, 8, 2, True, 4)):
        N, T, Cin, H, W, Cmid, stride, proj, fd = case
        got, ref, _, _ = run_infer_block(N, T, Cin, H, W, Cmid, 4 * Cmid, stride, proj, fd, "f32", layout)
        compare_act(got, ref, 1e-4, "fp32 block inference %s" % (case,), "f32", elem=False)


def test_block_infer_paper_order_bf16():
    got, ref, refq, _ = run_infer_block(1, 4, 256, 14, 14, 64, 256, 1, False, 8, "bf16", "ntchw")
    compare_act(got, refq, 2e-2, "bf16 block inference, paper order", "bf16", elem=False)
