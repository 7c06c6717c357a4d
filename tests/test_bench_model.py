"""The work model bench.py prices its kernel classes with, against what the paper fixes (no GPU needed).

bench.py counts algorithmic work from a layer table of TSM-ResNet-50 (never from padded tiles): the table must add up to
the model-level figure the paper prints (Table 1: 33G multiply-accumulates for TSM-ResNet-50 on 8 frames of 224x224; the
classifier is not a convolution and is not in the table), and the per-class sums must add up to the table again whatever
kernels the classes name."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import bench  # noqa: E402


def test_layer_table_adds_up_to_the_papers_multiply_accumulates():
    layers = bench.conv_layers(8, 224)                # one clip of 8 frames
    assert len(layers) == 53                          # stem + 16 blocks x 3 + 4 projections
    macs = sum(float(rout) * cout * cin * taps for _, _, cin, rout, cout, taps, _ in layers)
    # Table 1: 33G; the convolutions alone (no classifier) are 32.7G
    assert 32.5e9 < macs < 33.0e9, macs
    # only the stem has no data gradient (its input is the image)
    assert [n for n, *_, hd in layers if not hd] == ["conv1"]


@pytest.mark.parametrize("clips", [8, 16, 64])
def test_class_work_and_bytes_cover_every_layer_once(clips):
    F = clips * 8
    layers = bench.conv_layers(F, 224)
    fwd = sum(2.0 * rout * cout * cin * taps for _, _, cin, rout, cout, taps, _ in layers)
    dg = sum(2.0 * rout * cout * cin * taps for _, _, cin, rout, cout, taps, hd in layers if hd)
    work = bench.class_work(F, 224)
    assert np.isclose(sum(work.values()), 2 * fwd + dg, rtol=1e-12)
    byt = bench.class_bytes(F, 224)
    assert set(byt) == set(work)                      # every class that has work has bytes and the other way round
    assert all(v > 0 for v in byt.values())
    # without the reads of the fused epilogues a class can only move less
    plain = bench.class_bytes(F, 224, epilogue_reads=False)
    assert all(plain[k] <= byt[k] for k in byt)


def test_elementwise_bytes_closed_form():
    """Every convolution output but the stem's passes through the BatchNorm-backward map (two tensors in, one out; a
    projection's map shares the read of the upstream gradient), the outputs of a block's first two convolutions through
    BatchNorm + ReLU (one in, one out), a block's last output through the tail (two in, one out, one bit per value)."""
    F = 64 * 8
    layers = [l for l in bench.conv_layers(F, 224) if l[0] != "conv1"]
    y = {n: 2.0 * rout * cout for n, _, _, rout, cout, _, _ in layers}
    ew = bench.elementwise_bytes(F, 224)
    assert np.isclose(ew["bn_bwd_apply"], sum(3.0 * v for n, v in y.items() if not n.endswith(".ds")) +
                      sum(2.0 * v for n, v in y.items() if n.endswith(".ds")))
    assert np.isclose(ew["bn_relu_apply"], sum(2.0 * v for n, v in y.items() if n.endswith((".c1", ".c2"))))
    assert np.isclose(ew["block_tail_fwd"], sum((3.0 + 1.0 / 16.0) * v for n, v in y.items() if n.endswith(".c3")))
