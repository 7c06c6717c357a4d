"""The stem kernels inside the whole step: one train step at full frame size with each, one with the general kernel
in their place (TSM_STEM_KERNEL=0; the switches are read at every call).  The block-wide stem kernel and the general
kernel multiply the same operands in the same order and add the partial sums of the statistics over the same number
of blocks, so the forward pass must agree bit for bit and the gradients up to the order of the atomic sums of the
weight gradients.  The wavefront-per-32-pixels stem kernel (the train step's default) produces the same convolution
output bit for bit but sums the statistics in another order: its step agrees with the others to fp32 rounding of the
batch statistics.  The general kernel itself is held to the oracle by the other tests; the 64-channel 3x3 kernel, which
deals its tiles to the blocks in another order and therefore is not bit-compatible, is held to the oracle in
test_gpu_conv.py and test_gpu_block.py."""
import numpy as np
import pytest
import torch

from paper_1910_00932_amd import binding as B
from paper_1910_00932_amd import inputs as I
from conftest import rel_l2
from gpu_util import workspace

pytestmark = pytest.mark.gpu


def _step(N, T, S, monkeypatch, stem_kernel, per_wavefront=False):
    monkeypatch.setenv("TSM_CONV3X3_C64_MIN_TILES", "1")   # 2 clips are fewer tiles than the library's threshold
    monkeypatch.setenv("TSM_STEM_KERNEL", "1" if stem_kernel else "0")
    monkeypatch.setenv("TSM_STEM_PW", "1" if per_wavefront else "0")
    table = B.tsm_resnet50_param_table(400)
    flat = I.init_params([(n, s) for n, _, s, _ in table], 1)
    d = B.R50Desc(N=N, T=T, size=S, num_classes=400, fold_div=8, lr=0.01, momentum=0.9, weight_decay=1e-4, bn_eps=1e-5,
                  bn_momentum=0.1, dtype=B.TSM_BF16)
    ws = workspace(B.tsm_resnet50_workspace_bytes(d))
    params = torch.from_numpy(flat).cuda()
    mom, grads = torch.zeros_like(params), torch.empty_like(params)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    logits = torch.empty((N, 400), dtype=torch.float32, device="cuda")
    clips = torch.from_numpy(I.clips(N, T, S, 0, "bf16")).to(torch.bfloat16).cuda()
    labels = torch.from_numpy(I.labels(N)).cuda()
    B.tsm_profile_begin()
    B.tsm_resnet50_step(d, clips, labels, params, mom, None, grads, loss, logits, 1, ws)
    classes = B.tsm_profile_end()
    return classes, float(loss.item()), logits.cpu().numpy(), grads.cpu().numpy(), params.cpu().numpy()


def test_step_with_the_stem_kernel_and_with_the_general_kernel(monkeypatch):
    N, T, S = 2, 8, 224
    c1, loss1, logits1, g1, p1 = _step(N, T, S, monkeypatch, True)
    c0, loss0, logits0, g0, p0 = _step(N, T, S, monkeypatch, False)
    assert "igemm_fwd_stem" in c1 and "igemm_fwd_stem" not in c0, (sorted(c1), sorted(c0))
    assert np.isfinite(loss1) and loss1 == loss0
    assert np.array_equal(logits1, logits0)
    assert rel_l2(g1, g0) < 1e-5 and rel_l2(p1, p0) < 1e-6
    c2, loss2, logits2, g2, p2 = _step(N, T, S, monkeypatch, True, per_wavefront=True)
    assert "igemm_fwd_stem" in c2, sorted(c2)
    # (the statistics differ in the last bits of fp32; bf16 storage downstream turns that into single roundings and,
    # through the ReLU decisions they move, into gradient entries: the bounds are those of two bf16 runs of one step)
    assert abs(loss2 - loss0) < 1e-3 * abs(loss0) and rel_l2(logits2, logits0) < 2e-2
    assert rel_l2(g2, g0) < 5e-2 and rel_l2(p2, p0) < 1e-4
