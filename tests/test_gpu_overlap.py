"""The backward entry points run their weight gradients on a second stream; TSM_WGRAD_OVERLAP=0 keeps one stream.
Both settings must give the same step (the switch is read once per process, so each setting runs in a process
of its own; results differ only by the order of the atomic sums of the weight gradients).

Steps run back to back, with no synchronisation in between -- the sequence that would expose a missing wait between
the tail of one step and the head of the next.  They use learning rate 0 and one last step applies the update:
every step sees the same parameters, the momentum buffer accumulates the gradients of all steps (a weight gradient
that finished after the update, or after the next step cleared the gradient buffer, would be missing from it), and
the two settings agree to the order of the atomic sums (1e-5).  Two sequences:

  * "same": the same clips in every step;
  * "fresh": different clips in every step, so that the activations in the workspace change from step to step -- a
    weight gradient still reading its operands when the next step's forward pass overwrites them reads other
    values (with the same clips the overwriting data would be identical and the race invisible).

Steps with a non-zero learning rate cannot be compared this tightly, at any size tried (up to 2 clips x 8 frames x
128x128, three updates: parameters 1e-2 apart, gradients of the last step more than 100 %): the atomic sums leave
the gradients of two runs a few 1e-8 apart, whatever the streams, and the untrained network amplifies such a
difference in the parameters from step to step -- two runs of the SAME setting drift apart like that."""
import os
import subprocess
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SCRIPT = r"""
import sys
sys.path.insert(0, %r); sys.path.insert(0, %r)
import numpy as np, torch
from paper_1910_00932_amd import binding as B
from paper_1910_00932_amd import inputs as I
fresh = sys.argv[3] == "fresh"
N, T, S = 2, 4, 64
bf = sys.argv[2] == "bf16"
table = B.tsm_resnet50_param_table(400)
flat = I.init_params([(n, s) for n, _, s, _ in table], 1)
desc = lambda lr: B.R50Desc(N=N, T=T, size=S, num_classes=400, fold_div=8, lr=lr, momentum=0.9, weight_decay=1e-4,
                            bn_eps=1e-5, bn_momentum=0.1, dtype=B.TSM_BF16 if bf else B.TSM_F32)
ws = torch.empty(B.tsm_resnet50_workspace_bytes(desc(0.0)), dtype=torch.uint8, device="cuda")
params = torch.from_numpy(flat).cuda(); mom = torch.zeros_like(params); grads = torch.empty_like(params)
loss = torch.zeros(1, dtype=torch.float32, device="cuda")
clips = [torch.from_numpy(I.clips(N, T, S, seed if fresh else 0, sys.argv[2])).to(torch.bfloat16 if bf else torch.float32).cuda()
         for seed in range(4)]
labels = torch.from_numpy(I.labels(N)).cuda()
for i, lr in enumerate((0.0, 0.0, 0.0, 0.01)):     # back to back, no synchronisation in between
    B.tsm_resnet50_step(desc(lr), clips[i], labels, params, mom, None, grads, loss, None, 1, ws)
torch.cuda.synchronize()
np.save(sys.argv[1], np.concatenate([params.cpu().numpy(), mom.cpu().numpy(), grads.cpu().numpy(), [float(loss.item())]]))
""" % (ROOT, os.path.join(ROOT, "tests"))


def _run(tmp_path, overlap, dtype, mode="same"):
    out = str(tmp_path / ("step_%s_%s_%s.npy" % (dtype, overlap, mode)))
    env = dict(os.environ, TSM_WGRAD_OVERLAP=overlap)
    subprocess.run([sys.executable, "-c", SCRIPT, out, dtype, mode], check=True, env=env, timeout=300)
    return np.load(out)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_one_stream_and_two_streams_agree(tmp_path, dtype):
    a, b = _run(tmp_path, "1", dtype), _run(tmp_path, "0", dtype)
    assert np.all(np.isfinite(a)) and np.all(np.isfinite(b))
    rel = np.linalg.norm(a - b) / np.linalg.norm(b)
    assert rel < 1e-5, rel


def test_one_stream_and_two_streams_agree_on_fresh_clips_every_step(tmp_path):
    a, b = _run(tmp_path, "1", "bf16", "fresh"), _run(tmp_path, "0", "bf16", "fresh")
    assert np.all(np.isfinite(a)) and np.all(np.isfinite(b))
    rel = np.linalg.norm(a - b) / np.linalg.norm(b)
    assert rel < 1e-5, rel
