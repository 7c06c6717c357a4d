"""The backward entry points run their weight gradients on a second stream; TSM_WGRAD_OVERLAP=0 keeps one stream.
Both settings must give the same step (the switch is read once per process, so each setting runs in a process
of its own; results differ only by the order of the atomic sums of the weight gradients)."""
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
N, T, S = 2, 4, 64
table = B.tsm_resnet50_param_table(400)
flat = I.init_params([(n, s) for n, _, s, _ in table], 1)
d = B.R50Desc(N=N, T=T, size=S, num_classes=400, fold_div=8, lr=0.01, momentum=0.9, weight_decay=1e-4, bn_eps=1e-5,
              bn_momentum=0.1, dtype=B.TSM_BF16)
ws = torch.empty(B.tsm_resnet50_workspace_bytes(d), dtype=torch.uint8, device="cuda")
params = torch.from_numpy(flat).cuda(); mom = torch.zeros_like(params); grads = torch.empty_like(params)
loss = torch.zeros(1, dtype=torch.float32, device="cuda")
clips = torch.from_numpy(I.clips(N, T, S, 0, "bf16")).to(torch.bfloat16).cuda()
labels = torch.from_numpy(I.labels(N)).cuda()
for _ in range(3):     # three updates: any race between the streams would show in the parameters
    B.tsm_resnet50_step(d, clips, labels, params, mom, None, grads, loss, None, 1, ws)
torch.cuda.synchronize()
np.save(sys.argv[1], np.concatenate([params.cpu().numpy(), grads.cpu().numpy(), [float(loss.item())]]))
""" % (ROOT, os.path.join(ROOT, "tests"))


def _run(tmp_path, overlap):
    out = str(tmp_path / ("step_%s.npy" % overlap))
    env = dict(os.environ, TSM_WGRAD_OVERLAP=overlap)
    subprocess.run([sys.executable, "-c", SCRIPT, out], check=True, env=env, timeout=300)
    return np.load(out)


def test_one_stream_and_two_streams_agree(tmp_path):
    a, b = _run(tmp_path, "1"), _run(tmp_path, "0")
    assert np.all(np.isfinite(a)) and np.all(np.isfinite(b))
    rel = np.linalg.norm(a - b) / np.linalg.norm(b)
    assert rel < 1e-5, rel
