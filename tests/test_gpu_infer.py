"""Parity of tsm_resnet50_infer (forward only, BatchNorm with running statistics; the configuration the
paper's throughput table measures, section 3a / Table 1) with the oracle's inference forward."""
import numpy as np
import pytest
import torch

from oracle import tsm_oracle as O
from paper_1910_00932_amd import binding as B
from paper_1910_00932_amd import inputs as I
from conftest import rel_l2
from gpu_util import workspace

pytestmark = pytest.mark.gpu


def setup(N, T, S, dtype, seed=1, K=400, g3=1.0):
    table = B.tsm_resnet50_param_table(K)
    flat = I.init_params([(n, s) for n, _, s, _ in table], seed)
    rng = np.random.default_rng(5)
    for name, off, shape, _ in table:      # make every BatchNorm scale/offset distinct
        if len(shape) == 1 and name != "fc.b":
            n = shape[0]
            flat[off:off + n] += (0.1 * rng.standard_normal(n)).astype(np.float32)
            if name.endswith("bn3.g"):     # scale of the residual branch
                flat[off:off + n] *= g3
    clips = I.clips(N, T, S, 0, dtype)
    P = O.unflatten_params(flat.astype(np.float64), K)
    # running statistics: what a training-mode forward over a different seeded batch records (oracle only),
    # so they are realistic for the network but not the statistics of the batch under test
    calib = I.clips(2, T, S, 9, "f32").astype(np.float64)
    state = O.resnet50_batch_stats(P, calib).astype(np.float32)
    return table, flat, clips, P, state


def run_infer(N, T, S, dtype, flat, clips, state, K=400, fold_div=8):
    d = B.R50Desc(N=N, T=T, size=S, num_classes=K, fold_div=fold_div, lr=0.0, momentum=0.9, weight_decay=1e-4,
                  bn_eps=1e-5, bn_momentum=0.1, dtype=B.TSM_BF16 if dtype == "bf16" else B.TSM_F32)
    ws = workspace(B.tsm_resnet50_infer_workspace_bytes(d))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    logits = torch.empty((N, K), dtype=torch.float32, device="cuda")
    B.tsm_resnet50_infer(d, torch.from_numpy(clips).to(tdt).cuda(), torch.from_numpy(flat).cuda(),
                         torch.from_numpy(state).cuda(), logits, ws)
    torch.cuda.synchronize()
    return logits.cpu().numpy()


def test_infer_fp32_against_oracle():
    """fp32 storage, plain kernels: every layer's wiring, BatchNorm slots and the head, to 1e-4."""
    N, T, S = 2, 4, 64
    table, flat, clips, P, state = setup(N, T, S, "f32")
    got = run_infer(N, T, S, "f32", flat, clips, state)
    ref = O.resnet50_infer(P, state.astype(np.float64), clips.astype(np.float64))
    assert rel_l2(got, ref) < 1e-4, rel_l2(got, ref)


def test_infer_bf16_against_oracle():
    """bf16 storage with the BatchNorm / shortcut / ReLU epilogues fused into the MFMA convolutions.
    Reference: the oracle with bf16-rounded weights and stored activations, to 2e-2 relative L2 on the logits.
    With fixed statistics nothing re-normalises the activations, so an untrained network with unit residual
    scales amplifies every rounding (the oracle's own logits move by 13% when its tensors are rounded to
    bf16); the residual branches are therefore scaled by 0.25 (last BatchNorm of each block), where that
    sensitivity is 1.6%, and the bound is 2e-2 or 1.5x the sensitivity, whichever is larger."""
    N, T, S = 2, 4, 64
    table, flat, clips, P, state = setup(N, T, S, "bf16", g3=0.25)
    got = run_infer(N, T, S, "bf16", flat, clips, state)
    c64, s64 = clips.astype(np.float64), state.astype(np.float64)
    refq = O.resnet50_infer(P, s64, c64, q=O.round_bf16, wq=O.round_bf16)
    ref = O.resnet50_infer(P, s64, c64)
    sens = rel_l2(refq, ref)
    errs = (rel_l2(got, refq), rel_l2(got, ref), sens)
    print("bf16 inference: logits err %.4f vs bf16 oracle, %.4f vs fp64 oracle (sens %.4f)" % errs)
    bound = max(2e-2, 1.5 * sens)
    assert errs[0] < bound and errs[1] < bound, errs


def test_infer_is_independent_of_the_batch_and_differs_from_training_statistics():
    """A clip's logits do not depend on the other clips of the batch (no batch statistics) beyond the
    accumulation order of differently sized launches; ragged sizes (N=3, T=3) go through the same kernels."""
    T, S = 3, 32
    table, flat, clips, P, state = setup(3, T, S, "bf16", g3=0.25)
    all3 = run_infer(3, T, S, "bf16", flat, clips, state)
    one = run_infer(1, T, S, "bf16", flat, clips[1:2], state)
    assert rel_l2(all3[1:2], one) < 2e-3, rel_l2(all3[1:2], one)
    ref = O.resnet50_infer(P, state.astype(np.float64), clips.astype(np.float64), q=O.round_bf16, wq=O.round_bf16)
    assert rel_l2(all3, ref) < 3e-2, rel_l2(all3, ref)


def test_infer_rejects_bad_arguments():
    table, flat, clips, P, state = setup(1, 2, 32, "bf16")
    d = B.R50Desc(N=1, T=2, size=32, num_classes=400, fold_div=8, lr=0.0, momentum=0.9, weight_decay=1e-4,
                  bn_eps=1e-5, bn_momentum=0.1, dtype=B.TSM_BF16)
    logits = torch.empty((1, 400), dtype=torch.float32, device="cuda")
    x = torch.from_numpy(clips).to(torch.bfloat16).cuda()
    p, st = torch.from_numpy(flat).cuda(), torch.from_numpy(state).cuda()
    with pytest.raises(B.TsmError):      # workspace too small
        B.tsm_resnet50_infer(d, x, p, st, logits, workspace(1024))
    with pytest.raises(B.TsmError):      # running statistics are required
        B.tsm_resnet50_infer(d, x, p, None, logits, workspace(B.tsm_resnet50_infer_workspace_bytes(d)))
    bad = B.R50Desc(N=1, T=2, size=40, num_classes=400, fold_div=8, lr=0.0, momentum=0.9, weight_decay=1e-4,
                    bn_eps=1e-5, bn_momentum=0.1, dtype=B.TSM_BF16)
    assert B.tsm_resnet50_infer_workspace_bytes(bad) == 0


def test_infer_full_size_batch16_sampled_clips():
    """The benchmark's launch configuration (16 clips x 8 frames x 224x224, bf16): inference is independent per
    clip, so the logits of two of the sixteen clips are checked against the oracle run on those two clips alone."""
    N, T, S = 16, 8, 224
    table, flat, clips2, P, state = setup(2, T, S, "bf16", g3=0.25)
    clips = np.concatenate([clips2[0:1]] + [I.clips(1, T, S, 20 + i, "bf16") for i in range(N - 2)] + [clips2[1:2]])
    got = run_infer(N, T, S, "bf16", flat, clips, state)
    assert np.all(np.isfinite(got))
    c64, s64 = clips2.astype(np.float64), state.astype(np.float64)
    refq = O.resnet50_infer(P, s64, c64, q=O.round_bf16, wq=O.round_bf16)
    ref = O.resnet50_infer(P, s64, c64)
    sens = rel_l2(refq, ref)
    pick = got[[0, N - 1]]
    errs = (rel_l2(pick, refq), rel_l2(pick, ref), sens)
    print("bf16 inference at batch 16, 224x224: err %.4f vs bf16 oracle, %.4f vs fp64 oracle (sens %.4f)" % errs)
    bound = max(2e-2, 1.5 * sens)
    assert errs[0] < bound and errs[1] < bound, errs


def test_infer_batch_64_agrees_with_batch_16_clip_by_clip():
    """Inference is independent per clip (fixed statistics), so a batch of 64 made of a batch of 16 four times over
    must give four bit-identical copies of the logits, wherever the clips fall in the tiles of the larger launch,
    and those must agree with the batch-16 call (which the test above holds to the oracle) up to the different
    tile choices the library makes at the two sizes (bf16 storage at the same points; different summation order
    inside a layer only where a different kernel takes it)."""
    T, S = 8, 224
    table, flat, clips2, P, state = setup(2, T, S, "bf16", g3=0.25)
    clips16 = np.concatenate([clips2] + [I.clips(1, T, S, 20 + i, "bf16") for i in range(14)])
    l16 = run_infer(16, T, S, "bf16", flat, clips16, state)
    l64 = run_infer(64, T, S, "bf16", flat, np.tile(clips16, (4, 1, 1, 1, 1)), state).reshape(4, 16, -1)
    assert np.array_equal(l64, np.broadcast_to(l64[0], l64.shape)), "logits differ between copies of a clip"
    err = rel_l2(l64[0], l16)
    print("bf16 inference, batch 64 against batch 16: %.1e" % err)
    assert err < 5e-3, err


def test_infer_replays_from_a_hip_graph():
    """The call is stream-ordered and allocates nothing, so it can be recorded into a HIP graph; every replay,
    with eager work and synchronisation in between, reproduces the eager logits bit for bit (the forward path
    has no atomics)."""
    N, T, S = 2, 4, 64
    table, flat, clips, P, state = setup(N, T, S, "bf16", g3=0.25)
    d = B.R50Desc(N=N, T=T, size=S, num_classes=400, fold_div=8, lr=0.0, momentum=0.9, weight_decay=1e-4,
                  bn_eps=1e-5, bn_momentum=0.1, dtype=B.TSM_BF16)
    ws = workspace(B.tsm_resnet50_infer_workspace_bytes(d))
    x = torch.from_numpy(clips).to(torch.bfloat16).cuda()
    p, st = torch.from_numpy(flat).cuda(), torch.from_numpy(state).cuda()
    logits = torch.empty((N, 400), dtype=torch.float32, device="cuda")
    B.tsm_resnet50_infer(d, x, p, st, logits, ws)
    torch.cuda.synchronize()
    eager = logits.cpu().numpy().copy()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.tsm_resnet50_infer(d, x, p, st, logits, ws, torch.cuda.current_stream())
    for i in range(3):
        logits.fill_(float(i))          # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(logits.cpu().numpy(), eager), i
    x2 = torch.from_numpy(I.clips(N, T, S, 7, "bf16")).to(torch.bfloat16).cuda()
    x.copy_(x2)                          # new input in the same buffer: the replay follows it
    g.replay()
    torch.cuda.synchronize()
    replayed = logits.cpu().numpy().copy()
    B.tsm_resnet50_infer(d, x, p, st, logits, ws)
    torch.cuda.synchronize()
    assert np.array_equal(logits.cpu().numpy(), replayed)
    assert not np.array_equal(replayed, eager)
