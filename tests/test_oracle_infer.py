"""Pins of the oracle's inference-mode (forward-only) functions: what the mathematics fixes."""
import numpy as np

from oracle import tsm_oracle as O
from paper_1910_00932_amd import inputs as I


def test_bn_eval_closed_form_and_sign_conventions():
    # one channel, hand numbers: y=3, mean=1, var=3, eps=1 -> (3-1)/2 = 1; gamma 5, beta -2 -> 3
    y = np.full((1, 1, 1, 1, 1), 3.0)
    z = O.bn_eval(y, np.array([5.0]), np.array([-2.0]), np.array([1.0]), np.array([3.0]), eps=1.0)
    assert z.shape == y.shape and abs(z.item() - 3.0) < 1e-15
    # a larger variance shrinks the deviation from the mean, a larger mean lowers the output
    assert O.bn_eval(y, np.ones(1), np.zeros(1), np.array([1.0]), np.array([15.0]), eps=1.0).item() == 0.5
    assert O.bn_eval(y, np.ones(1), np.zeros(1), np.array([2.0]), np.array([3.0]), eps=1.0).item() == 0.5


def test_bn_eval_with_batch_statistics_equals_training_mode():
    rng = np.random.default_rng(0)
    y = rng.normal(size=(2, 3, 5, 4, 4)) * 2 + 1
    g, b = rng.normal(size=5), rng.normal(size=5)
    z, (yhat, rstd, mu, var) = O.bn_fwd(y, g, b, 1e-5)
    assert np.allclose(O.bn_eval(y, g, b, mu, var, 1e-5), z, rtol=0, atol=1e-12)
    # channels are independent: changing the statistics of channel 0 leaves the others alone
    mu2 = mu.copy(); mu2[0] += 1.0
    z2 = O.bn_eval(y, g, b, mu2, var, 1e-5)
    assert np.array_equal(z2[:, :, 1:], O.bn_eval(y, g, b, mu, var, 1e-5)[:, :, 1:]) and not np.allclose(z2[:, :, 0], z[:, :, 0])


def test_bn_eval_folds_into_the_convolution_weights():
    # inference-mode BN after a convolution is the convolution with weights scaled per output channel plus a bias
    rng = np.random.default_rng(1)
    x = rng.normal(size=(1, 2, 6, 5, 5))
    w = rng.normal(size=(4, 6, 3, 3))
    g, b, mu, var = rng.normal(size=4), rng.normal(size=4), rng.normal(size=4), rng.uniform(0.5, 2.0, size=4)
    scale = g / np.sqrt(var + 1e-5)
    folded = O.conv_fwd(x, w * scale[:, None, None, None], 1, 1, 0) + (b - mu * scale).reshape(1, 1, -1, 1, 1)
    assert np.allclose(O.bn_eval(O.conv_fwd(x, w, 1, 1, 0), g, b, mu, var, 1e-5), folded, rtol=0, atol=1e-11)


def test_bottleneck_infer_with_batch_statistics_equals_training_forward():
    for proj, stride, cin in ((False, 1, 16), (True, 2, 8)):
        rng = np.random.default_rng(2)
        p = {"w1": rng.normal(size=(4, cin, 1, 1)), "w2": rng.normal(size=(4, 4, 3, 3)), "w3": rng.normal(size=(16, 4, 1, 1))}
        for i, c in (("1", 4), ("2", 4), ("3", 16)):
            p["g" + i], p["b" + i] = rng.normal(size=c), rng.normal(size=c)
        if proj:
            p["wd"], p["gd"], p["bd"] = rng.normal(size=(16, cin, 1, 1)), rng.normal(size=16), rng.normal(size=16)
        x = rng.normal(size=(2, 4, cin, 6, 6))
        out, c = O.bottleneck_fwd(x, p, stride, 8, 1e-5)
        st = {"1": c["bn1"][2:], "2": c["bn2"][2:], "3": c["bn3"][2:]}
        if proj:
            st["d"] = c["bnd"][2:]
        assert np.allclose(O.bottleneck_infer(x, p, st, stride, 8, 1e-5), out, rtol=0, atol=1e-10)
        # with other statistics the result differs (the statistics are really used)
        st["2"] = (st["2"][0] + 0.5, st["2"][1])
        assert not np.allclose(O.bottleneck_infer(x, p, st, stride, 8, 1e-5), out)


def test_bn_state_layout_and_network_inference_shape():
    slots = O.bn_state_slots()
    assert len(slots) == 53 and slots[0] == ("bn1", 64) and slots[1] == ("res2.0.bn1", 64)
    assert slots[4] == ("res2.0.dsbn", 256) and slots[-1] == ("res5.2.bn3", 2048)
    assert O.bn_state_count() == 2 * 26560   # 26,560 BatchNorm channels in ResNet-50
    # tiny input through the whole network: statistics mean 0 / variance 1 make every BN the map gamma*y/sqrt(1+eps)+beta
    table = O.resnet50_param_table(10)
    P = O.unflatten_params(I.init_params([(n, s) for n, s, _ in table], 1).astype(np.float64), 10)
    state = np.concatenate([np.concatenate([np.zeros(c), np.ones(c)]) for _, c in slots])
    clips = I.clips(1, 2, 32, 0, "f32").astype(np.float64)
    logits = O.resnet50_infer(P, state, clips)
    assert logits.shape == (1, 10) and np.all(np.isfinite(logits))
    # a clip is classified independently of the other clips in the batch (no batch statistics are involved)
    two = np.concatenate([clips, I.clips(1, 2, 32, 5, "f32").astype(np.float64)])
    assert np.allclose(O.resnet50_infer(P, state, two)[0], logits[0], rtol=0, atol=1e-9)


def test_inference_with_recorded_batch_statistics_equals_training_forward():
    """Whole network: the statistics recorded by a training-mode forward, fed back as running statistics,
    make the inference path reproduce the training-mode logits (computed by the separate forward+backward
    routine through bn_fwd).  A BatchNorm wired to the wrong slot, a missing shortcut BN or a swapped
    mean/variance breaks this."""
    table = O.resnet50_param_table(10)
    flat = I.init_params([(n, s) for n, s, _ in table], 3).astype(np.float64)
    rng = np.random.default_rng(4)
    off = 0
    for name, shape, _ in table:      # distinct BatchNorm scales/offsets
        n = int(np.prod(shape))
        if len(shape) == 1 and name != "fc.b":
            flat[off:off + n] += 0.1 * rng.standard_normal(n)
        off += n
    P = O.unflatten_params(flat, 10)
    clips = I.clips(2, 2, 32, 0, "f32").astype(np.float64)
    state = O.resnet50_batch_stats(P, clips)
    assert state.shape == (O.bn_state_count(),)
    S = O.unflatten_bn_state(state)
    assert all(np.all(v > 0) for _, v in S.values())          # second half of every slot is a variance
    _, logits_train, _ = O.resnet50_fwd_bwd(P, clips, np.array([1, 2]))
    assert np.allclose(O.resnet50_infer(P, state, clips), logits_train, rtol=0, atol=1e-9)
    # and the statistics matter: perturbing one variance changes the logits
    state2 = state.copy()
    state2[64:128] *= 4.0
    assert not np.allclose(O.resnet50_infer(P, state2, clips), logits_train, atol=1e-6)
