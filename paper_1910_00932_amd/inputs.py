"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method itself: only random tensors with the shapes and
value distributions of the workloads (Kinetics-shaped clips of 8 frames of
3x224x224, 400 classes; section 4.1 and Table 1 of the paper), which stand in
for the dataset.  Seeds: 0 inputs, 1 weights, 2 labels, 3 upstream gradients.
"""
import numpy as np
import torch


def bf16_grid(a):
    """Round a float array once, on the host, to values representable in bf16."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def _finish(a, dtype):
    a = a.astype(np.float32)
    return bf16_grid(a) if dtype == "bf16" else a


def normal(shape, seed, dtype="f32", scale=1.0):
    rng = np.random.default_rng(seed)
    return _finish(rng.standard_normal(shape) * scale, dtype)


def kaiming_conv(shape, seed, dtype="f32"):
    """N(0, 2/fan_out), fan_out = Cout * (kernel volume); shape [Cout, Cin, k...]."""
    fan_out = shape[0] * int(np.prod(shape[2:]))
    return normal(shape, seed, dtype, np.sqrt(2.0 / fan_out))


def clips(N, T, size, seed=0, dtype="bf16"):
    """Pixels u ~ U[0,1], normalised as (u - 0.5) / 0.25; layout [N,T,3,size,size]."""
    rng = np.random.default_rng(seed)
    u = rng.random((N, T, 3, size, size), dtype=np.float32)
    return _finish((u - 0.5) / 0.25, dtype)


def labels(N, num_classes=400, seed=2):
    rng = np.random.default_rng(seed)
    return rng.integers(0, num_classes, size=N).astype(np.int32)


def init_params(table, seed=1, fc_std=0.01):
    """Flat fp32 parameter vector for a (name, shape, ...) table: convolutions
    Kaiming-normal (fan-out), the linear head N(0, fc_std^2), scale parameters
    (names ending in '.g') 1, every other 1-d parameter 0."""
    rng = np.random.default_rng(seed)
    parts = []
    for entry in table:
        name, shape = entry[0], tuple(entry[1])
        n = int(np.prod(shape))
        if len(shape) >= 3:
            fan_out = shape[0] * int(np.prod(shape[2:]))
            v = rng.standard_normal(n) * np.sqrt(2.0 / fan_out)
        elif len(shape) == 2:
            v = rng.standard_normal(n) * fc_std
        elif name.endswith(".g"):
            v = np.ones(n)
        else:
            v = np.zeros(n)
        parts.append(v.astype(np.float32))
    return np.concatenate(parts)
