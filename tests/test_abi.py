"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol declared in include/tsm.h, and rejects bad arguments before launching."""
import ctypes
import os
import re

import pytest

from paper_1910_00932_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "tsm.h")).read()
    declared = set(re.findall(r"\b(tsm_[a-z0-9_]+)\s*\(", hdr))
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(B.EXPORTS)


def _conv_desc(**kw):
    d = B.ConvDesc(N=1, T=2, Cin=8, H=4, W=4, Cout=8, kh=3, kw=3, stride=1, pad=1, fold_div=8, dtype=B.TSM_F32,
                   layout=B.TSM_NTHWC)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_shift_argument_errors():
    L = B.lib()
    a = 4096   # fake, aligned, never dereferenced: argument checks come first
    assert L.tsm_shift_fwd(None, a, 1, 2, 8, 2, 2, 8, 0, 1, None) == -1
    assert L.tsm_shift_fwd(a, a + 65536, 1, 0, 8, 2, 2, 8, 0, 1, None) == -2
    assert L.tsm_shift_fwd(a, a + 65536, 1, 2, 8, 2, 2, 1, 0, 1, None) == -3
    assert L.tsm_shift_fwd(a, a + 65536, 1, 2, 8, 2, 2, -2, 0, 1, None) == -3
    assert L.tsm_shift_fwd(a, a + 65536, 1, 2, 8, 2, 2, 8, 7, 1, None) == -4
    assert L.tsm_shift_fwd(a, a + 65536, 1, 2, 8, 2, 2, 8, 0, 5, None) == -5
    assert L.tsm_shift_fwd(a + 2, a + 65536, 1, 2, 8, 2, 2, 8, 0, 1, None) == -7
    assert L.tsm_shift_bwd(a, a + 16, 1, 2, 8, 2, 2, 8, 0, 1, None) == -2     # overlap
    assert "overlap" in B.tsm_last_error()


def test_probe_argument_errors():
    L = B.lib()
    flops = ctypes.c_double(0.0)
    assert L.tsm_mfma_probe(0, 4096, ctypes.byref(flops), None) == -2
    assert L.tsm_mfma_probe(10, None, ctypes.byref(flops), None) == -1
    assert L.tsm_mfma_probe(10, 4096, None, None) == -1


def test_conv_argument_errors():
    L = B.lib()
    a = 4096
    d = _conv_desc()
    need = B.tsm_conv_workspace_bytes(d)
    assert need > 0
    assert L.tsm_conv_fwd(ctypes.addressof(d), None, a, a, None, None, a, need, None) == -1
    assert L.tsm_conv_fwd(None, a, a, a, None, None, a, need, None) == -1
    # an empty workspace is below the forward requirement of every descriptor (the statistics rows alone need some)
    assert L.tsm_conv_fwd(ctypes.addressof(d), a, a, a, None, None, a, 0, None) == -6
    d2 = _conv_desc(T=0)
    assert L.tsm_conv_fwd(ctypes.addressof(d2), a, a, a, None, None, a, 1 << 20, None) == -2
    d3 = _conv_desc(fold_div=1)
    assert L.tsm_conv_dgrad(ctypes.addressof(d3), a, a, a, a, 1 << 20, None) == -3
    d4 = _conv_desc(dtype=9)
    assert L.tsm_conv_wgrad(ctypes.addressof(d4), a, a, a, 0, a, 1 << 20, None) == -4
    d5 = _conv_desc(layout=B.TSM_NTCHW)
    need5 = B.tsm_conv_workspace_bytes(d5)
    assert need5 > 0
    assert L.tsm_conv_fwd(ctypes.addressof(d5), a, a, a, None, None, a, need5 - 1, None) == -6
    assert L.tsm_conv_fwd(ctypes.addressof(d5), a, a + 4, a, None, None, a, need5, None) == -7
    assert L.tsm_conv_fwd(ctypes.addressof(d5), a, a, a, a, None, a, need5, None) == -1   # only one stats pointer


def test_block_argument_errors():
    L = B.lib()
    a = 4096
    d = B.BlockDesc(kind=B.TSM_BLOCK_BOTTLENECK, N=1, T=2, Cin=16, H=4, W=4, Cmid=8, Cout=16, stride=1,
                    has_projection=0, fold_div=8, dtype=B.TSM_BF16, layout=B.TSM_NTHWC, bn_eps=1e-5)
    assert B.tsm_block_saved_bytes(d) > 0 and B.tsm_block_workspace_bytes(d) > 0
    ps = B.BlockParams()
    assert L.tsm_block_fwd(ctypes.addressof(d), a, ctypes.addressof(ps), a, a, a, 1 << 24, None) == -1   # null weights
    d.Cout = 32   # identity shortcut with Cout != Cin
    assert B.tsm_block_saved_bytes(d) == 0
    assert L.tsm_block_fwd(ctypes.addressof(d), a, ctypes.addressof(ps), a, a, a, 1 << 24, None) == -2
    d.kind = 7
    assert L.tsm_block_fwd(ctypes.addressof(d), a, ctypes.addressof(ps), a, a, a, 1 << 24, None) == -9


def _r50_desc(**kw):
    v = dict(N=1, T=2, size=32, num_classes=10, fold_div=8, lr=0.01, momentum=0.9, weight_decay=1e-4, bn_eps=1e-5,
             bn_momentum=0.1, dtype=B.TSM_BF16)
    v.update(kw)
    return B.R50Desc(**v)


def test_network_entry_points_argument_errors():
    """Argument checks of the whole-network entry points come before any GPU work."""
    L = B.lib()
    a = 4096   # fake, aligned, never dereferenced
    d = _r50_desc()
    need_step, need_inf = B.tsm_resnet50_workspace_bytes(d), B.tsm_resnet50_infer_workspace_bytes(d)
    assert need_step > need_inf > 0
    da = ctypes.addressof(d)
    assert L.tsm_resnet50_infer(None, a, a, a, a, a, need_inf, None) == -1
    assert L.tsm_resnet50_infer(da, a, a, None, a, a, need_inf, None) == -1            # running statistics required
    assert L.tsm_resnet50_infer(da, a, a, a, a, a, need_inf - 1, None) == -6
    assert "workspace" in B.tsm_last_error()
    assert L.tsm_resnet50_infer(da, a + 4, a, a, a, a, need_inf, None) == -7
    for bad in (_r50_desc(size=40), _r50_desc(N=0), _r50_desc(fold_div=1), _r50_desc(dtype=5)):
        assert B.tsm_resnet50_infer_workspace_bytes(bad) == 0 and B.tsm_resnet50_workspace_bytes(bad) == 0
    assert L.tsm_resnet50_step(da, a, a, a, a, None, None, a, None, 1, a, need_step - 1, None) == -6
    assert L.tsm_resnet50_step(da, a, None, a, a, None, None, a, None, 1, a, need_step, None) == -1
    assert L.tsm_resnet50_accum_step(da, a, a, a, a, None, a, a, None, 2, 2, a, need_step, None) == -2  # index out of range
    assert L.tsm_resnet50_accum_step(da, a, a, a, a, None, None, a, None, 0, 2, a, need_step, None) == -1
    assert L.tsm_resnet50_accum_step(da, a, a, a, a, None, a + 4, a, None, 0, 2, a, need_step, None) == -7


def test_workspace_plan_switches_kernels_at_2_gib():
    """The general forward kernel addresses its tensors with 32-bit byte offsets; tensors of 2 GiB and more go to
    the register-prefetch kernel, which runs two blocks of 128-row tiles per compute unit instead of one block of
    256-row tiles.  The workspace plan shows the switch: the statistics epilogue gets one row per block."""
    def stats_rows(N):
        d = B.ConvDesc(N=N, T=8, Cin=64, H=112, W=112, Cout=64, kh=1, kw=1, stride=1, pad=0, fold_div=8,
                       dtype=B.TSM_BF16, layout=B.TSM_NTHWC)
        need = B.tsm_conv_workspace_bytes(d)
        packed = 64 * 64 * 2                      # bf16 working copy of the weights (a multiple of 256 bytes)
        rows, rem = divmod(need - packed, 2 * 64 * 4)
        assert rem == 0
        return N * 8 * 112 * 112 * 64 * 2, rows
    below, rows_below = stats_rows(166)
    above, rows_above = stats_rows(168)
    assert below < 0x7ff00000 <= above
    assert rows_above == 2 * rows_below and rows_below % 8 == 0


def test_block_infer_argument_errors():
    L = B.lib()
    a = 4096
    d = B.BlockDesc(kind=B.TSM_BLOCK_BOTTLENECK, N=1, T=2, Cin=16, H=4, W=4, Cmid=8, Cout=16, stride=1,
                    has_projection=0, fold_div=8, dtype=B.TSM_F32, layout=B.TSM_NTHWC, bn_eps=1e-5)
    need = B.tsm_block_infer_workspace_bytes(d)
    assert need > 0
    ps, ss = B.BlockParams(), B.BlockStats()
    for n, _ in B.BlockParams._fields_:
        setattr(ps, n, a)
    for n, _ in B.BlockStats._fields_:
        setattr(ss, n, a)
    args = lambda **kw: [kw.get("d", ctypes.addressof(d)), kw.get("x", a), kw.get("p", ctypes.addressof(ps)),
                         kw.get("s", ctypes.addressof(ss)), kw.get("out", a), a, kw.get("n", need), None]
    assert L.tsm_block_infer(*args(x=None)) == -1
    assert L.tsm_block_infer(*args(p=None)) == -1
    assert L.tsm_block_infer(*args(s=None)) == -1
    assert L.tsm_block_infer(*args(n=need - 1)) == -6
    assert L.tsm_block_infer(*args(out=a + 8)) == -7
    ss.m2 = None
    assert L.tsm_block_infer(*args()) == -1 and "statistics" in B.tsm_last_error()
    bad = B.BlockDesc(kind=B.TSM_BLOCK_BOTTLENECK, N=1, T=2, Cin=16, H=4, W=4, Cmid=8, Cout=32, stride=1,
                      has_projection=0, fold_div=8, dtype=B.TSM_F32, layout=B.TSM_NTHWC, bn_eps=1e-5)
    assert B.tsm_block_infer_workspace_bytes(bad) == 0
