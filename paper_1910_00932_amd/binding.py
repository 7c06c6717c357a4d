"""ctypes binding of libtsm_hip.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
``include/tsm.h``.  Tensor arguments are torch CUDA tensors (device memory and
streams are all PyTorch is used for) or ``None`` for optional pointers; nothing
is computed in Python.  A missing library is an error, never a fallback."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtsm_hip.so")

TSM_F32, TSM_BF16 = 0, 1
TSM_NTCHW, TSM_NTHWC = 0, 1
TSM_BLOCK_BASIC, TSM_BLOCK_BOTTLENECK, TSM_BLOCK_BOTTLENECK_T3 = 0, 1, 2

STATUS = {0: "TSM_OK", -1: "TSM_ERR_NULLPTR", -2: "TSM_ERR_SHAPE", -3: "TSM_ERR_FOLD", -4: "TSM_ERR_DTYPE",
          -5: "TSM_ERR_LAYOUT", -6: "TSM_ERR_WORKSPACE", -7: "TSM_ERR_ALIGN", -8: "TSM_ERR_LAUNCH",
          -9: "TSM_ERR_UNSUPPORTED"}

EXPORTS = ["tsm_last_error", "tsm_profile_begin", "tsm_profile_end", "tsm_mfma_probe", "tsm_shift_fwd", "tsm_shift_bwd", "tsm_conv_workspace_bytes", "tsm_conv_fwd",
           "tsm_conv_fwd_noalloc",
           "tsm_conv_dgrad", "tsm_conv_wgrad", "tsm_block_saved_bytes", "tsm_block_workspace_bytes",
           "tsm_block_fwd", "tsm_block_bwd", "tsm_block_infer_workspace_bytes", "tsm_block_infer", "tsm_resnet50_param_count", "tsm_resnet50_num_tensors",
           "tsm_resnet50_param_info", "tsm_resnet50_bn_state_count", "tsm_resnet50_workspace_bytes",
           "tsm_resnet50_step", "tsm_resnet50_workspace_tensor", "tsm_resnet50_infer_workspace_bytes", "tsm_resnet50_infer",
           "tsm_resnet50_accum_step", "tsm_lr_schedule"]


class TsmError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("%s (%d): %s" % (STATUS.get(code, "?"), code, msg))
        self.code = code


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("N", "T", "Cin", "H", "W", "Cout", "kh", "kw", "stride", "pad", "fold_div", "dtype", "layout")]


class BlockDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("kind", "N", "T", "Cin", "H", "W", "Cmid", "Cout", "stride", "has_projection", "fold_div", "dtype",
                 "layout")] + [("bn_eps", ctypes.c_float)]


class BlockParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("w1", "w2", "w3", "wd", "g1", "b1", "g2", "b2", "g3", "b3", "gd", "bd")]


class BlockGrads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("dw1", "dw2", "dw3", "dwd", "dg1", "db1", "dg2", "db2", "dg3", "db3", "dgd", "dbd")]


class BlockStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("m1", "v1", "m2", "v2", "m3", "v3", "md", "vd")]


class R50Desc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int), ("T", ctypes.c_int), ("size", ctypes.c_int), ("num_classes", ctypes.c_int),
                ("fold_div", ctypes.c_int), ("lr", ctypes.c_float), ("momentum", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("bn_eps", ctypes.c_float), ("bn_momentum", ctypes.c_float),
                ("dtype", ctypes.c_int)]


_LIB = None


def lib():
    """Loads the HIP library; raises if it has not been built."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libtsm_hip.so is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        def sig(name, restype, argtypes):
            fn = getattr(L, name, None)     # a symbol that is missing fails when it is called
            if fn is not None:
                fn.restype = restype
                if argtypes is not None:
                    fn.argtypes = argtypes

        vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        sig("tsm_last_error", ctypes.c_char_p, [])
        sig("tsm_profile_begin", ci, [vp])
        sig("tsm_profile_end", ci, [ctypes.c_char_p, sz])
        sig("tsm_mfma_probe", ci, [ci, vp, ctypes.POINTER(ctypes.c_double), vp])
        for n in ("tsm_conv_workspace_bytes", "tsm_block_saved_bytes", "tsm_block_workspace_bytes", "tsm_block_infer_workspace_bytes",
                  "tsm_resnet50_workspace_bytes", "tsm_resnet50_infer_workspace_bytes"):
            sig(n, sz, [vp])
        sig("tsm_resnet50_param_count", ctypes.c_int64, [ci])
        sig("tsm_resnet50_num_tensors", ci, [])
        sig("tsm_resnet50_bn_state_count", ctypes.c_int64, [])
        sig("tsm_shift_fwd", ci, [vp, vp] + [ci] * 8 + [vp])
        sig("tsm_shift_bwd", ci, [vp, vp] + [ci] * 8 + [vp])
        sig("tsm_conv_fwd", ci, [vp, vp, vp, vp, vp, vp, vp, sz, vp])
        sig("tsm_conv_fwd_noalloc", ci, [vp, vp, vp, vp, vp, vp, vp])
        sig("tsm_conv_dgrad", ci, [vp, vp, vp, vp, vp, sz, vp])
        sig("tsm_conv_wgrad", ci, [vp, vp, vp, vp, ci, vp, sz, vp])
        sig("tsm_block_fwd", ci, [vp, vp, vp, vp, vp, vp, sz, vp])
        sig("tsm_block_infer", ci, [vp, vp, vp, vp, vp, vp, sz, vp])
        sig("tsm_block_bwd", ci, [vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp])
        sig("tsm_resnet50_param_info", ci, [ci, ci, ctypes.c_char_p, ci, ctypes.POINTER(ctypes.c_int64),
                                            ctypes.POINTER(ci), ctypes.POINTER(ci * 4), ctypes.POINTER(ci)])
        sig("tsm_resnet50_step", ci, [vp, vp, vp, vp, vp, vp, vp, vp, vp, ci, vp, sz, vp])
        sig("tsm_resnet50_workspace_tensor", ci, [vp, ctypes.c_char_p, ctypes.POINTER(sz), ctypes.POINTER(ci * 4),
                                                  ctypes.POINTER(ci)])
        sig("tsm_resnet50_infer", ci, [vp, vp, vp, vp, vp, vp, sz, vp])
        sig("tsm_resnet50_accum_step", ci, [vp, vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, vp, sz, vp])
        sig("tsm_lr_schedule", ctypes.c_double, [ctypes.c_double, ci, ci, ctypes.c_double, ctypes.c_double])
        _LIB = L
    return _LIB


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("expected a CUDA tensor")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else stream


def _check(rc):
    if rc != 0:
        raise TsmError(rc, lib().tsm_last_error().decode())


def _ws(ws):
    return (_ptr(ws), ws.numel() * ws.element_size()) if ws is not None else (None, 0)


def tsm_last_error():
    return lib().tsm_last_error().decode()


def tsm_profile_begin(stream=None):
    _check(lib().tsm_profile_begin(_stream(stream)))


def tsm_mfma_probe(iters, sink, stream=None):
    """Launches the register-only MFMA kernel; returns the floating-point operations of the launch."""
    flops = ctypes.c_double(0.0)
    _check(lib().tsm_mfma_probe(int(iters), _ptr(sink), ctypes.byref(flops), _stream(stream)))
    return flops.value


def tsm_profile_end():
    """Returns {kernel class: (launches, total_ms)}."""
    buf = ctypes.create_string_buffer(1 << 16)
    _check(lib().tsm_profile_end(buf, len(buf)))
    out = {}
    for line in buf.value.decode().splitlines():
        name, n, ms = line.rsplit(" ", 2)
        out[name] = (int(n), float(ms))
    return out


def tsm_shift_fwd(x, y, N, T, C, H, W, fold_div, dtype, layout, stream=None):
    _check(lib().tsm_shift_fwd(_ptr(x), _ptr(y), N, T, C, H, W, fold_div, dtype, layout, _stream(stream)))


def tsm_shift_bwd(gy, gx, N, T, C, H, W, fold_div, dtype, layout, stream=None):
    _check(lib().tsm_shift_bwd(_ptr(gy), _ptr(gx), N, T, C, H, W, fold_div, dtype, layout, _stream(stream)))


def tsm_conv_workspace_bytes(desc):
    return int(lib().tsm_conv_workspace_bytes(ctypes.addressof(desc)))


def tsm_conv_fwd(desc, x, w, y, ch_sum, ch_sumsq, ws, stream=None):
    p, n = _ws(ws)
    _check(lib().tsm_conv_fwd(ctypes.addressof(desc), _ptr(x), _ptr(w), _ptr(y), _ptr(ch_sum), _ptr(ch_sumsq), p, n,
                              _stream(stream)))


NOALLOC_SCRATCH_BYTES = 16 << 20   # TSM_NOALLOC_SCRATCH_BYTES of include/tsm.h


def tsm_conv_fwd_noalloc(desc, x, w, y, ch_sum, ch_sumsq, stream=None):
    _check(lib().tsm_conv_fwd_noalloc(ctypes.addressof(desc), _ptr(x), _ptr(w), _ptr(y), _ptr(ch_sum), _ptr(ch_sumsq),
                                      _stream(stream)))


def tsm_conv_dgrad(desc, dy, w, dx, ws, stream=None):
    p, n = _ws(ws)
    _check(lib().tsm_conv_dgrad(ctypes.addressof(desc), _ptr(dy), _ptr(w), _ptr(dx), p, n, _stream(stream)))


def tsm_conv_wgrad(desc, x, dy, dw, accumulate, ws, stream=None):
    p, n = _ws(ws)
    _check(lib().tsm_conv_wgrad(ctypes.addressof(desc), _ptr(x), _ptr(dy), _ptr(dw), int(accumulate), p, n,
                                _stream(stream)))


def tsm_block_saved_bytes(desc):
    return int(lib().tsm_block_saved_bytes(ctypes.addressof(desc)))


def tsm_block_workspace_bytes(desc):
    return int(lib().tsm_block_workspace_bytes(ctypes.addressof(desc)))


def _fill_struct(cls, tensors):
    s = cls()
    for name, _ in cls._fields_:
        setattr(s, name, _ptr(tensors.get(name)))
    return s


def tsm_block_fwd(desc, x, params, out, saved, ws, stream=None):
    """params: dict field name -> tensor (fields of tsm_block_params)."""
    ps = _fill_struct(BlockParams, params)
    p, n = _ws(ws)
    _check(lib().tsm_block_fwd(ctypes.addressof(desc), _ptr(x), ctypes.addressof(ps), _ptr(out), _ptr(saved), p, n,
                               _stream(stream)))


def tsm_block_infer_workspace_bytes(desc):
    return int(lib().tsm_block_infer_workspace_bytes(ctypes.addressof(desc)))


def tsm_block_infer(desc, x, params, stats, out, ws, stream=None):
    """params: dict of tsm_block_params fields; stats: dict of tsm_block_stats fields (m1, v1, ...)."""
    ps = _fill_struct(BlockParams, params)
    ss = _fill_struct(BlockStats, stats)
    p, n = _ws(ws)
    _check(lib().tsm_block_infer(ctypes.addressof(desc), _ptr(x), ctypes.addressof(ps), ctypes.addressof(ss), _ptr(out), p, n,
                                 _stream(stream)))


def tsm_block_bwd(desc, x, out, dout, saved, params, dx, grads, ws, stream=None):
    ps = _fill_struct(BlockParams, params)
    gs = _fill_struct(BlockGrads, grads)
    p, n = _ws(ws)
    _check(lib().tsm_block_bwd(ctypes.addressof(desc), _ptr(x), _ptr(out), _ptr(dout), _ptr(saved),
                               ctypes.addressof(ps), _ptr(dx), ctypes.addressof(gs), p, n, _stream(stream)))


def tsm_resnet50_param_count(num_classes=400):
    return int(lib().tsm_resnet50_param_count(num_classes))


def tsm_resnet50_num_tensors():
    return int(lib().tsm_resnet50_num_tensors())


def tsm_resnet50_param_info(num_classes, index):
    """Returns (name, offset, shape tuple, decays)."""
    name = ctypes.create_string_buffer(64)
    off, nd, dec = ctypes.c_int64(), ctypes.c_int(), ctypes.c_int()
    shape = (ctypes.c_int * 4)()
    _check(lib().tsm_resnet50_param_info(num_classes, index, name, 64, ctypes.byref(off), ctypes.byref(nd),
                                         ctypes.byref(shape), ctypes.byref(dec)))
    return name.value.decode(), off.value, tuple(shape[i] for i in range(nd.value)), bool(dec.value)


def tsm_resnet50_param_table(num_classes=400):
    return [tsm_resnet50_param_info(num_classes, i) for i in range(tsm_resnet50_num_tensors())]


def tsm_resnet50_bn_state_count():
    return int(lib().tsm_resnet50_bn_state_count())


def tsm_resnet50_workspace_bytes(desc):
    return int(lib().tsm_resnet50_workspace_bytes(ctypes.addressof(desc)))


def tsm_resnet50_step(desc, clips, labels, params, momentum, bn_state, grads_out, loss_out, logits_out, update, ws,
                      stream=None):
    p, n = _ws(ws)
    _check(lib().tsm_resnet50_step(ctypes.addressof(desc), _ptr(clips), _ptr(labels), _ptr(params), _ptr(momentum),
                                   _ptr(bn_state), _ptr(grads_out), _ptr(loss_out), _ptr(logits_out), int(update),
                                   p, n, _stream(stream)))


def tsm_resnet50_workspace_tensor(desc, name):
    """Returns (byte offset in the step's workspace, (frames, rows, columns, channels), element bytes)."""
    off, eb = ctypes.c_size_t(), ctypes.c_int()
    shape = (ctypes.c_int * 4)()
    _check(lib().tsm_resnet50_workspace_tensor(ctypes.addressof(desc), name.encode(), ctypes.byref(off),
                                               ctypes.byref(shape), ctypes.byref(eb)))
    return off.value, tuple(shape), eb.value


def tsm_resnet50_infer_workspace_bytes(desc):
    return int(lib().tsm_resnet50_infer_workspace_bytes(ctypes.addressof(desc)))


def tsm_resnet50_infer(desc, clips, params, bn_state, logits_out, ws, stream=None):
    p, n = _ws(ws)
    _check(lib().tsm_resnet50_infer(ctypes.addressof(desc), _ptr(clips), _ptr(params), _ptr(bn_state),
                                    _ptr(logits_out), p, n, _stream(stream)))


def tsm_resnet50_accum_step(desc, clips, labels, params, momentum, bn_state, grads_accum, loss_out, logits_out,
                            micro_index, micro_count, ws, stream=None):
    p, n = _ws(ws)
    _check(lib().tsm_resnet50_accum_step(ctypes.addressof(desc), _ptr(clips), _ptr(labels), _ptr(params), _ptr(momentum),
                                         _ptr(bn_state), _ptr(grads_accum), _ptr(loss_out), _ptr(logits_out),
                                         int(micro_index), int(micro_count), p, n, _stream(stream)))


def tsm_lr_schedule(epoch, total_batch, warm_batch=8, warmup_epochs=5.0, total_epochs=100.0):
    v = float(lib().tsm_lr_schedule(float(epoch), int(total_batch), int(warm_batch), float(warmup_epochs),
                                    float(total_epochs)))
    if v < 0:
        _check(-2)
    return v
