"""Thin ctypes binding of libvgg_mi355x.so (see include/vgg_mi355x.h).

Argument marshalling only: every function takes torch CUDA tensors (used as
device buffers), passes their ``data_ptr()`` and the current stream to the C
entry point of the same name, and raises :class:`VggError` on a non-zero
status.  There is no CPU fallback; a missing library raises at first use.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvgg_mi355x.so")

F32, BF16 = 0, 1
NUM_CONV, NUM_FC = 16, 3

EXPORTS = [
    "vgg_strerror", "vgg_padded_channels", "vgg_conv_pack_weights", "vgg_conv_unpack_weights",
    "vgg_nchw_to_nhwc", "vgg_nhwc_to_nchw", "vgg_convert",
    "vgg_conv3x3_fwd_workspace_bytes", "vgg_conv3x3_fwd", "vgg_conv3x3_fwd_pool", "vgg_conv3x3_fwd_first", "vgg_conv3x3_fwd_first_pair",
    "vgg_conv3x3_bwd_data_workspace_bytes", "vgg_conv3x3_bwd_data",
    "vgg_conv3x3_bwd_weight_workspace_bytes", "vgg_conv3x3_bwd_weight",
    "vgg_maxpool2x2", "vgg_maxpool2x2_bwd",
    "vgg_fc_workspace_bytes", "vgg_fc", "vgg_fc_bwd_workspace_bytes", "vgg_fc_bwd",
    "vgg_softmax", "vgg_softmax_xent_bwd", "vgg_sgd_update",
    "vgg19_packed_bytes", "vgg19_forward_workspace_bytes", "vgg19_train_workspace_bytes",
    "vgg19_pack_params", "vgg19_unpack_params", "vgg19_forward", "vgg19_train_step", "vgg19_plan",
    "vgg19_timed", "vgg_mfma_probe_sink_bytes", "vgg_mfma_probe", "vgg_conv3x3_plan",
    "vgg_fc_static",
]


class VggError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().vgg_strerror(status).decode() if _LIB is not None else "?"
        super().__init__(f"{where}: {msg} ({status})")


class VggConfig(C.Structure):
    _fields_ = [("dtype", C.c_int), ("N", C.c_int), ("H", C.c_int), ("W", C.c_int),
                ("fc_hidden", C.c_int), ("classes", C.c_int), ("lr", C.c_float), ("flags", C.c_int)]


class Vgg19Params(C.Structure):
    _fields_ = [("conv_w", C.c_void_p * NUM_CONV), ("conv_b", C.c_void_p * NUM_CONV),
                ("fc_w", C.c_void_p * NUM_FC), ("fc_b", C.c_void_p * NUM_FC)]


_LIB: Optional[C.CDLL] = None
_vp, _sz, _i = C.c_void_p, C.c_size_t, C.c_int


def lib() -> C.CDLL:
    """Loads the shared library (once).  Raises if it has not been built."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1810_09868_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.vgg_strerror.restype = C.c_char_p
        L.vgg_strerror.argtypes = [_i]
        L.vgg_padded_channels.argtypes = [_i, _i]
        L.vgg_conv_pack_weights.argtypes = [_i, _i, _i, _vp, _vp, _i, _vp]
        L.vgg_conv_unpack_weights.argtypes = [_i, _i, _vp, _vp, _vp]
        L.vgg_nchw_to_nhwc.argtypes = [_i] * 6 + [_vp, _vp, _vp]
        L.vgg_nhwc_to_nchw.argtypes = [_i] * 6 + [_vp, _vp, _vp]
        L.vgg_convert.argtypes = [_i, _i, _sz, _vp, _vp, _vp]
        for n in ("vgg_conv3x3_fwd_workspace_bytes", "vgg_conv3x3_bwd_data_workspace_bytes",
                  "vgg_conv3x3_bwd_weight_workspace_bytes"):
            getattr(L, n).restype = _sz
            getattr(L, n).argtypes = [_i] * 6
        L.vgg_conv3x3_fwd.argtypes = [_i] * 6 + [_vp, _vp, _vp, _vp, _i, _vp, _sz, _vp]
        L.vgg_conv3x3_fwd_pool.argtypes = [_i] * 6 + [_vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _sz, _vp]
        L.vgg_conv3x3_fwd_first.argtypes = [_i] * 4 + [_vp, _vp, _vp, _vp, _i, _vp]
        L.vgg_conv3x3_fwd_first_pair.argtypes = [_i] * 4 + [_vp] * 8
        L.vgg_conv3x3_bwd_data.argtypes = [_i] * 6 + [_vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.vgg_conv3x3_bwd_weight.argtypes = [_i] * 6 + [_vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.vgg_maxpool2x2.argtypes = [_i] * 5 + [_vp, _vp, _vp, _vp]
        L.vgg_maxpool2x2_bwd.argtypes = [_i] * 5 + [_vp, _vp, _vp, _vp]
        for n in ("vgg_fc_workspace_bytes", "vgg_fc_bwd_workspace_bytes"):
            getattr(L, n).restype = _sz
            getattr(L, n).argtypes = [_i] * 4
        L.vgg_fc.argtypes = [_i] * 4 + [_vp, _vp, _vp, _vp, _i, _i, _vp, _sz, _vp]
        L.vgg_fc_static.argtypes = [_i] * 4 + [_vp, _vp, _vp, _vp, _i, _i, _vp]
        L.vgg_fc_bwd.argtypes = [_i] * 4 + [_vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _sz, _vp]
        L.vgg_softmax.argtypes = [_i, _i, _vp, _vp, _vp]
        L.vgg_softmax_xent_bwd.argtypes = [_i, _i, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.vgg_sgd_update.argtypes = [_sz, _vp, _vp, C.c_float, _vp]
        cfgp = C.POINTER(VggConfig)
        prmp = C.POINTER(Vgg19Params)
        for n in ("vgg19_packed_bytes", "vgg19_forward_workspace_bytes", "vgg19_train_workspace_bytes"):
            getattr(L, n).restype = _sz
            getattr(L, n).argtypes = [cfgp]
        L.vgg19_pack_params.argtypes = [cfgp, prmp, _vp, _sz, _vp]
        L.vgg19_unpack_params.argtypes = [cfgp, _vp, _sz, prmp, _vp]
        L.vgg19_forward.argtypes = [cfgp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.vgg19_train_step.argtypes = [cfgp, _vp, _vp, _vp, _sz, prmp, _vp, _vp, _vp, _sz, _vp]
        L.vgg19_plan.argtypes = [cfgp, _i, C.POINTER(C.c_int), _i]
        L.vgg19_timed.argtypes = [cfgp, _i, _vp, _vp, _vp, _sz, _vp, _vp, _sz, C.POINTER(C.c_int),
                                  C.POINTER(C.c_float), _i, _vp]
        L.vgg_conv3x3_plan.argtypes = [_i] * 7 + [C.POINTER(C.c_int), _i]
        L.vgg_mfma_probe_sink_bytes.restype = _sz
        L.vgg_mfma_probe_sink_bytes.argtypes = []
        L.vgg_mfma_probe.argtypes = [_i, _i, _i, _vp, _sz, C.POINTER(C.c_double), _vp]
        _LIB = L
    return _LIB


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _chk(rc: int, where: str):
    if rc != 0:
        raise VggError(rc, where)


FLAG_FP32_MASTER = 1  # VGG_FLAG_FP32_MASTER


def make_config(dtype: int, N: int, H: int, W: int, fc_hidden: int, classes: int, lr: float = 0.01,
                flags: int = 0) -> VggConfig:
    return VggConfig(dtype, N, H, W, fc_hidden, classes, lr, flags)


def make_params(conv_w: Sequence, conv_b: Sequence, fc_w: Sequence, fc_b: Sequence) -> Vgg19Params:
    p = Vgg19Params()
    for l in range(NUM_CONV):
        p.conv_w[l] = conv_w[l].data_ptr()
        p.conv_b[l] = conv_b[l].data_ptr()
    for l in range(NUM_FC):
        p.fc_w[l] = fc_w[l].data_ptr()
        p.fc_b[l] = fc_b[l].data_ptr()
    return p


# ------------------------------------------------------------------ per-op
def vgg_padded_channels(dtype: int, Cc: int) -> int:
    return lib().vgg_padded_channels(dtype, Cc)


def vgg_conv_pack_weights(dtype, Cin, Cout, w_oihw, w_packed, transpose_flip=0):
    _chk(lib().vgg_conv_pack_weights(dtype, Cin, Cout, _ptr(w_oihw), _ptr(w_packed), int(transpose_flip), _stream()),
         "vgg_conv_pack_weights")


def vgg_conv_unpack_weights(Cin, Cout, w_packed, w_oihw):
    _chk(lib().vgg_conv_unpack_weights(Cin, Cout, _ptr(w_packed), _ptr(w_oihw), _stream()), "vgg_conv_unpack_weights")


def vgg_nchw_to_nhwc(dtype, N, Cc, H, W, Cpad, x_nchw, y_nhwc):
    _chk(lib().vgg_nchw_to_nhwc(dtype, N, Cc, H, W, Cpad, _ptr(x_nchw), _ptr(y_nhwc), _stream()), "vgg_nchw_to_nhwc")


def vgg_nhwc_to_nchw(dtype, N, Cc, H, W, Cpad, x_nhwc, y_nchw):
    _chk(lib().vgg_nhwc_to_nchw(dtype, N, Cc, H, W, Cpad, _ptr(x_nhwc), _ptr(y_nchw), _stream()), "vgg_nhwc_to_nchw")


def vgg_convert(src_dtype, dst_dtype, n, src, dst):
    _chk(lib().vgg_convert(src_dtype, dst_dtype, n, _ptr(src), _ptr(dst), _stream()), "vgg_convert")


def vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, Cin, Cout) -> int:
    return lib().vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, Cin, Cout)


def vgg_conv3x3_fwd(dtype, N, H, W, Cin, Cout, x, w_packed, bias, y, relu, ws=None):
    _chk(lib().vgg_conv3x3_fwd(dtype, N, H, W, Cin, Cout, _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(y), int(relu),
                               _ptr(ws), _nbytes(ws), _stream()), "vgg_conv3x3_fwd")


def vgg_conv3x3_fwd_pool(dtype, N, H, W, Cin, Cout, x, w_packed, bias, y, pooled, relu, ws=None, argmax=None):
    _chk(lib().vgg_conv3x3_fwd_pool(dtype, N, H, W, Cin, Cout, _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(y), _ptr(pooled),
                                    _ptr(argmax), int(relu), _ptr(ws), _nbytes(ws), _stream()), "vgg_conv3x3_fwd_pool")


def vgg_conv3x3_fwd_first(dtype, N, H, W, x_nchw, w_packed, bias, y, relu):
    _chk(lib().vgg_conv3x3_fwd_first(dtype, N, H, W, _ptr(x_nchw), _ptr(w_packed), _ptr(bias), _ptr(y), int(relu),
                                     _stream()), "vgg_conv3x3_fwd_first")


def vgg_conv3x3_fwd_first_pair(dtype, N, H, W, x_nchw, w1_packed, bias1, w2_packed, bias2, y2, pooled):
    _chk(lib().vgg_conv3x3_fwd_first_pair(dtype, N, H, W, _ptr(x_nchw), _ptr(w1_packed), _ptr(bias1), _ptr(w2_packed),
                                          _ptr(bias2), _ptr(y2), _ptr(pooled), _stream()), "vgg_conv3x3_fwd_first_pair")


def vgg_conv3x3_bwd_data_workspace_bytes(dtype, N, H, W, Cin, Cout) -> int:
    return lib().vgg_conv3x3_bwd_data_workspace_bytes(dtype, N, H, W, Cin, Cout)


def vgg_conv3x3_bwd_data(dtype, N, H, W, Cin, Cout, g, w_tf, relu_src, dx, ws=None):
    _chk(lib().vgg_conv3x3_bwd_data(dtype, N, H, W, Cin, Cout, _ptr(g), _ptr(w_tf), _ptr(relu_src), _ptr(dx),
                                    _ptr(ws), _nbytes(ws), _stream()), "vgg_conv3x3_bwd_data")


def vgg_conv3x3_bwd_weight_workspace_bytes(dtype, N, H, W, Cin, Cout) -> int:
    return lib().vgg_conv3x3_bwd_weight_workspace_bytes(dtype, N, H, W, Cin, Cout)


def vgg_conv3x3_bwd_weight(dtype, N, H, W, Cin, Cout, x, g, dw_packed, db, ws):
    _chk(lib().vgg_conv3x3_bwd_weight(dtype, N, H, W, Cin, Cout, _ptr(x), _ptr(g), _ptr(dw_packed), _ptr(db),
                                      _ptr(ws), _nbytes(ws), _stream()), "vgg_conv3x3_bwd_weight")


def vgg_maxpool2x2(dtype, N, H, W, Cc, x, y, argmax=None):
    _chk(lib().vgg_maxpool2x2(dtype, N, H, W, Cc, _ptr(x), _ptr(y), _ptr(argmax), _stream()), "vgg_maxpool2x2")


def vgg_maxpool2x2_bwd(dtype, N, H, W, Cc, dy, argmax, dx):
    _chk(lib().vgg_maxpool2x2_bwd(dtype, N, H, W, Cc, _ptr(dy), _ptr(argmax), _ptr(dx), _stream()), "vgg_maxpool2x2_bwd")


def vgg_fc_workspace_bytes(dtype, N, In, Out) -> int:
    return lib().vgg_fc_workspace_bytes(dtype, N, In, Out)


def vgg_fc(dtype, N, In, Out, a, w, bias, z, z_dtype, relu, ws):
    _chk(lib().vgg_fc(dtype, N, In, Out, _ptr(a), _ptr(w), _ptr(bias), _ptr(z), z_dtype, int(relu), _ptr(ws),
                      _nbytes(ws), _stream()), "vgg_fc")


FC_STATIC_SCRATCH_BYTES = 32 << 20  # VGG_FC_STATIC_SCRATCH_BYTES


def vgg_fc_static(dtype, N, In, Out, a, w, bias, z, z_dtype, relu):
    _chk(lib().vgg_fc_static(dtype, N, In, Out, _ptr(a), _ptr(w), _ptr(bias), _ptr(z), z_dtype, int(relu), _stream()),
         "vgg_fc_static")


def vgg_fc_bwd_workspace_bytes(dtype, N, In, Out) -> int:
    return lib().vgg_fc_bwd_workspace_bytes(dtype, N, In, Out)


def vgg_fc_bwd(dtype, N, In, Out, a, w, dz, dw, db, da, relu_mask, ws):
    _chk(lib().vgg_fc_bwd(dtype, N, In, Out, _ptr(a), _ptr(w), _ptr(dz), _ptr(dw), _ptr(db), _ptr(da), int(relu_mask),
                          _ptr(ws), _nbytes(ws), _stream()), "vgg_fc_bwd")


def vgg_softmax(N, K, z, p):
    _chk(lib().vgg_softmax(N, K, _ptr(z), _ptr(p), _stream()), "vgg_softmax")


def vgg_softmax_xent_bwd(N, K, p, labels, loss, dz, ws):
    _chk(lib().vgg_softmax_xent_bwd(N, K, _ptr(p), _ptr(labels), _ptr(loss), _ptr(dz), _ptr(ws), _nbytes(ws), _stream()),
         "vgg_softmax_xent_bwd")


def vgg_sgd_update(n, theta, grad, lr):
    _chk(lib().vgg_sgd_update(n, _ptr(theta), _ptr(grad), float(lr), _stream()), "vgg_sgd_update")


# ------------------------------------------------------------- whole model
def vgg19_packed_bytes(cfg: VggConfig) -> int:
    return lib().vgg19_packed_bytes(C.byref(cfg))


def vgg19_forward_workspace_bytes(cfg: VggConfig) -> int:
    return lib().vgg19_forward_workspace_bytes(C.byref(cfg))


def vgg19_train_workspace_bytes(cfg: VggConfig) -> int:
    return lib().vgg19_train_workspace_bytes(C.byref(cfg))


def vgg19_pack_params(cfg, params: Vgg19Params, packed):
    _chk(lib().vgg19_pack_params(C.byref(cfg), C.byref(params), _ptr(packed), _nbytes(packed), _stream()),
         "vgg19_pack_params")


def vgg19_unpack_params(cfg, packed, params_out: Vgg19Params):
    _chk(lib().vgg19_unpack_params(C.byref(cfg), _ptr(packed), _nbytes(packed), C.byref(params_out), _stream()),
         "vgg19_unpack_params")


def vgg19_forward(cfg, x_nchw, packed, logits, probs, ws):
    _chk(lib().vgg19_forward(C.byref(cfg), _ptr(x_nchw), _ptr(packed), _ptr(logits), _ptr(probs), _ptr(ws),
                             _nbytes(ws), _stream()), "vgg19_forward")


def vgg19_train_step(cfg, x_nchw, labels, packed, grads: Optional[Vgg19Params], loss, logits, ws):
    gp = C.byref(grads) if grads is not None else None
    _chk(lib().vgg19_train_step(C.byref(cfg), _ptr(x_nchw), _ptr(labels), _ptr(packed), _nbytes(packed), gp,
                                _ptr(loss), _ptr(logits), _ptr(ws), _nbytes(ws), _stream()), "vgg19_train_step")


def vgg19_plan(cfg, training: bool) -> List[int]:
    n = lib().vgg19_plan(C.byref(cfg), int(training), None, 0)
    if n < 0:
        raise VggError(n, "vgg19_plan")
    buf = (C.c_int * n)()
    lib().vgg19_plan(C.byref(cfg), int(training), buf, n)
    return list(buf)


PLAN_FWD, PLAN_FWD_POOL, PLAN_BWD_DATA, PLAN_BWD_WEIGHT = 0, 1, 2, 3


def vgg_conv3x3_plan(op: int, dtype: int, N: int, H: int, W: int, Cin: int, Cout: int) -> List[int]:
    """Launch plan of one convolution call (see the header): kernel, tile, splits, workgroups."""
    info = (C.c_int * 7)()
    _chk(lib().vgg_conv3x3_plan(op, dtype, N, H, W, Cin, Cout, info, 7), "vgg_conv3x3_plan")
    return list(info)


def vgg19_timed(cfg, training: bool, x_nchw, labels, packed, logits, ws):
    """Returns (kinds, ms): per-step kind codes and elapsed milliseconds of one pass."""
    n = lib().vgg19_plan(C.byref(cfg), int(training), None, 0)
    if n < 0:
        raise VggError(n, "vgg19_plan")
    kinds = (C.c_int * n)()
    ms = (C.c_float * n)()
    rc = lib().vgg19_timed(C.byref(cfg), int(training), _ptr(x_nchw), _ptr(labels), _ptr(packed), _nbytes(packed),
                           _ptr(logits), _ptr(ws), _nbytes(ws), kinds, ms, n, _stream())
    if rc < 0:
        raise VggError(rc, "vgg19_timed")
    return list(kinds), list(ms)


def vgg_mfma_probe_sink_bytes() -> int:
    return lib().vgg_mfma_probe_sink_bytes()


def vgg_mfma_probe(dtype, random_operands: bool, iters: int, sink, shape_16x16x32: bool = False) -> float:
    """Enqueues the MFMA-only loop; returns the number of floating-point operations it performs."""
    flops = C.c_double(0.0)
    mode = int(bool(random_operands)) | (2 if shape_16x16x32 else 0)
    _chk(lib().vgg_mfma_probe(dtype, mode, iters, _ptr(sink), _nbytes(sink), C.byref(flops), _stream()),
         "vgg_mfma_probe")
    return flops.value
