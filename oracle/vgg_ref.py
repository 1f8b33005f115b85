"""Python face of the fp64 CPU oracle (TEST INFRASTRUCTURE ONLY).

The per-op functions marshal numpy float64 arrays into ``libvgg_ref.so``
(vgg_ref.c, direct-loop definitions); the two model-level functions compose
them in the order the paper's VGG19 runs them (section "VGG19 forward pass":
16 convolutions with bias and ReLU, 5 window maxima, 3 dense layers, softmax;
section "VGG19 backward pass": the reverse sweep).  Only tests, the smoke
check and the benchmark's CPU-baseline leg may import this module; it imports
nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None

# Architecture as given by the workload description (the paper cites the
# VGG paper for it; the appendix instruction table confirms 16/5/3).
_CONV_CHANNELS = [(3, 64), (64, 64), (64, 128), (128, 128),
                  (128, 256), (256, 256), (256, 256), (256, 256),
                  (256, 512), (512, 512), (512, 512), (512, 512),
                  (512, 512), (512, 512), (512, 512), (512, 512)]
_POOL_AFTER = {1, 3, 7, 11, 15}

_dp = C.POINTER(C.c_double)
_u8p = C.POINTER(C.c_uint8)
_i32p = C.POINTER(C.c_int32)


def lib() -> C.CDLL:
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libvgg_ref.so")
        if not os.path.exists(path):
            from . import build as _b
            _b.build()
        _LIB = C.CDLL(path)
        _LIB.ref_num_threads.restype = C.c_int
    return _LIB


def num_threads() -> int:
    return int(lib().ref_num_threads())


def _d(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags.c_contiguous
    return a.ctypes.data_as(_dp)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _chk(rc: int):
    if rc != 0:
        raise ValueError(f"oracle returned {rc}")


def conv3x3_fwd(x, w, b=None, relu=True) -> np.ndarray:
    x, w = _f64(x), _f64(w)
    b = None if b is None else _f64(b)
    N, Cin, H, W = x.shape
    Cout = w.shape[0]
    assert w.shape == (Cout, Cin, 3, 3)
    y = np.empty((N, Cout, H, W), dtype=np.float64)
    _chk(lib().ref_conv3x3_fwd(N, Cin, Cout, H, W, _d(x), _d(w), _d(b), int(bool(relu)), _d(y)))
    return y


def conv3x3_bwd_data(g, w) -> np.ndarray:
    g, w = _f64(g), _f64(w)
    N, Cout, H, W = g.shape
    Cin = w.shape[1]
    assert w.shape == (Cout, Cin, 3, 3)
    dx = np.empty((N, Cin, H, W), dtype=np.float64)
    _chk(lib().ref_conv3x3_bwd_data(N, Cin, Cout, H, W, _d(g), _d(w), _d(dx)))
    return dx


def conv3x3_bwd_weight(x, g):
    x, g = _f64(x), _f64(g)
    N, Cin, H, W = x.shape
    Cout = g.shape[1]
    assert g.shape == (N, Cout, H, W)
    dw = np.empty((Cout, Cin, 3, 3), dtype=np.float64)
    db = np.empty((Cout,), dtype=np.float64)
    _chk(lib().ref_conv3x3_bwd_weight(N, Cin, Cout, H, W, _d(x), _d(g), _d(dw), _d(db)))
    return dw, db


def maxpool2x2(x):
    x = _f64(x)
    N, Cc, H, W = x.shape
    p = np.empty((N, Cc, H // 2, W // 2), dtype=np.float64)
    arg = np.empty((N, Cc, H // 2, W // 2), dtype=np.uint8)
    _chk(lib().ref_maxpool2x2(N, Cc, H, W, _d(x), _d(p), arg.ctypes.data_as(_u8p)))
    return p, arg


def maxpool2x2_bwd(dp, arg) -> np.ndarray:
    dp = _f64(dp)
    arg = np.ascontiguousarray(arg, dtype=np.uint8)
    N, Cc, Ho, Wo = dp.shape
    dx = np.empty((N, Cc, 2 * Ho, 2 * Wo), dtype=np.float64)
    _chk(lib().ref_maxpool2x2_bwd(N, Cc, 2 * Ho, 2 * Wo, _d(dp), arg.ctypes.data_as(_u8p), _d(dx)))
    return dx


def fc(a, w, b=None, relu=False) -> np.ndarray:
    a, w = _f64(a), _f64(w)
    b = None if b is None else _f64(b)
    N, In = a.shape
    Out = w.shape[0]
    assert w.shape == (Out, In)
    z = np.empty((N, Out), dtype=np.float64)
    _chk(lib().ref_fc(N, In, Out, _d(a), _d(w), _d(b), int(bool(relu)), _d(z)))
    return z


def fc_bwd(a, w, dz, need_da=True):
    a, w, dz = _f64(a), _f64(w), _f64(dz)
    N, In = a.shape
    Out = w.shape[0]
    dw = np.empty((Out, In), dtype=np.float64)
    db = np.empty((Out,), dtype=np.float64)
    da = np.empty((N, In), dtype=np.float64) if need_da else None
    _chk(lib().ref_fc_bwd(N, In, Out, _d(a), _d(w), _d(dz), _d(dw), _d(db), _d(da)))
    return dw, db, da


def softmax(z) -> np.ndarray:
    z = _f64(z)
    N, K = z.shape
    p = np.empty_like(z)
    _chk(lib().ref_softmax(N, K, _d(z), _d(p)))
    return p


def softmax_vjp(p, u) -> np.ndarray:
    p, u = _f64(p), _f64(u)
    N, K = p.shape
    dz = np.empty_like(p)
    _chk(lib().ref_softmax_vjp(N, K, _d(p), _d(u), _d(dz)))
    return dz


def softmax_xent(p, labels):
    p = _f64(p)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    N, K = p.shape
    loss = C.c_double(0.0)
    dz = np.empty_like(p)
    _chk(lib().ref_softmax_xent(N, K, _d(p), labels.ctypes.data_as(_i32p), C.byref(loss), _d(dz)))
    return float(loss.value), dz


def relu_bwd(y, dy) -> np.ndarray:
    y, dy = _f64(y), _f64(dy)
    g = np.empty_like(y)
    lib().ref_relu_bwd.argtypes = [C.c_size_t, _dp, _dp, _dp]
    _chk(lib().ref_relu_bwd(y.size, _d(y), _d(dy), _d(g)))
    return g


def sgd(theta, grad, lr: float) -> np.ndarray:
    theta = _f64(theta).copy()
    grad = _f64(grad)
    lib().ref_sgd.argtypes = [C.c_size_t, _dp, _dp, C.c_double]
    _chk(lib().ref_sgd(theta.size, _d(theta), _d(grad), float(lr)))
    return theta


def round_bf16(a) -> np.ndarray:
    """Nearest bfloat16 value (8 significant bits, ties to even), returned as
    float64: the operand precision of the accelerator's matrix unit, which
    multiplies bfloat16 values and accumulates in float32 (section on the TPU
    hardware).  Exponent range is float32's, so for the magnitudes that occur
    here no overflow or underflow handling is needed."""
    a = _f64(a)
    m, e = np.frexp(a)                       # a = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0), e - 8)   # np.rint rounds halves to even


# --------------------------------------------------------------------------
# Whole model
# --------------------------------------------------------------------------

def vgg19_forward(x, conv_w: Sequence, conv_b: Sequence, fc_w: Sequence, fc_b: Sequence,
                  keep: bool = False, operand_round=None, progress=None) -> Dict[str, object]:
    """images [N,3,H,W] -> logits, probs (and every intermediate when keep).

    Order of operations: for each of the 16 convolutions, cross-correlate,
    add bias, clamp at zero; after convolutions 2, 4, 8, 12 and 16 take the
    2x2 maximum; flatten in C,H,W order; dense+ReLU, dense+ReLU, dense;
    softmax over the classes of each image.

    ``operand_round`` (e.g. round_bf16) models reduced-precision matrix
    operands: it is applied to everything that enters a product (the images,
    every weight tensor, every layer's output after its ReLU); biases, sums,
    the logits and the softmax stay in full precision.

    ``progress`` (optional) is called with a short text after every layer, for
    callers that must show signs of life during a long run.
    """
    rd = operand_round if operand_round is not None else (lambda a: a)
    say = progress if progress is not None else (lambda text: None)
    assert len(conv_w) == 16 and len(fc_w) == 3
    out: Dict[str, object] = {}
    acts: List[np.ndarray] = []      # input of every conv layer
    pres: List[np.ndarray] = []      # pre-activation (bias added, before ReLU) of every conv layer
    ys: List[np.ndarray] = []        # post-ReLU output of every conv layer
    args: Dict[int, np.ndarray] = {}
    h = rd(_f64(x))
    for l, (cin, cout) in enumerate(_CONV_CHANNELS):
        assert conv_w[l].shape == (cout, cin, 3, 3)
        if keep:
            acts.append(h)
            pre = conv3x3_fwd(h, rd(conv_w[l]), conv_b[l], relu=False)
            pres.append(pre)
            h = rd(np.maximum(pre, 0.0))
            ys.append(h)
        else:
            h = rd(conv3x3_fwd(h, rd(conv_w[l]), conv_b[l], relu=True))
        if l in _POOL_AFTER:
            h, a = maxpool2x2(h)
            if keep:
                args[l] = a
        say("oracle forward: convolution %d done" % l)
    N = h.shape[0]
    flat = h.reshape(N, -1)
    pre1 = fc(flat, rd(fc_w[0]), fc_b[0], relu=False)
    z1 = rd(np.maximum(pre1, 0.0))
    pre2 = fc(z1, rd(fc_w[1]), fc_b[1], relu=False)
    z2 = rd(np.maximum(pre2, 0.0))
    logits = fc(z2, rd(fc_w[2]), fc_b[2], relu=False)
    out["logits"] = logits
    out["probs"] = softmax(logits)
    if keep:
        out.update(conv_in=acts, conv_pre=pres, conv_out=ys, pool_arg=args, pool5=h, flat=flat, z1=z1, z2=z2,
                   fc_pre=[pre1, pre2])
    return out


def vgg19_gradients(f: Dict[str, object], labels, conv_w, fc_w, operand_round=None, progress=None) -> Dict[str, object]:
    """Backward sweep from a kept forward pass ``f`` (vgg19_forward(keep=True)):
    the gradient of the mean softmax cross-entropy.  A ReLU passes gradient
    where its pre-activation (``f["conv_pre"]``, ``f["fc_pre"]``) is strictly
    positive, a pool routes its gradient to the recorded first maximum
    (``f["pool_arg"]``), and the first convolution's input gradient is not
    formed (the paper's optimised backward pass has 47 convolutions, not 48).

    ``operand_round`` as in vgg19_forward (f must come from a forward pass with
    the same setting): the gradient that enters the convolution stack and the
    result of every data-gradient convolution are rounded, as are the
    weights a data gradient multiplies with (convolution and dense) and the
    gradient with respect to a dense layer's pre-activation where it enters
    one of that layer's two backward products; sums (bias gradients
    included) are not rounded.  ``progress`` as in vgg19_forward.
    """
    rd = operand_round if operand_round is not None else (lambda a: a)
    say = progress if progress is not None else (lambda text: None)

    def relu_mask(pre, d):
        return np.where(pre > 0.0, d, 0.0)

    loss, dlogits = softmax_xent(f["probs"], labels)
    dfc_w = [None] * 3
    dfc_b = [None] * 3
    def dense_bwd(a, w, dz):
        # with operand rounding the two products see the rounded dz and the rounded weights; the bias
        # gradient is a plain sum of the unrounded dz
        dw, _, da = fc_bwd(a, rd(w), rd(dz))
        return dw, _f64(dz).sum(axis=0), da

    dfc_w[2], dfc_b[2], dz2 = dense_bwd(f["z2"], fc_w[2], dlogits)
    dz2 = relu_mask(f["fc_pre"][1], dz2)
    dfc_w[1], dfc_b[1], dz1 = dense_bwd(f["z1"], fc_w[1], dz2)
    dz1 = relu_mask(f["fc_pre"][0], dz1)
    dfc_w[0], dfc_b[0], dflat = dense_bwd(f["flat"], fc_w[0], dz1)
    d = rd(dflat.reshape(f["pool5"].shape))
    dconv_w = [None] * 16
    dconv_b = [None] * 16
    for l in range(15, -1, -1):
        if l in _POOL_AFTER:
            d = maxpool2x2_bwd(d, f["pool_arg"][l])
        g = relu_mask(f["conv_pre"][l], d)
        dconv_w[l], dconv_b[l] = conv3x3_bwd_weight(f["conv_in"][l], g)
        if l > 0:
            d = rd(conv3x3_bwd_data(g, rd(conv_w[l])))
        say("oracle backward: convolution %d done" % l)
    return dict(loss=loss, dconv_w=dconv_w, dconv_b=dconv_b, dfc_w=dfc_w, dfc_b=dfc_b)


def vgg19_train_step(x, labels, conv_w, conv_b, fc_w, fc_b, lr: float = 0.01, operand_round=None) -> Dict[str, object]:
    """One step: forward, mean softmax cross-entropy, full backward, plain SGD.

    Returns loss, logits, probs, the 38 gradient tensors (dconv_w/dconv_b/
    dfc_w/dfc_b), the updated parameters (new_*) and the kept forward pass
    (``fwd``, the input of vgg19_gradients).  With ``operand_round``
    the update is applied to the unrounded (master) parameters.
    """
    f = vgg19_forward(x, conv_w, conv_b, fc_w, fc_b, keep=True, operand_round=operand_round)
    res = vgg19_gradients(f, labels, conv_w, fc_w, operand_round=operand_round)
    res.update(logits=f["logits"], probs=f["probs"], fwd=f)
    res["new_conv_w"] = [sgd(conv_w[l], res["dconv_w"][l], lr) for l in range(16)]
    res["new_conv_b"] = [sgd(conv_b[l], res["dconv_b"][l], lr) for l in range(16)]
    res["new_fc_w"] = [sgd(fc_w[l], res["dfc_w"][l], lr) for l in range(3)]
    res["new_fc_b"] = [sgd(fc_b[l], res["dfc_b"][l], lr) for l in range(3)]
    return res
