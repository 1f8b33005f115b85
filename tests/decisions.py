"""Test policy for the discrete decisions of the network (which units a ReLU lets through, which
element of a window a pool picks).  Not part of the oracle: nothing here computes the model.

The gradient of the training step is unique only where no pre-activation is exactly zero and no
pooling window has two equal largest values.  A value within rounding of such a boundary can be
decided differently by an fp32 evaluation and by the fp64 oracle, and one such decision moves a
gradient tensor by far more than the fp32 tolerance, so the two gradients cannot be compared as they
stand.  The comparison is made decision-matched instead:

  1. take the decisions the GPU made (from its own activations and recorded pool positions);
  2. check that every decision that differs from the oracle's lies within a stated band of its
     boundary in the oracle's own fp64 values (so it is a legitimate alternative, not an error);
  3. run the oracle's backward sweep on the oracle's forward values with those decisions in place
     of its own, and hold every gradient tensor to the plain tolerance, element by element.

Step 3 needs no new arithmetic: the oracle's sweep reads the decisions from its kept forward pass
(the sign of `conv_pre` / `fc_pre`, the entries of `pool_arg`), so `impose` only replaces those
fields.  tests/test_decisions_cpu.py pins this module on the CPU.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

POOL_AFTER = (1, 3, 7, 11, 15)


def windows(y: np.ndarray) -> np.ndarray:
    """[N,C,H,W] -> [N,C,H/2,W/2,4]: the 2x2 windows, elements in the order (0,0),(0,1),(1,0),(1,1)."""
    N, Cc, H, W = y.shape
    return y.reshape(N, Cc, H // 2, 2, W // 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, Cc, H // 2, W // 2, 4)


def unwindow(w: np.ndarray) -> np.ndarray:
    """Inverse of windows()."""
    N, Cc, Ho, Wo, _ = w.shape
    return w.reshape(N, Cc, Ho, Wo, 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, Cc, 2 * Ho, 2 * Wo)


def pooled_layer_mask(pooled_positive: np.ndarray, arg: np.ndarray) -> np.ndarray:
    """ReLU decisions of a convolution whose output went straight into a pool, at the un-pooled
    resolution: true at the picked element of every window whose maximum is positive.  (The other
    three elements of a window receive no gradient, so their decisions do not matter.)"""
    onehot = np.arange(4, dtype=np.uint8) == arg[..., None]
    return unwindow(onehot & pooled_positive[..., None])


def impose(f: Dict[str, object], relu_conv: Sequence[np.ndarray], pool_arg: Dict[int, np.ndarray],
           relu_fc: Sequence[np.ndarray]) -> Dict[str, object]:
    """Copy of a kept forward pass whose decisions are replaced: relu_conv[l] / relu_fc[l] are boolean
    arrays shaped like the layer's output (true = the unit passes gradient), pool_arg[l] the picked
    element 0..3 of every window.  All values of the forward pass are kept as they are."""
    assert len(relu_conv) == 16 and len(relu_fc) == 2 and sorted(pool_arg) == list(POOL_AFTER)
    g = dict(f)
    for m, p in zip(list(relu_conv) + list(relu_fc), list(f["conv_pre"]) + list(f["fc_pre"])):
        assert m.dtype == np.bool_ and m.shape == p.shape
    g["conv_pre"] = [np.where(m, np.int8(1), np.int8(-1)) for m in relu_conv]      # only the sign is read
    g["fc_pre"] = [np.where(m, np.int8(1), np.int8(-1)) for m in relu_fc]
    for l in POOL_AFTER:
        assert pool_arg[l].shape == f["pool_arg"][l].shape and pool_arg[l].max() <= 3
    g["pool_arg"] = {l: np.ascontiguousarray(pool_arg[l], dtype=np.uint8) for l in POOL_AFTER}
    return g


def differences(f: Dict[str, object], relu_conv: Sequence[np.ndarray], pool_arg: Dict[int, np.ndarray],
                relu_fc: Sequence[np.ndarray]) -> Dict[str, object]:
    """How the given decisions differ from those of the kept forward pass f.

    relu: number of units decided differently and the largest |pre-activation| among them, relative to
    the largest magnitude in their layer.  For a convolution followed by a pool only the element that
    the GIVEN pool decision picks is compared (the others receive no gradient).
    pool: number of windows with a positive maximum whose picked element differs, and the largest gap
    between the oracle's values at the two picked elements, relative to the layer's largest value.
    """
    n_relu = n_pool = 0
    worst_relu = worst_pool = 0.0
    units = 0
    relu_by_layer, pool_by_layer = [], {}
    pres: List[np.ndarray] = list(f["conv_pre"]) + list(f["fc_pre"])
    masks = list(relu_conv) + list(relu_fc)
    for l, (pre, m) in enumerate(zip(pres, masks)):
        own = pre > 0.0
        if l in POOL_AFTER:
            picked = np.arange(4, dtype=np.uint8) == pool_arg[l][..., None]
            diff = (windows(own) != windows(m)) & picked
            mag = np.abs(windows(pre))[diff]
            units += picked.sum()
        else:
            diff = own != m
            mag = np.abs(pre)[diff]
            units += pre.size
        relu_by_layer.append(int(mag.size))
        if mag.size:
            n_relu += int(mag.size)
            worst_relu = max(worst_relu, float(mag.max() / np.abs(pre).max()))
    for l in POOL_AFTER:
        y = f["conv_out"][l]
        win = windows(y)
        a_ref, a_new = f["pool_arg"][l], pool_arg[l]
        v_ref = np.take_along_axis(win, a_ref[..., None].astype(np.int64), axis=-1)[..., 0]
        v_new = np.take_along_axis(win, a_new[..., None].astype(np.int64), axis=-1)[..., 0]
        diff = (a_ref != a_new) & (v_ref > 0.0)      # an all-zero window passes no gradient whichever element is picked
        pool_by_layer[l] = int(diff.sum())
        if diff.any():
            n_pool += int(diff.sum())
            worst_pool = max(worst_pool, float((v_ref - v_new)[diff].max() / np.abs(y).max()))
    return dict(relu=n_relu, relu_margin=worst_relu, pool=n_pool, pool_margin=worst_pool, units=int(units),
                relu_by_layer=relu_by_layer, pool_by_layer=pool_by_layer)
