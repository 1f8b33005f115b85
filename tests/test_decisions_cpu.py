"""CPU pins of tests/decisions.py (the policy that compares gradients decision-matched): against the
oracle's own decisions, against hand-placed pre-activations and window values a hair on either side of
their decision boundary, and against the oracle's pool routine for the window order."""
import numpy as np

from oracle import vgg_ref as R
from paper_1810_09868_amd import synth

import decisions as D


def _f64(lst):
    return [np.asarray(a, dtype=np.float64).copy() for a in lst]


def _own_decisions(f):
    relu_conv = []
    for l, pre in enumerate(f["conv_pre"]):
        if l in D.POOL_AFTER:
            pooled, arg = R.maxpool2x2(f["conv_out"][l])
            relu_conv.append(D.pooled_layer_mask(pooled > 0.0, arg))
        else:
            relu_conv.append(pre > 0.0)
    return relu_conv, {l: f["pool_arg"][l].copy() for l in D.POOL_AFTER}, [p > 0.0 for p in f["fc_pre"]]


def _grads(x, labels, cw, cb, fw, fb):
    f = R.vgg19_forward(x, cw, cb, fw, fb, keep=True)
    return f, R.vgg19_gradients(f, labels, cw, fw)


def _worst(a, b):
    worst = 0.0
    for k in ("dconv_w", "dconv_b", "dfc_w", "dfc_b"):
        for u, v in zip(a[k], b[k]):
            worst = max(worst, float(np.abs(u - v).max() / max(np.abs(v).max(), 1e-300)))
    return worst


def test_window_order_is_the_pool_routines():
    rng = np.random.default_rng(5)
    y = rng.standard_normal((2, 3, 6, 8))
    pooled, arg = R.maxpool2x2(y)
    w = D.windows(y)
    assert np.array_equal(w.argmax(-1).astype(np.uint8), arg)          # numpy's argmax also takes the first maximum
    assert np.array_equal(w.max(-1), pooled)
    assert np.array_equal(D.unwindow(w), y)
    # element k of a window is (k // 2, k % 2)
    for k in range(4):
        assert np.array_equal(w[..., k], y[:, :, k // 2::2, k % 2::2])
    # scattering a mask to the picked elements is what the pool's backward routine does to a gradient
    pos = rng.random(pooled.shape) > 0.4
    assert np.array_equal(D.pooled_layer_mask(pos, arg), R.maxpool2x2_bwd(pos.astype(np.float64), arg) > 0)


def test_own_decisions_reproduce_the_gradient_exactly():
    inp = synth.tiny_config(seed=0)
    cw, cb, fw, fb = _f64(inp.conv_w), _f64(inp.conv_b), _f64(inp.fc_w), _f64(inp.fc_b)
    f, g = _grads(inp.x, inp.labels, cw, cb, fw, fb)
    rc, pa, rf = _own_decisions(f)
    # (for a pooled layer only the picked elements carry a decision: the mask is not the full y > 0)
    assert not np.array_equal(rc[1], f["conv_pre"][1] > 0)
    g2 = R.vgg19_gradients(D.impose(f, rc, pa, rf), inp.labels, cw, fw)
    assert _worst(g2, g) == 0.0 and g2["loss"] == g["loss"]
    d = D.differences(f, rc, pa, rf)
    assert d["relu"] == 0 and d["pool"] == 0 and d["relu_margin"] == 0.0 and d["pool_margin"] == 0.0
    # the forward values are untouched by impose
    f2 = D.impose(f, rc, pa, rf)
    assert f2["conv_in"] is f["conv_in"] and f2["probs"] is f["probs"] and f["conv_pre"][3].dtype == np.float64


def _two_sides(make, eps):
    """make(delta) -> (x, cw, cb, fw, fb); returns forward and gradient on either side of the boundary."""
    return [_grads(*make(s * eps)) for s in (+1.0, -1.0)]


def test_imposed_relu_decisions_give_the_neighbouring_gradient():
    # A dense unit and a convolution unit whose pre-activation is placed at +eps / -eps through their bias:
    # the two networks differ by 2 eps in one number, yet their gradients differ by a finite amount, and
    # the gradient on the minus side with the plus side's decisions imposed is the plus side's.
    inp = synth.tiny_config(seed=3)
    base = (_f64(inp.conv_w), _f64(inp.conv_b), _f64(inp.fc_w), _f64(inp.fc_b))
    f0 = R.vgg19_forward(inp.x, *base, keep=True)
    eps = 1e-9
    j = int(np.argmax(f0["fc_pre"][0][0]))              # an active unit of the first dense layer (image 0)
    c = int(np.argmax(f0["conv_pre"][8][0].max(axis=(1, 2))))
    hw = np.unravel_index(int(np.argmax(f0["conv_pre"][8][0, c])), f0["conv_pre"][8].shape[2:])

    def dense_case(delta):
        cw, cb, fw, fb = (_f64(t) for t in base)
        fb[0][j] += delta - f0["fc_pre"][0][0, j]
        return inp.x, inp.labels, cw, cb, fw, fb

    def conv_case(delta):
        cw, cb, fw, fb = (_f64(t) for t in base)
        cb[8][c] += delta - f0["conv_pre"][8][0, c, hw[0], hw[1]]
        return inp.x, inp.labels, cw, cb, fw, fb

    for case, where in ((dense_case, ("fc_pre", 0, (0, j))), (conv_case, ("conv_pre", 8, (0, c) + tuple(hw)))):
        (fp, gp), (fm, gm) = _two_sides(case, eps)
        key, l, idx = where
        assert 0 < fp[key][l][idx] < 10 * eps and -10 * eps < fm[key][l][idx] < 0
        assert _worst(gm, gp) > 1e-4                     # one decision, a finite change
        args = case(-eps)
        gi = R.vgg19_gradients(D.impose(fm, *_own_decisions(fp)), args[1], args[2], args[4])
        assert _worst(gi, gp) < 1e-6
        d = D.differences(fm, *_own_decisions(fp))
        assert d["relu"] == 1 and d["pool"] == 0 and 0 < d["relu_margin"] < 1e-8


def test_imposed_pool_decisions_give_the_neighbouring_gradient():
    # The first two convolutions pass the first image channel through unchanged (centre-tap delta kernels,
    # zero bias; the images are non-negative), so a window of the first pool in that channel holds four
    # image pixels.  Two of them are set to v and v +- eps: the pool picks the one or the other.
    inp = synth.tiny_config(seed=4)
    eps = 1e-9

    def case(delta):
        cw, cb, fw, fb = _f64(inp.conv_w), _f64(inp.conv_b), _f64(inp.fc_w), _f64(inp.fc_b)
        for l in (0, 1):
            cw[l][0] = 0.0
            cw[l][0, 0, 1, 1] = 1.0
            cb[l][0] = 0.0
        x = np.asarray(inp.x, dtype=np.float64).copy()
        x[0, 0, 4:6, 6:8] = 0.25
        x[0, 0, 4, 6] = 0.9
        x[0, 0, 5, 7] = 0.9 + delta
        return x, inp.labels, cw, cb, fw, fb

    (fp, gp), (fm, gm) = _two_sides(case, eps)
    assert fp["pool_arg"][1][0, 0, 2, 3] == 3 and fm["pool_arg"][1][0, 0, 2, 3] == 0
    assert np.array_equal(fp["conv_out"][1][0, 0], case(eps)[0][0, 0])      # the channel really is the image
    assert _worst(gm, gp) > 1e-4
    args = case(-eps)
    gi = R.vgg19_gradients(D.impose(fm, *_own_decisions(fp)), args[1], args[2], args[4])
    assert _worst(gi, gp) < 1e-6
    d = D.differences(fm, *_own_decisions(fp))
    assert d["pool"] == 1 and 0 < d["pool_margin"] < 1e-8 and d["relu"] == 0
