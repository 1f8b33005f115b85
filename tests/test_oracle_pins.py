"""Pins for the fp64 CPU oracle: each test checks it against something other
than itself -- closed forms, library routines on special cases, brute force,
finite differences, and counts the paper prints."""
import itertools
import os

import numpy as np
import pytest
import scipy.signal

from oracle import vgg_ref as R

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(12345)


# ----------------------------------------------------------------- conv fwd
def test_conv_offcentre_delta_pins_orientation_and_padding():
    # weight = 1 at tap (kh,kw)=(0,0) for co==ci: pre[h,w] = x[h-1,w-1], zero at top/left border
    N, Cc, H, W = 2, 3, 5, 6
    x = rng.standard_normal((N, Cc, H, W))
    for kh, kw in itertools.product(range(3), range(3)):
        w = np.zeros((Cc, Cc, 3, 3))
        for c in range(Cc):
            w[c, c, kh, kw] = 1.0
        y = R.conv3x3_fwd(x, w, None, relu=False)
        exp = np.zeros_like(x)
        for h in range(H):
            for ww in range(W):
                hi, wi = h + kh - 1, ww + kw - 1
                if 0 <= hi < H and 0 <= wi < W:
                    exp[:, :, h, ww] = x[:, :, hi, wi]
        assert np.array_equal(y, exp), (kh, kw)


def test_conv_channel_mixing_delta():
    # weight[co=1, ci=2, centre] = 1 only: y[:,1] = x[:,2], other outputs zero (pins OIHW order)
    x = rng.standard_normal((1, 3, 4, 4))
    w = np.zeros((2, 3, 3, 3))
    w[1, 2, 1, 1] = 1.0
    y = R.conv3x3_fwd(x, w, None, relu=False)
    assert np.array_equal(y[:, 1], x[:, 2]) and not y[:, 0].any()


def test_conv_all_ones_closed_form():
    Cin, H, W = 5, 6, 7
    y = R.conv3x3_fwd(np.ones((1, Cin, H, W)), np.ones((2, Cin, 3, 3)), None, relu=False)
    exp = np.full((H, W), 9.0 * Cin)
    exp[0, :] = exp[-1, :] = exp[:, 0] = exp[:, -1] = 6.0 * Cin
    exp[0, 0] = exp[0, -1] = exp[-1, 0] = exp[-1, -1] = 4.0 * Cin
    assert np.array_equal(y[0, 0], exp) and np.array_equal(y[0, 1], exp)


def test_conv_matches_scipy_correlate2d():
    # special case reducing to a library routine: sum over ci of 2-D 'same' cross-correlations
    N, Cin, Cout, H, W = 2, 4, 3, 9, 7
    x = rng.standard_normal((N, Cin, H, W))
    w = rng.standard_normal((Cout, Cin, 3, 3))
    b = rng.standard_normal(Cout)
    y = R.conv3x3_fwd(x, w, b, relu=False)
    for n in range(N):
        for co in range(Cout):
            exp = b[co] + sum(scipy.signal.correlate2d(x[n, ci], w[co, ci], mode="same",
                                                       boundary="fill", fillvalue=0.0)
                              for ci in range(Cin))
            np.testing.assert_allclose(y[n, co], exp, rtol=0, atol=1e-12)


def test_conv_bruteforce_patch_and_relu_bias():
    N, Cin, Cout, H, W = 2, 6, 5, 8, 8
    x = rng.standard_normal((N, Cin, H, W))
    w = rng.standard_normal((Cout, Cin, 3, 3))
    b = rng.standard_normal(Cout)
    y = R.conv3x3_fwd(x, w, b, relu=True)
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
    for _ in range(50):
        n, co, h, ww = (rng.integers(N), rng.integers(Cout), rng.integers(H), rng.integers(W))
        patch = xp[n, :, h:h + 3, ww:ww + 3]
        pre = b[co] + float(np.dot(patch.ravel(), w[co].ravel()))
        assert abs(y[n, co, h, ww] - max(0.0, pre)) < 1e-12
    assert (y >= 0).all() and (y == 0).any()


def test_conv_linearity():
    x1, x2 = rng.standard_normal((2, 1, 3, 5, 5))
    w1, w2 = rng.standard_normal((2, 4, 3, 3, 3))
    a, b = 0.7, -1.3
    f = lambda x, w: R.conv3x3_fwd(x, w, None, relu=False)
    np.testing.assert_allclose(f(a * x1 + b * x2, w1), a * f(x1, w1) + b * f(x2, w1), atol=1e-12)
    np.testing.assert_allclose(f(x1, a * w1 + b * w2), a * f(x1, w1) + b * f(x1, w2), atol=1e-12)


# ------------------------------------------------------------ conv backward
def test_conv_adjoint_identities():
    N, Cin, Cout, H, W = 2, 3, 4, 6, 5
    x = rng.standard_normal((N, Cin, H, W))
    w = rng.standard_normal((Cout, Cin, 3, 3))
    g = rng.standard_normal((N, Cout, H, W))
    y = R.conv3x3_fwd(x, w, None, relu=False)
    dx = R.conv3x3_bwd_data(g, w)
    dw, db = R.conv3x3_bwd_weight(x, g)
    lhs = float((y * g).sum())
    assert abs(lhs - float((x * dx).sum())) < 1e-10
    assert abs(lhs - float((w * dw).sum())) < 1e-10
    np.testing.assert_allclose(db, g.sum(axis=(0, 2, 3)), atol=1e-12)


def test_conv_bwd_elementwise_vs_finite_differences():
    # the adjoint identity alone leaves e.g. a symmetric mistake possible: check element by element
    N, Cin, Cout, H, W = 1, 2, 2, 4, 4
    x = rng.standard_normal((N, Cin, H, W))
    w = rng.standard_normal((Cout, Cin, 3, 3))
    g = rng.standard_normal((N, Cout, H, W))
    loss = lambda x_, w_: float((R.conv3x3_fwd(x_, w_, None, relu=False) * g).sum())
    dx = R.conv3x3_bwd_data(g, w)
    dw, _ = R.conv3x3_bwd_weight(x, g)
    h = 1e-6
    for idx in np.ndindex(x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        assert abs((loss(xp, w) - loss(xm, w)) / (2 * h) - dx[idx]) < 1e-7
    for idx in np.ndindex(w.shape):
        wp, wm = w.copy(), w.copy()
        wp[idx] += h
        wm[idx] -= h
        assert abs((loss(x, wp) - loss(x, wm)) / (2 * h) - dw[idx]) < 1e-7


# --------------------------------------------------------------------- pool
def test_pool_bruteforce_and_argmax_rules():
    x = rng.standard_normal((2, 3, 6, 8))
    p, a = R.maxpool2x2(x)
    exp = x.reshape(2, 3, 3, 2, 4, 2).transpose(0, 1, 2, 4, 3, 5).reshape(2, 3, 3, 4, 4)
    assert np.array_equal(p, exp.max(-1))
    assert np.array_equal(a, exp.argmax(-1))        # numpy argmax = first maximum, order (0,0),(0,1),(1,0),(1,1)
    _, a0 = R.maxpool2x2(np.full((1, 1, 4, 4), 2.5))
    assert (a0 == 0).all()                           # ties -> first
    ramp = np.arange(16.0).reshape(1, 1, 4, 4)
    _, a3 = R.maxpool2x2(ramp)
    assert (a3 == 3).all()


def test_pool_bwd_scatter():
    x = rng.standard_normal((1, 2, 4, 6))
    p, a = R.maxpool2x2(x)
    dp = rng.standard_normal(p.shape)
    dx = R.maxpool2x2_bwd(dp, a)
    assert np.count_nonzero(dx) == dp.size
    # d/dx of sum(dp * pool(x)) is dp at the (untied) max location, zero elsewhere
    up = np.repeat(np.repeat(p, 2, 2), 2, 3)
    updp = np.repeat(np.repeat(dp, 2, 2), 2, 3)
    assert np.array_equal(dx, np.where(x == up, updp, 0.0))


# ----------------------------------------------------------------- fc/dense
def test_dense_matches_paper_definition_shape_10():
    # dense(W, x, b) = W*x + b with W 10x10, x and b length 10 (the paper's worked example shape)
    W = rng.standard_normal((10, 10))
    x = rng.standard_normal(10)
    b = rng.standard_normal(10)
    z = R.fc(x[None, :], W, b, relu=False)[0]
    np.testing.assert_allclose(z, W @ x + b, atol=1e-13)


def test_fc_triple_loop_and_relu():
    N, In, Out = 3, 4, 5
    a = rng.standard_normal((N, In))
    w = rng.standard_normal((Out, In))
    b = rng.standard_normal(Out)
    exp = np.zeros((N, Out))
    for n in range(N):
        for o in range(Out):
            s = b[o]
            for i in range(In):
                s += w[o, i] * a[n, i]
            exp[n, o] = s
    np.testing.assert_allclose(R.fc(a, w, b, relu=False), exp, atol=1e-13)
    np.testing.assert_allclose(R.fc(a, w, b, relu=True), np.maximum(exp, 0), atol=1e-13)


def test_fc_bwd_vs_matrix_identities():
    N, In, Out = 4, 6, 3
    a = rng.standard_normal((N, In))
    w = rng.standard_normal((Out, In))
    dz = rng.standard_normal((N, Out))
    dw, db, da = R.fc_bwd(a, w, dz)
    np.testing.assert_allclose(dw, dz.T @ a, atol=1e-13)
    np.testing.assert_allclose(db, dz.sum(0), atol=1e-13)
    np.testing.assert_allclose(da, dz @ w, atol=1e-13)


# ------------------------------------------------------------------ softmax
def test_softmax_golden_closed_form():
    lines = [l for l in open(os.path.join(GOLD, "softmax_values.txt")) if not l.startswith("#")]
    env = {"ln2": np.log(2.0), "ln3": np.log(3.0), "ln4": np.log(4.0)}
    logits = [env.get(t, None) if t in env else float(t) for t in lines[0].split()[1:]]
    probs = [float(t) for t in lines[1].split()[1:]]
    p = R.softmax(np.array([logits]))
    np.testing.assert_allclose(p[0], probs, atol=1e-15)


def test_softmax_properties():
    z = rng.standard_normal((5, 11)) * 4
    p = R.softmax(z)
    np.testing.assert_allclose(p.sum(1), 1.0, atol=1e-14)
    np.testing.assert_allclose(R.softmax(z + 123.0), p, atol=1e-13)
    np.testing.assert_allclose(R.softmax(np.zeros((2, 8))), 1 / 8, atol=1e-16)
    np.testing.assert_allclose(p, np.exp(z) / np.exp(z).sum(1, keepdims=True), atol=1e-14)  # paper's literal form
    big = np.array([[1000.0, 1000.0]])
    assert np.isfinite(R.softmax(big)).all()


def test_paper_standin_loss_sum_has_zero_logit_gradient():
    # backwards(m, x) = derivative(m -> sum(m(x)), m): rows of softmax sum to 1, so the gradient
    # of the sum with respect to the logits vanishes identically.
    z = rng.standard_normal((3, 7))
    p = R.softmax(z)
    dz = R.softmax_vjp(p, np.ones_like(p))
    assert np.abs(dz).max() < 1e-15


def test_softmax_vjp_vs_finite_differences():
    z = rng.standard_normal((2, 5))
    u = rng.standard_normal((2, 5))
    dz = R.softmax_vjp(R.softmax(z), u)
    h = 1e-6
    for idx in np.ndindex(z.shape):
        zp, zm = z.copy(), z.copy()
        zp[idx] += h
        zm[idx] -= h
        fd = ((R.softmax(zp) - R.softmax(zm)) * u).sum() / (2 * h)
        assert abs(fd - dz[idx]) < 1e-8


def test_xent_closed_forms_and_gradient():
    K = 6
    p = R.softmax(np.zeros((4, K)))
    loss, dz = R.softmax_xent(p, np.array([0, 1, 2, 3]))
    assert abs(loss - np.log(K)) < 1e-14
    z = rng.standard_normal((3, K))
    labels = np.array([5, 0, 2])
    f = lambda zz: R.softmax_xent(R.softmax(zz), labels)[0]
    _, dz = R.softmax_xent(R.softmax(z), labels)
    h = 1e-6
    for idx in np.ndindex(z.shape):
        zp, zm = z.copy(), z.copy()
        zp[idx] += h
        zm[idx] -= h
        assert abs((f(zp) - f(zm)) / (2 * h) - dz[idx]) < 1e-8
    np.testing.assert_allclose(dz.sum(1), 0, atol=1e-15)


def test_relu_bwd_and_sgd():
    y = np.array([0.0, 1.0, 0.0, 2.0])
    dy = np.array([5.0, 6.0, 7.0, 8.0])
    assert np.array_equal(R.relu_bwd(y, dy), [0.0, 6.0, 0.0, 8.0])
    th = np.array([1.0, 2.0])
    assert np.allclose(R.sgd(th, np.array([10.0, -10.0]), 0.01), [0.9, 2.1])
    assert np.array_equal(th, [1.0, 2.0])


# ------------------------------------------------------- composed tiny net
def test_small_chain_backward_vs_finite_differences():
    # conv+relu -> conv+relu -> pool -> dense -> softmax-xent, every parameter and input element
    r = np.random.default_rng(7)
    N, H, W = 2, 6, 6
    x = r.standard_normal((N, 2, H, W))
    w1 = r.standard_normal((3, 2, 3, 3)) * 0.5
    b1 = r.standard_normal(3) * 0.1
    w2 = r.standard_normal((4, 3, 3, 3)) * 0.5
    b2 = r.standard_normal(4) * 0.1
    wf = r.standard_normal((5, 4 * 3 * 3)) * 0.3
    bf = r.standard_normal(5) * 0.1
    labels = np.array([1, 4])

    def fwd(x, w1, b1, w2, b2, wf, bf):
        y1 = R.conv3x3_fwd(x, w1, b1, True)
        y2 = R.conv3x3_fwd(y1, w2, b2, True)
        p, a = R.maxpool2x2(y2)
        z = R.fc(p.reshape(N, -1), wf, bf, False)
        pr = R.softmax(z)
        return y1, y2, p, a, z, pr

    y1, y2, p, a, z, pr = fwd(x, w1, b1, w2, b2, wf, bf)
    _, dz = R.softmax_xent(pr, labels)
    dwf, dbf, dflat = R.fc_bwd(p.reshape(N, -1), wf, dz)
    d = R.maxpool2x2_bwd(dflat.reshape(p.shape), a)
    g2 = R.relu_bwd(y2, d)
    dw2, db2 = R.conv3x3_bwd_weight(y1, g2)
    g1 = R.relu_bwd(y1, R.conv3x3_bwd_data(g2, w2))
    dw1, db1 = R.conv3x3_bwd_weight(x, g1)
    dx = R.conv3x3_bwd_data(g1, w1)

    params = [x, w1, b1, w2, b2, wf, bf]
    grads = [dx, dw1, db1, dw2, db2, dwf, dbf]
    loss = lambda ps: R.softmax_xent(fwd(*ps)[5], labels)[0]
    h = 1e-6
    checked = 0
    for k, (par, gr) in enumerate(zip(params, grads)):
        for idx in np.ndindex(par.shape):
            pp = [q.copy() for q in params]
            pm = [q.copy() for q in params]
            pp[k][idx] += h
            pm[k][idx] -= h
            fp, fm = fwd(*pp), fwd(*pm)
            # skip samples where the perturbation crosses a ReLU kink or flips a pool argmax
            if any(((u > 0) != (v > 0)).any() for u, v in ((fp[0], fm[0]), (fp[1], fm[1]))) or \
                    (fp[3] != fm[3]).any():
                continue
            fd = (R.softmax_xent(fp[5], labels)[0] - R.softmax_xent(fm[5], labels)[0]) / (2 * h)
            assert abs(fd - gr[idx]) < 1e-7 * max(1.0, abs(gr[idx])), (k, idx, fd, gr[idx])
            checked += 1
    assert checked > 300


# ------------------------------------------------------------- whole model
def _golden_counts():
    out = {}
    for line in open(os.path.join(GOLD, "hlo_counts.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, f, b = line.split()
        out[name] = (int(f), int(b))
    return out


def test_model_structure_matches_paper_counts(monkeypatch):
    from paper_1810_09868_amd import synth
    calls = {"conv": 0, "pool": 0, "fc": 0, "wgrad": 0, "dgrad": 0, "poolb": 0, "fcb": 0}

    def wrap(name, key):
        orig = getattr(R, name)

        def f(*a, **k):
            calls[key] += 1
            return orig(*a, **k)
        monkeypatch.setattr(R, name, f)
    for n, k in [("conv3x3_fwd", "conv"), ("maxpool2x2", "pool"), ("fc", "fc"),
                 ("conv3x3_bwd_weight", "wgrad"), ("conv3x3_bwd_data", "dgrad"),
                 ("maxpool2x2_bwd", "poolb"), ("fc_bwd", "fcb")]:
        wrap(n, k)
    inp = synth.vgg19_inputs(1, 32, 32, 16, 10, seed=3)
    R.vgg19_train_step(inp.x, inp.labels, inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    gold = _golden_counts()
    assert calls["conv"] == gold["convolution"][0] == 16
    assert calls["pool"] == gold["reduce-window"][0] == 5
    assert calls["fc"] == gold["dot"][0] == 3
    # backward column counts forward ops again: 47 = 16 fwd + 16 weight grads + 15 data grads
    assert calls["conv"] + calls["wgrad"] + calls["dgrad"] == gold["convolution"][1] == 47
    assert calls["dgrad"] == 15 and gold["reverse"][1] == 16
    assert calls["poolb"] == gold["select-and-scatter"][1] == 5
    assert calls["fc"] + 2 * calls["fcb"] == gold["dot"][1] == 9
    # 23 maxima = 16 conv ReLU + 2 dense ReLU + 5 pool reducers
    assert 16 + 2 + calls["pool"] == gold["maximum"][0]


def test_tiny_vgg19_forward_properties_and_train_step_fd():
    from paper_1810_09868_amd import synth
    inp = synth.vgg19_inputs(1, 32, 32, 32, 10, seed=1)
    cw = [w.astype(np.float64) for w in inp.conv_w]
    cb = [b.astype(np.float64) for b in inp.conv_b]
    fw = [w.astype(np.float64) for w in inp.fc_w]
    fb = [b.astype(np.float64) for b in inp.fc_b]
    x = inp.x.astype(np.float64)
    res = R.vgg19_train_step(x, inp.labels, cw, cb, fw, fb, lr=0.01)
    assert res["logits"].shape == (1, 10)
    np.testing.assert_allclose(res["probs"].sum(1), 1.0, atol=1e-14)
    assert abs(res["loss"] + np.log(res["probs"][0, inp.labels[0]])) < 1e-14
    np.testing.assert_allclose(res["new_conv_w"][3], cw[3] - 0.01 * res["dconv_w"][3], atol=1e-16)
    np.testing.assert_allclose(res["new_fc_b"][2], fb[2] - 0.01 * res["dfc_b"][2], atol=1e-16)

    def loss_with(kind, l, idx, delta):
        cw2, cb2, fw2, fb2 = [a.copy() for a in cw], [a.copy() for a in cb], \
            [a.copy() for a in fw], [a.copy() for a in fb]
        {"cw": cw2, "cb": cb2, "fw": fw2, "fb": fb2}[kind][l][idx] += delta
        f = R.vgg19_forward(x, cw2, cb2, fw2, fb2)
        return R.softmax_xent(f["probs"], inp.labels)[0]

    r = np.random.default_rng(5)
    h = 1e-5
    picks = [("cw", 0), ("cb", 0), ("cw", 1), ("cw", 4), ("cb", 7), ("cw", 8), ("cw", 15), ("cb", 15),
             ("fw", 0), ("fb", 0), ("fw", 1), ("fw", 2), ("fb", 2)]
    gname = {"cw": "dconv_w", "cb": "dconv_b", "fw": "dfc_w", "fb": "dfc_b"}
    for kind, l in picks:
        g = res[gname[kind]][l]
        # choose the entry with the largest gradient so the FD signal is well above rounding
        idx = np.unravel_index(np.argmax(np.abs(g)), g.shape)
        fd = (loss_with(kind, l, idx, h) - loss_with(kind, l, idx, -h)) / (2 * h)
        assert abs(fd - g[idx]) < 2e-5 * max(abs(g[idx]), 1e-3), (kind, l, idx, fd, g[idx])


def test_round_bf16_closed_forms_and_library_conversion():
    # bfloat16 keeps 8 significant bits (format definition): representable values are fixed points,
    # halves go to the even neighbour, everything else to the nearest
    rep = np.array([0.0, 1.0, -1.0, 0.5, 1.5, 255.0, 1.0 + 2.0 ** -7, -3.0 * 2.0 ** -20, 2.0 ** 100])
    assert np.array_equal(R.round_bf16(rep), rep)
    ulp = 2.0 ** -7                                             # spacing in [1, 2)
    assert R.round_bf16(np.array([1.0 + 0.5 * ulp]))[0] == 1.0                 # tie -> even (mantissa 0)
    assert R.round_bf16(np.array([1.0 + 1.5 * ulp]))[0] == 1.0 + 2.0 * ulp     # tie -> even (mantissa 2)
    assert R.round_bf16(np.array([1.0 + 0.49 * ulp]))[0] == 1.0
    assert R.round_bf16(np.array([1.0 + 0.51 * ulp]))[0] == 1.0 + ulp
    assert R.round_bf16(np.array([-(1.0 + 0.51 * ulp)]))[0] == -(1.0 + ulp)
    assert R.round_bf16(np.array([2.0 - 0.25 * ulp]))[0] == 2.0                # rounds up into the next binade
    # an independent conversion routine on random float32 values
    import torch
    rng = np.random.default_rng(5)
    v = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(R.round_bf16(v), want)
    r = R.round_bf16(v)
    assert np.all(np.abs(r - v) <= np.abs(v) * 2.0 ** -8)        # relative error bound of 8 significant bits
    assert np.array_equal(R.round_bf16(r), r)                    # idempotent


def test_rounded_operand_model_reduces_to_plain_model_on_representable_data():
    # With every operand already a bfloat16 value only the rounding of layer outputs differs from the
    # plain model; with an identity "rounding" nothing does.  Pins that operand_round touches no sums.
    from paper_1810_09868_amd import synth
    inp = synth.tiny_config(seed=4)
    f64 = lambda lst: [a.astype(np.float64) for a in lst]
    plain = R.vgg19_train_step(inp.x, inp.labels, f64(inp.conv_w), f64(inp.conv_b), f64(inp.fc_w), f64(inp.fc_b), lr=0.01)
    ident = R.vgg19_train_step(inp.x, inp.labels, f64(inp.conv_w), f64(inp.conv_b), f64(inp.fc_w), f64(inp.fc_b), lr=0.01,
                               operand_round=lambda a: a)
    assert np.array_equal(plain["logits"], ident["logits"])
    for k in ("dconv_w", "dfc_w", "new_conv_w", "new_fc_b"):
        for a, b in zip(plain[k], ident[k]):
            assert np.array_equal(a, b)
    # bfloat16 operands: every product operand the model kept is a fixed point of the rounding, the
    # result stays within the format's error of the plain model, and the update moves the unrounded parameters
    rb = R.vgg19_train_step(inp.x, inp.labels, f64(inp.conv_w), f64(inp.conv_b), f64(inp.fc_w), f64(inp.fc_b), lr=0.01,
                            operand_round=R.round_bf16)
    f = rb["fwd"]
    for a in list(f["conv_in"]) + list(f["conv_out"]) + [f["z1"], f["z2"], f["flat"]]:
        assert np.array_equal(R.round_bf16(a), a)
    assert not np.array_equal(R.round_bf16(f["logits"]), f["logits"])
    scale = np.abs(plain["logits"]).max()
    err = np.abs(rb["logits"] - plain["logits"]).max() / scale
    assert 1e-5 < err < 2e-2
    for l in range(16):
        upd = rb["new_conv_w"][l] - inp.conv_w[l].astype(np.float64)
        np.testing.assert_allclose(upd, -0.01 * rb["dconv_w"][l], rtol=0, atol=1e-12 * max(1.0, np.abs(upd).max()))
