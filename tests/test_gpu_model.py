"""Whole-model parity of the HIP path against the fp64 CPU oracle: the tiny
VGG19 (forward in both dtypes, training step), the single-layer
microbenchmark shape, and the full 224x224 batch-100 configurations on sampled
images / via batch linearity."""
import numpy as np
import pytest
import torch

from oracle import vgg_ref as R
from paper_1810_09868_amd import binding as B
from paper_1810_09868_amd import synth
from paper_1810_09868_amd.model import Vgg19

from gpu_util import TDT, TOL, dev, from_nhwc, max_rel_err, to_nhwc, ws_bytes

pytestmark = pytest.mark.gpu


def _f64(lst):
    return [a.astype(np.float64) for a in lst]


# A ReLU or a window maximum decided on a value within fp32 rounding of the decision boundary can
# come out differently on the GPU (fp32) and in the oracle (fp64); one such flip changes a gradient
# tensor by about 1/sqrt(number of active elements), far more than 1e-4.  BAND is the relative
# distance from the boundary below which a decision is treated as not unique.
BAND = 2e-5


def _gradient_check(g, ref, inp, tol):
    """Every gradient tensor within tol of the oracle's, plus twice the spread of the oracle's own
    gradient when the decisions inside BAND are taken the other way.  A tensor that no ambiguous
    decision reaches (always the last dense layer; every tensor when there is none) has zero spread
    and is held to tol alone."""
    keys = (("conv_w", "dconv_w"), ("conv_b", "dconv_b"), ("fc_w", "dfc_w"), ("fc_b", "dfc_b"))
    f = ref["fwd"]
    alts = [R.vgg19_gradients(f, inp.labels, _f64(inp.conv_w), _f64(inp.fc_w), mask_shift=+BAND),
            R.vgg19_gradients(f, inp.labels, _f64(inp.conv_w), _f64(inp.fc_w), mask_shift=-BAND)]
    if R.decision_margins(f)["pool"] < BAND:
        alts.append(R.vgg19_gradients(f, inp.labels, _f64(inp.conv_w), _f64(inp.fc_w), pool_second_within=BAND))
    worst = 0.0
    spread = {}
    for k, rk in keys:
        for l, (a, b) in enumerate(zip(g[k], ref[rk])):
            a = a.cpu().numpy().astype(np.float64)
            scale = np.abs(b).max()
            spread[(k, l)] = 2.0 * sum(np.abs(alt[rk][l] - b).max() for alt in alts)
            e = np.abs(a - b).max()
            worst = max(worst, e / scale)
            assert e <= tol * scale + spread[(k, l)], (k, l, e / scale, spread[(k, l)] / scale)
    return worst, spread


def _updated_params_check(after, ref, spread, tol, lr):
    """theta_new within tol of the oracle's, plus lr times the gradient's decision spread."""
    for k, rk in (("conv_w", "new_conv_w"), ("conv_b", "new_conv_b"), ("fc_w", "new_fc_w"), ("fc_b", "new_fc_b")):
        for l, (a, b) in enumerate(zip(after[k], ref[rk])):
            e = np.abs(a.astype(np.float64) - b).max()
            assert e <= tol * np.abs(b).max() + lr * spread[(k, l)], (k, l, e)


def _check_probs(probs, logits, ref, dtype):
    """fp32: probabilities to the stated relative tolerance.  bf16: the stated tolerance is on the
    logits; a logit deviation of at most d moves every softmax output by a factor within
    exp(+-2d), so |p - p_ref| <= p_ref * (exp(2d) - 1) with d the deviation actually measured."""
    if dtype == B.F32:
        assert max_rel_err(probs, ref["probs"]) <= TOL[dtype]
        return
    d = float(np.abs(logits.astype(np.float64) - ref["logits"]).max())
    bound = ref["probs"] * np.expm1(2 * d) + 1e-7
    assert (np.abs(probs.astype(np.float64) - ref["probs"]) <= bound).all()


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
def test_tiny_vgg19_forward(dtype):
    inp = synth.tiny_config(seed=0)
    ref = R.vgg19_forward(inp.x, inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    m = Vgg19(dtype, 2, 32, 32, 512, 10)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    m.forward(dev(inp.x))
    torch.cuda.synchronize()
    assert max_rel_err(m.logits.cpu().numpy(), ref["logits"]) <= TOL[dtype]
    _check_probs(m.probs.cpu().numpy(), m.logits.cpu().numpy(), ref, dtype)
    np.testing.assert_allclose(m.probs.sum(1).cpu().numpy(), 1.0, atol=1e-5)


def test_tiny_vgg19_train_step_fp32():
    inp = synth.tiny_config(seed=0)
    ref = R.vgg19_train_step(inp.x, inp.labels, _f64(inp.conv_w), _f64(inp.conv_b), _f64(inp.fc_w),
                             _f64(inp.fc_b), lr=0.01)
    m = Vgg19(B.F32, 2, 32, 32, 512, 10, lr=0.01, training=True)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    before = m.unpack()
    for k, src in (("conv_w", inp.conv_w), ("conv_b", inp.conv_b), ("fc_w", inp.fc_w), ("fc_b", inp.fc_b)):
        for a, b in zip(before[k], src):
            assert np.array_equal(a, b)                    # pack -> unpack is the identity
    g = m.train_step(dev(inp.x), dev(inp.labels), want_grads=True)
    torch.cuda.synchronize()
    tol = TOL[B.F32]
    assert abs(m.loss.item() - ref["loss"]) <= tol * abs(ref["loss"])
    assert max_rel_err(m.logits.cpu().numpy(), ref["logits"]) <= tol
    worst, spread = _gradient_check(g, ref, inp, tol)
    print("worst gradient error", worst)
    after = m.unpack()
    _updated_params_check(after, ref, spread, tol, 0.01)
    for k in ("conv_w", "conv_b", "fc_w", "fc_b"):
        for l, a in enumerate(after[k]):
            # the applied update is theta - lr * (the gradient the step reported), to fp32 rounding
            upd = a.astype(np.float64) - before[k][l].astype(np.float64)
            want = -0.01 * g[k][l].cpu().numpy().astype(np.float64)
            assert np.abs(upd - want).max() <= 2e-7 * np.abs(before[k][l]).max() + 1e-6 * np.abs(want).max(), (k, l)


def test_conv_microbenchmark_shape_sampled_images():
    # 128 -> 256 channels, 56x56, batch 100 on the GPU; the oracle recomputes three of the images
    N, H, W, Cin, Cout = 100, 56, 56, 128, 256
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=0)
    for dtype in (B.F32, B.BF16):
        x = to_nhwc(d["x"], dtype)
        wp = torch.empty((9, Cout, Cin), dtype=TDT[dtype], device="cuda")
        B.vgg_conv_pack_weights(dtype, Cin, Cout, dev(d["w"]), wp, 0)
        y = torch.empty((N, H, W, Cout), dtype=TDT[dtype], device="cuda")
        B.vgg_conv3x3_fwd(dtype, N, H, W, Cin, Cout, x, wp, dev(d["b"]), y, 1, None)
        torch.cuda.synchronize()
        for n in (0, 57, 99):
            ref = R.conv3x3_fwd(d["x"][n:n + 1], d["w"], d["b"], relu=True)
            assert max_rel_err(from_nhwc(y[n:n + 1]), ref) <= TOL[dtype], (dtype, n)


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
def test_full_vgg19_forward_batch100_sampled_images(dtype):
    N = 100
    inp = synth.full_config(N, seed=0, with_labels=False)
    m = Vgg19(dtype, N, 224, 224, 4096, 1000)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    m.forward(dev(inp.x))
    torch.cuda.synchronize()
    logits = m.logits.cpu().numpy()
    probs = m.probs.cpu().numpy()
    assert np.isfinite(logits).all()
    np.testing.assert_allclose(probs.sum(1), 1.0, atol=1e-4)
    # images from every part of the batch: a launch's workgroups run out of order across the chip, so a
    # buffer that is read and written by the same launch would corrupt some images and not others
    for n in (0, 1, 5, 13, 24, 38, 57, 76, 99):
        ref = R.vgg19_forward(inp.x[n:n + 1], inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
        assert max_rel_err(logits[n:n + 1], ref["logits"]) <= TOL[dtype], n
        _check_probs(probs[n:n + 1], logits[n:n + 1], ref, dtype)


@pytest.mark.parametrize("N", [1, 10])
@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
def test_full_vgg19_forward_small_batches(dtype, N):
    # the other batch sizes of the paper's timing table (Table "timing": 1, 10 and 100 images): the last
    # stages then have fewer pixels than one workgroup tile per CU
    inp = synth.full_config(N, seed=3, with_labels=False)
    m = Vgg19(dtype, N, 224, 224, 4096, 1000)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    m.forward(dev(inp.x))
    torch.cuda.synchronize()
    logits = m.logits.cpu().numpy()
    probs = m.probs.cpu().numpy()
    for n in sorted({0, N // 3, N - 1}):
        ref = R.vgg19_forward(inp.x[n:n + 1], inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
        assert max_rel_err(logits[n:n + 1], ref["logits"]) <= TOL[dtype], n
        _check_probs(probs[n:n + 1], logits[n:n + 1], ref, dtype)


def test_full_vgg19_train_step_224_vs_oracle_batch2():
    inp = synth.vgg19_inputs(2, 224, 224, 4096, 1000, seed=1)
    ref = R.vgg19_train_step(inp.x, inp.labels, _f64(inp.conv_w), _f64(inp.conv_b), _f64(inp.fc_w),
                             _f64(inp.fc_b), lr=0.01)
    m = Vgg19(B.F32, 2, 224, 224, 4096, 1000, lr=0.01, training=True)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    g = m.train_step(dev(inp.x), dev(inp.labels), want_grads=True)
    torch.cuda.synchronize()
    tol = TOL[B.F32]
    assert abs(m.loss.item() - ref["loss"]) <= tol * abs(ref["loss"])
    assert max_rel_err(m.logits.cpu().numpy(), ref["logits"]) <= tol
    worst, spread = _gradient_check(g, ref, inp, tol)
    print("worst gradient error", worst)
    _updated_params_check(m.unpack(), ref, spread, tol, 0.01)


def test_full_vgg19_train_step_batch100_is_mean_of_chunks():
    # The loss is a mean over images, so the batch-100 gradient equals the mean of the gradients of
    # five batch-20 steps from the same parameters (a property that holds at any size); the batch-2
    # test above ties the same kernels at the same spatial sizes to the oracle.  The chunks must run
    # the same arithmetic per image as the full batch: a ReLU or pooling decision that rounding
    # flips moves a gradient by far more than the tolerance.  Halves do (below roughly 40 images
    # the 14x14 layers split their contraction over several workgroups, another summation order).
    N, chunk = 100, 50
    inp = synth.full_config(N, seed=2)
    big = Vgg19(B.F32, N, 224, 224, 4096, 1000, lr=0.01, training=True)
    big.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    gb = big.train_step(dev(inp.x), dev(inp.labels), want_grads=True)
    torch.cuda.synchronize()
    loss_big = big.loss.item()
    logits_big = big.logits.cpu().numpy()
    gb = {k: [a.double().cpu() for a in v] for k, v in gb.items()}
    new_big = big.unpack()
    del big
    torch.cuda.empty_cache()
    small = Vgg19(B.F32, chunk, 224, 224, 4096, 1000, lr=0.01, training=True)
    acc = None
    losses = []
    for c in range(N // chunk):
        sl = slice(c * chunk, (c + 1) * chunk)
        small.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
        g = small.train_step(dev(inp.x[sl]), dev(inp.labels[sl]), want_grads=True)
        torch.cuda.synchronize()
        losses.append(small.loss.item())
        assert max_rel_err(small.logits.cpu().numpy(), logits_big[sl]) <= 1e-5
        g = {k: [a.double().cpu() for a in v] for k, v in g.items()}
        acc = g if acc is None else {k: [a + b for a, b in zip(acc[k], g[k])] for k in acc}
    assert abs(np.mean(losses) - loss_big) <= 1e-5 * abs(loss_big)
    for k in acc:
        for l, (a, b) in enumerate(zip(acc[k], gb[k])):
            assert max_rel_err(b.numpy(), (a / (N // chunk)).numpy()) <= TOL[B.F32], (k, l)
    # SGD applied: theta_new = theta - lr * grad
    for k, src in (("conv_w", inp.conv_w), ("fc_b", inp.fc_b)):
        for l in range(len(src)):
            upd = new_big[k][l].astype(np.float64) - src[l].astype(np.float64)
            assert max_rel_err(upd, -0.01 * gb[k][l].numpy()) <= 1e-3, (k, l)


def test_training_loop_as_one_graph_matches_eager_steps():
    # K steps recorded once and replayed as a single launch must leave exactly the parameters that K eager
    # steps leave (every kernel is deterministic); replayed several times, with eager work and
    # synchronisations in between, and checked after every replay.
    cfg = synth.tiny_config(seed=5)
    K = 3
    eager = Vgg19(B.F32, 2, 32, 32, 512, 10, lr=0.01, training=True)
    graph = Vgg19(B.F32, 2, 32, 32, 512, 10, lr=0.01, training=True)
    for m in (eager, graph):
        m.pack(cfg.conv_w, cfg.conv_b, cfg.fc_w, cfg.fc_b)
    x, lab = dev(cfg.x), dev(cfg.labels)
    eager.train_step(x, lab)
    graph.train_step(x, lab)      # warm-up before capture (and both models stay in step)
    torch.cuda.synchronize()
    g = graph.capture_train_steps(x, lab, K)
    # capture only records: the parameters have not moved
    assert torch.equal(eager.packed, graph.packed)
    for replay in range(3):
        g.replay()
        for _ in range(K):
            eager.train_step(x, lab)
        torch.cuda.synchronize()
        assert torch.equal(eager.packed, graph.packed), replay
        assert torch.equal(eager.loss, graph.loss), replay
        assert torch.equal(eager.logits, graph.logits), replay
        # unrelated eager work between the replays
        scratch = torch.rand((1 << 16,), device="cuda").sum().item()
        assert scratch > 0
