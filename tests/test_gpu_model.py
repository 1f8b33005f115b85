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


def _gradient_check(g, ref, inp, tol, rd=None):
    """Every gradient tensor within tol of the oracle's, plus twice the spread of the oracle's own
    gradient when the decisions inside BAND are taken the other way.  A tensor that no ambiguous
    decision reaches (always the last dense layer; every tensor when there is none) has zero spread
    and is held to tol alone."""
    keys = (("conv_w", "dconv_w"), ("conv_b", "dconv_b"), ("fc_w", "dfc_w"), ("fc_b", "dfc_b"))
    f = ref["fwd"]
    alts = [R.vgg19_gradients(f, inp.labels, _f64(inp.conv_w), _f64(inp.fc_w), mask_shift=+BAND, operand_round=rd),
            R.vgg19_gradients(f, inp.labels, _f64(inp.conv_w), _f64(inp.fc_w), mask_shift=-BAND, operand_round=rd)]
    if R.decision_margins(f)["pool"] < BAND:
        alts.append(R.vgg19_gradients(f, inp.labels, _f64(inp.conv_w), _f64(inp.fc_w), pool_second_within=BAND,
                                      operand_round=rd))
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


def _bf16_train_step_vs_oracle(inp, N, H, W, hidden, classes):
    """bf16 training step against the oracle run with bfloat16 operands (the accelerator's matrix-unit
    precision).  Rounding to 8 bits after every layer is a chaotic quantiser: two correct
    implementations that sum in a different order disagree by one bf16 step on some activations after
    the first layer and, nineteen layers on, take different ReLU and pooling decisions on a fraction of
    a percent of the units.  Loss, logits and the last dense layer's gradient (which no decision
    reaches) are held to the bf16 tolerance; every other gradient tensor can only be held to an
    aggregate bound here (wrong wiring gives a relative L2 error near or above 1), and the per-layer
    kernels are held to the tolerance on the oracle's own tensors in the test below."""
    ref = R.vgg19_train_step(inp.x, inp.labels, _f64(inp.conv_w), _f64(inp.conv_b), _f64(inp.fc_w), _f64(inp.fc_b),
                             lr=0.01, operand_round=R.round_bf16)
    m = Vgg19(B.BF16, N, H, W, hidden, classes, lr=0.01, training=True)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    before = m.unpack()
    for k, src in (("conv_w", inp.conv_w), ("conv_b", inp.conv_b), ("fc_w", inp.fc_w), ("fc_b", inp.fc_b)):
        for a, b in zip(before[k], src):
            assert np.array_equal(a, b)                    # the fp32 master copy is what unpack returns
    g = m.train_step(dev(inp.x), dev(inp.labels), want_grads=True)
    torch.cuda.synchronize()
    tol = TOL[B.BF16]
    assert abs(m.loss.item() - ref["loss"]) <= tol * abs(ref["loss"])
    assert max_rel_err(m.logits.cpu().numpy(), ref["logits"]) <= tol
    assert max_rel_err(g["fc_w"][2].cpu().numpy(), ref["dfc_w"][2]) <= tol
    assert max_rel_err(g["fc_b"][2].cpu().numpy(), ref["dfc_b"][2]) <= tol
    worst = 0.0
    for k, rk in (("conv_w", "dconv_w"), ("conv_b", "dconv_b"), ("fc_w", "dfc_w"), ("fc_b", "dfc_b")):
        for l, (a, b) in enumerate(zip(g[k], ref[rk])):
            e = np.linalg.norm(a.cpu().numpy().astype(np.float64) - b) / np.linalg.norm(b)
            worst = max(worst, e)
            assert e <= 0.4, (k, l, e)
    print("worst relative L2 gradient error", worst)
    after = m.unpack()
    for k in ("conv_w", "conv_b", "fc_w", "fc_b"):
        for l, a in enumerate(after[k]):
            # the master parameters moved by -lr * (the gradient the step reported), to fp32 rounding
            upd = a.astype(np.float64) - before[k][l].astype(np.float64)
            want = -0.01 * g[k][l].cpu().numpy().astype(np.float64)
            assert np.abs(upd - want).max() <= 2e-7 * np.abs(before[k][l]).max() + 1e-6 * np.abs(want).max(), (k, l)
    # the bf16 parameters the next forward pass reads are the rounded new master parameters: packing the
    # master values afresh gives the same working block, bit for bit
    m2 = Vgg19(B.BF16, N, H, W, hidden, classes)
    m2.pack(after["conv_w"], after["conv_b"], after["fc_w"], after["fc_b"])
    nb = m2.packed.numel()
    assert torch.equal(m.packed[:nb], m2.packed)


def _bf16_backward_kernels_on_oracle_tensors(inp):
    """Every convolution layer's bf16 weight- and data-gradient launch, and every pool's backward, on
    the tensors of the oracle's own bf16-operand pass (inputs from the oracle, so both sides start
    from identical values and no decision is left to rounding): held to the bf16 tolerance."""
    rd = R.round_bf16
    cw = _f64(inp.conv_w)
    f = R.vgg19_forward(inp.x, cw, _f64(inp.conv_b), _f64(inp.fc_w), _f64(inp.fc_b), keep=True, operand_round=rd)
    _, dlogits = R.softmax_xent(f["probs"], inp.labels)
    _, _, dz2 = R.fc_bwd(f["z2"], inp.fc_w[2], dlogits)
    dz2 = np.where(f["fc_pre"][1] > 0, dz2, 0.0)
    _, _, dz1 = R.fc_bwd(f["z1"], inp.fc_w[1], dz2)
    dz1 = np.where(f["fc_pre"][0] > 0, dz1, 0.0)
    _, _, dflat = R.fc_bwd(f["flat"], inp.fc_w[0], dz1)
    d = rd(dflat.reshape(f["pool5"].shape))
    tol = TOL[B.BF16]
    worst = 0.0
    for l in range(15, -1, -1):
        x = f["conv_in"][l]
        N, Cin, H, W = x.shape
        Cout = cw[l].shape[0]
        if l in (1, 3, 7, 11, 15):
            arg = f["pool_arg"][l]
            want = R.maxpool2x2_bwd(d, arg)
            dy = to_nhwc(d, B.BF16)
            a = torch.from_numpy(np.ascontiguousarray(arg.transpose(0, 2, 3, 1))).cuda()
            dx = torch.empty((N, H, W, Cout), dtype=torch.bfloat16, device="cuda")
            B.vgg_maxpool2x2_bwd(B.BF16, N, H, W, Cout, dy, a, dx)
            torch.cuda.synchronize()
            assert np.array_equal(from_nhwc(dx), want), l      # routing only: exact
            d = want
        gmask = np.where(f["conv_pre"][l] > 0, d, 0.0)         # bf16 values
        dw_ref, db_ref = R.conv3x3_bwd_weight(x, gmask)
        xg, gg = to_nhwc(x, B.BF16), to_nhwc(gmask, B.BF16)
        cp = B.vgg_padded_channels(B.BF16, Cin)
        dwp = torch.empty((9, Cout, cp), device="cuda")
        db = torch.empty((Cout,), device="cuda")
        ws = ws_bytes(B.vgg_conv3x3_bwd_weight_workspace_bytes(B.BF16, N, H, W, Cin, Cout))
        B.vgg_conv3x3_bwd_weight(B.BF16, N, H, W, Cin, Cout, xg, gg, dwp, db, ws)
        torch.cuda.synchronize()
        dw = dwp[:, :, :Cin].reshape(3, 3, Cout, Cin).permute(2, 3, 0, 1).cpu().numpy()
        e = max(max_rel_err(dw, dw_ref), max_rel_err(db.cpu().numpy(), db_ref))
        worst = max(worst, e)
        assert e <= tol, ("weight gradient", l, e)
        if l == 0:
            break
        want = rd(R.conv3x3_bwd_data(gmask, rd(cw[l])))
        wtf = torch.empty((9, Cin, B.vgg_padded_channels(B.BF16, Cout)), dtype=torch.bfloat16, device="cuda")
        B.vgg_conv_pack_weights(B.BF16, Cin, Cout, dev(inp.conv_w[l]), wtf, 1)
        dxg = torch.empty((N, H, W, Cin), dtype=torch.bfloat16, device="cuda")
        ws = ws_bytes(B.vgg_conv3x3_bwd_data_workspace_bytes(B.BF16, N, H, W, Cin, Cout))
        B.vgg_conv3x3_bwd_data(B.BF16, N, H, W, Cin, Cout, gg, wtf, xg, dxg, ws)
        torch.cuda.synchronize()
        e = max_rel_err(from_nhwc(dxg), want * (x > 0))
        worst = max(worst, e)
        assert e <= tol, ("data gradient", l, e)
        d = want                                               # (the next layer's mask is applied to it there)
    return worst


_CONV = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256), (256, 256),
         (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
_POOLED = (1, 3, 7, 11, 15)


def _bf16_step_from_single_op_calls(inp, N, H, W, hidden, classes):
    """The 38 gradients of one bf16 training step, computed by chaining the single-operation entry points
    (each held to the oracle in test_gpu_ops.py and in the per-layer test above) from Python in the order
    the model-level call documents.  Same kernels, same shapes, deterministic sums: vgg19_train_step must
    reproduce these bit for bit, which pins its buffer plumbing without any tolerance."""
    bf = torch.bfloat16
    ws = lambda n: ws_bytes(n)
    x = torch.empty((N, H, W, 32), dtype=bf, device="cuda")
    B.vgg_nchw_to_nhwc(B.BF16, N, 3, H, W, 32, dev(inp.x), x)
    acts_in, args, sizes = [], {}, []
    h, w = H, W
    cur = x
    for l, (ci, co) in enumerate(_CONV):
        acts_in.append(cur)
        sizes.append((h, w))
        cp = B.vgg_padded_channels(B.BF16, ci)
        wp = torch.empty((9, co, cp), dtype=bf, device="cuda")
        B.vgg_conv_pack_weights(B.BF16, ci, co, dev(inp.conv_w[l]), wp, 0)
        wsb = ws(B.vgg_conv3x3_fwd_workspace_bytes(B.BF16, N, h, w, cp, co))
        if l in _POOLED:
            pooled = torch.empty((N, h // 2, w // 2, co), dtype=bf, device="cuda")
            arg = torch.empty((N, h // 2, w // 2, co), dtype=torch.uint8, device="cuda")
            if l > 0 and h % 16 == 0 and w % 16 == 0:      # pool taken in the convolution's epilogue
                B.vgg_conv3x3_fwd_pool(B.BF16, N, h, w, cp, co, cur, wp, dev(inp.conv_b[l]), None, pooled, 1, wsb, argmax=arg)
            else:
                y = torch.empty((N, h, w, co), dtype=bf, device="cuda")
                B.vgg_conv3x3_fwd(B.BF16, N, h, w, cp, co, cur, wp, dev(inp.conv_b[l]), y, 1, wsb)
                B.vgg_maxpool2x2(B.BF16, N, h, w, co, y, pooled, arg)
            args[l] = arg
            cur = pooled
            h, w = h // 2, w // 2
        else:
            y = torch.empty((N, h, w, co), dtype=bf, device="cuda")
            if l == 0:      # the first convolution reads the NCHW batch itself
                B.vgg_conv3x3_fwd_first(B.BF16, N, h, w, dev(inp.x), wp, dev(inp.conv_b[l]), y, 1)
            else:
                B.vgg_conv3x3_fwd(B.BF16, N, h, w, cp, co, cur, wp, dev(inp.conv_b[l]), y, 1, wsb)
            cur = y
    flat = 512 * h * w
    dims = [(flat, hidden), (hidden, hidden), (hidden, classes)]
    # dense weights: the first layer's columns in H,W,C order (the order the NHWC tensor is flattened in)
    fcw32 = [dev(inp.fc_w[0]).view(hidden, 512, h * w).permute(0, 2, 1).reshape(hidden, flat).contiguous(),
             dev(inp.fc_w[1]), dev(inp.fc_w[2])]
    a_in = [cur.reshape(N, flat)]
    for l, (i, o) in enumerate(dims):
        last = l == 2
        z = torch.empty((N, o), dtype=torch.float32 if last else bf, device="cuda")
        B.vgg_fc(B.BF16, N, i, o, a_in[l], fcw32[l].to(bf), dev(inp.fc_b[l]), z, B.F32 if last else B.BF16, 0 if last else 1,
                 ws(B.vgg_fc_workspace_bytes(B.BF16, N, i, o)))
        a_in.append(z)
    logits = a_in[3]
    probs = torch.empty_like(logits)
    B.vgg_softmax(N, classes, logits, probs)
    dz = torch.empty_like(logits)
    loss = torch.zeros((1,), device="cuda")
    B.vgg_softmax_xent_bwd(N, classes, probs, dev(inp.labels), loss, dz, ws(4 * N + 256))
    g = dict(conv_w=[None] * 16, conv_b=[None] * 16, fc_w=[None] * 3, fc_b=[None] * 3)
    for l in (2, 1, 0):
        i, o = dims[l]
        dw = torch.empty((o, i), device="cuda")
        db = torch.empty((o,), device="cuda")
        da = torch.empty((N, i), device="cuda")
        B.vgg_fc_bwd(B.BF16, N, i, o, a_in[l], fcw32[l].to(bf), dz, dw, db, da, 1, ws(B.vgg_fc_bwd_workspace_bytes(B.BF16, N, i, o)))
        g["fc_w"][l], g["fc_b"][l] = dw, db
        dz = da
    g["fc_w"][0] = g["fc_w"][0].view(hidden, h * w, 512).permute(0, 2, 1).reshape(hidden, flat).contiguous()
    d = dz.to(bf).view(N, h, w, 512)
    for l in range(15, -1, -1):
        ci, co = _CONV[l]
        hh, ww = sizes[l]
        cp = B.vgg_padded_channels(B.BF16, ci)
        if l in _POOLED:
            up = torch.empty((N, hh, ww, co), dtype=bf, device="cuda")
            B.vgg_maxpool2x2_bwd(B.BF16, N, hh, ww, co, d, args[l], up)
            d = up
        dwp = torch.empty((9, co, cp), device="cuda")
        db = torch.empty((co,), device="cuda")
        B.vgg_conv3x3_bwd_weight(B.BF16, N, hh, ww, cp, co, acts_in[l], d, dwp, db,
                                 ws(B.vgg_conv3x3_bwd_weight_workspace_bytes(B.BF16, N, hh, ww, cp, co)))
        g["conv_w"][l] = dwp[:, :, :ci].reshape(3, 3, co, ci).permute(2, 3, 0, 1).contiguous()
        g["conv_b"][l] = db
        if l > 0:
            wtf = torch.empty((9, ci, co), dtype=bf, device="cuda")
            B.vgg_conv_pack_weights(B.BF16, ci, co, dev(inp.conv_w[l]), wtf, 1)
            dx = torch.empty((N, hh, ww, ci), dtype=bf, device="cuda")
            B.vgg_conv3x3_bwd_data(B.BF16, N, hh, ww, ci, co, d, wtf, acts_in[l], dx,
                                   ws(B.vgg_conv3x3_bwd_data_workspace_bytes(B.BF16, N, hh, ww, ci, co)))
            d = dx
    torch.cuda.synchronize()
    return logits, loss, g


@pytest.mark.parametrize("size", ["tiny", "224"])
def test_bf16_train_step_equals_chained_single_op_calls(size):
    if size == "tiny":
        inp, shp = synth.tiny_config(seed=0), (2, 32, 32, 512, 10)
    else:
        inp, shp = synth.vgg19_inputs(2, 224, 224, 4096, 1000, seed=1), (2, 224, 224, 4096, 1000)
    logits, loss, want = _bf16_step_from_single_op_calls(inp, *shp)
    m = Vgg19(B.BF16, *shp, lr=0.01, training=True)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    got = m.train_step(dev(inp.x), dev(inp.labels), want_grads=True)
    torch.cuda.synchronize()
    assert torch.equal(m.logits, logits)
    assert torch.equal(m.loss, loss)
    for k in ("conv_w", "conv_b", "fc_w", "fc_b"):
        for l, (a, b) in enumerate(zip(got[k], want[k])):
            assert torch.equal(a, b), (k, l, float((a - b).abs().max()))


def test_tiny_vgg19_train_step_bf16():
    _bf16_train_step_vs_oracle(synth.tiny_config(seed=0), 2, 32, 32, 512, 10)


def test_full_vgg19_train_step_bf16_224_vs_oracle_batch2():
    _bf16_train_step_vs_oracle(synth.vgg19_inputs(2, 224, 224, 4096, 1000, seed=1), 2, 224, 224, 4096, 1000)


def test_bf16_backward_kernels_on_oracle_tensors_tiny():
    print("worst error", _bf16_backward_kernels_on_oracle_tensors(synth.tiny_config(seed=0)))


def test_bf16_backward_kernels_on_oracle_tensors_224():
    print("worst error", _bf16_backward_kernels_on_oracle_tensors(synth.vgg19_inputs(2, 224, 224, 4096, 1000, seed=1)))


def test_bf16_training_needs_the_master_copy():
    cfg = B.make_config(B.BF16, 2, 32, 32, 512, 10, 0.01)          # no master copy
    assert B.vgg19_train_workspace_bytes(cfg) == 0
    cfgm = B.make_config(B.BF16, 2, 32, 32, 512, 10, 0.01, B.FLAG_FP32_MASTER)
    assert B.vgg19_train_workspace_bytes(cfgm) > 0
    assert B.vgg19_packed_bytes(cfgm) > 3 * B.vgg19_packed_bytes(cfg) - 4096 * 38    # bf16 + fp32 copy (biases fp32 in both)
    assert B.vgg19_packed_bytes(B.make_config(B.F32, 2, 32, 32, 512, 10, 0.01, B.FLAG_FP32_MASTER)) == 0   # bf16 only


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


def test_forward_as_one_graph_matches_eager():
    # replays of a recorded forward pass give bit-identical logits, also with eager work between replays
    inp = synth.full_config(1, seed=3, with_labels=False)
    m = Vgg19(B.BF16, 1, 224, 224, 4096, 1000)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    x = dev(inp.x)
    m.forward(x)
    torch.cuda.synchronize()
    want_logits, want_probs = m.logits.clone(), m.probs.clone()
    g = m.capture_forward(x, 2)
    for _ in range(3):
        m.logits.zero_(); m.probs.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(m.logits, want_logits) and torch.equal(m.probs, want_probs)
        m.forward(dev(inp.x * 0.5))      # eager work on the same buffers in between
        torch.cuda.synchronize()


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


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
def test_full_vgg19_train_step_batch100_is_mean_of_chunks(dtype):
    # The loss is a mean over images, so the batch-100 gradient equals the mean of the gradients of
    # five batch-20 steps from the same parameters (a property that holds at any size); the batch-2
    # test above ties the same kernels at the same spatial sizes to the oracle.  The chunks must run
    # the same arithmetic per image as the full batch: a ReLU or pooling decision that rounding
    # flips moves a gradient by far more than the tolerance.  Halves do (below roughly 40 images
    # the 14x14 layers split their contraction over several workgroups, another summation order).
    # bf16: the forward pass and the data gradients are then bit-identical per image, so the same holds.
    N, chunk = 100, 50
    inp = synth.full_config(N, seed=2)
    big = Vgg19(dtype, N, 224, 224, 4096, 1000, lr=0.01, training=True)
    big.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    gb = big.train_step(dev(inp.x), dev(inp.labels), want_grads=True)
    torch.cuda.synchronize()
    loss_big = big.loss.item()
    logits_big = big.logits.cpu().numpy()
    gb = {k: [a.double().cpu() for a in v] for k, v in gb.items()}
    new_big = big.unpack()
    del big
    torch.cuda.empty_cache()
    small = Vgg19(dtype, chunk, 224, 224, 4096, 1000, lr=0.01, training=True)
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


@pytest.mark.parametrize("size", ["tiny", "224"])
@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
def test_train_step_without_gradient_output_leaves_the_same_parameters(dtype, size):
    # Asking for the gradients (which adds the conversions to the canonical layout) must not change
    # the step: parameters, master and working copy, come out bit-identical either way -- over two
    # steps, so that the second runs on the first's updated weights.
    if size == "tiny":
        inp, shape = synth.tiny_config(seed=9), (2, 32, 32, 512, 10)
    else:
        inp, shape = synth.full_config(2, seed=9, with_labels=True), (2, 224, 224, 4096, 1000)
    plain = Vgg19(dtype, *shape, lr=0.01, training=True)
    fused = Vgg19(dtype, *shape, lr=0.01, training=True)
    for m in (plain, fused):
        m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    assert torch.equal(plain.packed, fused.packed)
    x, lab = dev(inp.x), dev(inp.labels)
    for step in range(2):
        plain.train_step(x, lab, want_grads=True)
        fused.train_step(x, lab, want_grads=False)
        torch.cuda.synchronize()
        assert torch.equal(plain.loss, fused.loss), step
        assert torch.equal(plain.logits, fused.logits), step
        assert torch.equal(plain.packed, fused.packed), step
    # and the step did move the dense weights
    before = np.asarray(inp.fc_w[2], dtype=np.float32)
    assert np.abs(fused.unpack()["fc_w"][2] - before).max() > 0


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
