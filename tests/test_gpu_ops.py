"""Per-operation parity of the HIP kernels against the fp64 CPU oracle, through
the C ABI, on seeded inputs at sizes that span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import vgg_ref as R
from paper_1810_09868_amd import binding as B
from paper_1810_09868_amd import synth

from gpu_util import TDT, TOL, dev, from_nhwc, max_rel_err, to_nhwc, ws_bytes

pytestmark = pytest.mark.gpu

# (N, H, W, Cin, Cout): 2-D patch tiling (H, W multiples of 16), linear tiling with images and rows
# crossing inside a tile, ragged channel counts, a last partial tile, tiny images.
CONV_SHAPES = [
    (2, 32, 32, 64, 128),
    (3, 14, 14, 32, 64),
    (2, 28, 28, 96, 160),
    (3, 5, 7, 3, 20),
    (1, 2, 2, 16, 64),
    (5, 16, 48, 32, 192),
    (1, 56, 56, 64, 64),
    (1, 6, 100, 16, 32),   # wide rows: halo beyond the direct-to-LDS kernels' limit, weight-gradient halo in several batches
    # few tiles and a long contraction: several workgroups share a tile, each with a range of channel
    # chunks (uneven ranges: 9 or 18 chunks of 64 bytes; fp32 only: 5 chunks in two ranges)
    (1, 20, 20, 288, 64),
    (2, 14, 14, 80, 96),
    (1, 14, 14, 512, 512),
]


def _random_conv_shapes(count, seed=11):
    """Seeded shapes that mix the kernels' variants: patch and linear tiles, 64- and 128-wide column tiles,
    odd and even numbers of channel chunks, channel counts off the tile sizes, tiles that cross images."""
    import random
    rnd = random.Random(seed)
    hw = [(5, 7), (16, 16), (17, 16), (28, 28), (30, 33), (56, 56), (14, 14), (32, 48), (9, 100), (64, 64), (2, 2), (112, 16), (3, 130)]
    out = []
    while len(out) < count:
        H, W = rnd.choice(hw)
        N = rnd.choice([1, 2, 3, 5, 9])
        ci = rnd.choice([3, 8, 16, 24, 32, 40, 64, 96, 128, 160])
        co = rnd.choice([8, 20, 64, 72, 128, 136, 192, 256, 320])
        if N * H * W * ci * co * 9 <= 3e9:
            out.append((N, H, W, ci, co))
    return out


RANDOM_CONV_SHAPES = _random_conv_shapes(24)


def _pack(dtype, w, flip=0):
    Cout, Cin = w.shape[:2]
    rows, cols = (Cin, Cout) if flip else (Cout, Cin)
    out = torch.empty((9, rows, B.vgg_padded_channels(dtype, cols)), dtype=TDT[dtype], device="cuda")
    B.vgg_conv_pack_weights(dtype, Cin, Cout, dev(w), out, flip)
    return out


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv3x3_fwd(dtype, shape):
    N, H, W, Cin, Cout = shape
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=sum(shape))
    ref = R.conv3x3_fwd(d["x"], d["w"], d["b"], relu=True)
    x = to_nhwc(d["x"], dtype)
    y = torch.empty((N, H, W, Cout), dtype=TDT[dtype], device="cuda")
    ws = ws_bytes(B.vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, Cin, Cout))
    B.vgg_conv3x3_fwd(dtype, N, H, W, Cin, Cout, x, _pack(dtype, d["w"]), dev(d["b"]), y, 1, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(y), ref) <= TOL[dtype]
    # no bias, no ReLU
    ref2 = R.conv3x3_fwd(d["x"], d["w"], None, relu=False)
    B.vgg_conv3x3_fwd(dtype, N, H, W, Cin, Cout, x, _pack(dtype, d["w"]), None, y, 0, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(y), ref2) <= TOL[dtype]


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("shape", [(2, 32, 32, 64, 128), (3, 16, 48, 32, 64), (1, 112, 112, 32, 192)])
def test_conv3x3_fwd_with_fused_pool(dtype, shape):
    N, H, W, Cin, Cout = shape
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=sum(shape) + 7)
    x = to_nhwc(d["x"], dtype)
    y = torch.full((N, H, W, Cout), float("nan"), dtype=TDT[dtype], device="cuda")
    pooled = torch.full((N, H // 2, W // 2, Cout), float("nan"), dtype=TDT[dtype], device="cuda")
    B.vgg_conv3x3_fwd_pool(dtype, N, H, W, Cin, Cout, x, _pack(dtype, d["w"]), dev(d["b"]), y, pooled, 1)
    torch.cuda.synchronize()
    ref = R.conv3x3_fwd(d["x"], d["w"], d["b"], relu=True)
    pref, _ = R.maxpool2x2(ref)
    assert max_rel_err(from_nhwc(y), ref) <= TOL[dtype]
    assert max_rel_err(from_nhwc(pooled), pref) <= TOL[dtype]
    # the pooled tensor is exactly the 2x2 maximum of what the same launch wrote un-pooled
    pgpu, _ = R.maxpool2x2(from_nhwc(y))
    assert np.array_equal(from_nhwc(pooled), pgpu)
    # un-pooled output suppressed; positions of the maxima requested
    pooled2 = torch.empty_like(pooled)
    arg = torch.full((N, H // 2, W // 2, Cout), 255, dtype=torch.uint8, device="cuda")
    B.vgg_conv3x3_fwd_pool(dtype, N, H, W, Cin, Cout, x, _pack(dtype, d["w"]), dev(d["b"]), None, pooled2, 1, argmax=arg)
    torch.cuda.synchronize()
    assert torch.equal(pooled, pooled2)
    # bit-exact against the first-maximum rule applied to what the launch wrote un-pooled
    _, agpu = R.maxpool2x2(from_nhwc(y))
    assert np.array_equal(arg.permute(0, 3, 1, 2).cpu().numpy(), agpu)
    # and the same bytes as the stand-alone pooling kernel gives
    arg2 = torch.empty_like(arg)
    B.vgg_maxpool2x2(dtype, N, H, W, Cout, y, pooled2, arg2)
    torch.cuda.synchronize()
    assert torch.equal(arg, arg2) and torch.equal(pooled, pooled2)
    with pytest.raises(B.VggError):
        B.vgg_conv3x3_fwd_pool(dtype, N, 14, 14, Cin, Cout, x, _pack(dtype, d["w"]), dev(d["b"]), None, pooled2, 1)


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("shape", [(2, 32, 48), (3, 20, 9), (1, 224, 224), (70, 16, 16)])
def test_conv3x3_fwd_first_layer_from_nchw(dtype, shape):
    N, H, W = shape
    d = synth.conv_layer_inputs(N, H, W, 3, 64, seed=sum(shape))
    y = torch.full((N, H, W, 64), float("nan"), dtype=TDT[dtype], device="cuda")
    for relu in (1, 0):
        ref = R.conv3x3_fwd(d["x"], d["w"], d["b"], relu=bool(relu))
        B.vgg_conv3x3_fwd_first(dtype, N, H, W, dev(d["x"]), _pack(dtype, d["w"]), dev(d["b"]), y, relu)
        torch.cuda.synchronize()
        assert max_rel_err(from_nhwc(y), ref) <= TOL[dtype]


@pytest.mark.parametrize("shape", [(1, 16, 32), (2, 32, 64), (3, 48, 32), (22, 64, 128)])
def test_conv3x3_fwd_first_pair(shape):
    """The first two convolutions and the first pool as one call: against the oracle's three operations and
    against the library's separate calls (same products; the first layer adds its 27 in another order, so a
    few values differ by a rounding step).  The pooled tensor must be exactly the 2x2 maximum of the
    un-pooled one.  The last shape has 352 patches, more than the launch has workgroups."""
    N, H, W = shape
    dtype = B.BF16
    d1 = synth.conv_layer_inputs(N, H, W, 3, 64, seed=sum(shape))
    d2 = synth.conv_layer_inputs(1, 4, 4, 64, 64, seed=sum(shape) + 1)
    x = np.abs(d1["x"])      # image-like: non-negative
    b1 = np.linspace(-0.2, 0.3, 64).astype(np.float32)
    b2 = np.linspace(0.1, -0.4, 64).astype(np.float32)
    y1 = R.conv3x3_fwd(x, d1["w"], b1, relu=True)
    y2 = R.conv3x3_fwd(y1, d2["w"], b2, relu=True)
    pooled_ref, _ = R.maxpool2x2(y2)
    w1, w2 = _pack(dtype, d1["w"]), _pack(dtype, d2["w"])
    xd = dev(x.astype(np.float32))
    y2_g = torch.empty((N, H, W, 64), dtype=TDT[dtype], device="cuda")
    po_g = torch.empty((N, H // 2, W // 2, 64), dtype=TDT[dtype], device="cuda")
    B.vgg_conv3x3_fwd_first_pair(dtype, N, H, W, xd, w1, dev(b1), w2, dev(b2), y2_g, po_g)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(y2_g), y2) <= TOL[dtype]
    assert max_rel_err(from_nhwc(po_g), pooled_ref) <= TOL[dtype]
    # pooled == 2x2 maximum of the un-pooled output, bit for bit
    po_chk = torch.empty_like(po_g)
    B.vgg_maxpool2x2(dtype, N, H, W, 64, y2_g, po_chk)
    torch.cuda.synchronize()
    assert torch.equal(po_g.view(torch.int16), po_chk.view(torch.int16))
    # the separate calls: bf16 roundings of slightly different fp32 sums
    y1_s = torch.empty((N, H, W, 64), dtype=TDT[dtype], device="cuda")
    y2_s = torch.empty_like(y2_g)
    po_s = torch.empty_like(po_g)
    B.vgg_conv3x3_fwd_first(dtype, N, H, W, xd, w1, dev(b1), y1_s, 1)
    ws = ws_bytes(B.vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, 64, 64))
    B.vgg_conv3x3_fwd_pool(dtype, N, H, W, 64, 64, y1_s, w2, dev(b2), y2_s, po_s, 1, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(y2_g), from_nhwc(y2_s)) <= 2.0 ** -7
    # only one of the two outputs
    po_only = torch.zeros_like(po_g)
    B.vgg_conv3x3_fwd_first_pair(dtype, N, H, W, xd, w1, dev(b1), w2, dev(b2), None, po_only)
    torch.cuda.synchronize()
    assert torch.equal(po_only.view(torch.int16), po_g.view(torch.int16))
    y_only = torch.zeros_like(y2_g)
    B.vgg_conv3x3_fwd_first_pair(dtype, N, H, W, xd, w1, dev(b1), w2, dev(b2), y_only, None)
    torch.cuda.synchronize()
    assert torch.equal(y_only.view(torch.int16), y2_g.view(torch.int16))


def test_conv3x3_fwd_first_pair_rejects_other_shapes_and_dtypes():
    x = torch.zeros((1, 3, 16, 16), device="cuda")
    w = torch.zeros((9 * 64 * 64,), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((1, 16, 16, 64), dtype=torch.bfloat16, device="cuda")
    L = B.lib()
    args = (x.data_ptr(), w.data_ptr(), None, w.data_ptr(), None, y.data_ptr(), None, None)
    assert L.vgg_conv3x3_fwd_first_pair(B.BF16, 1, 16, 16, *args) == -7      # W not a multiple of 32
    assert L.vgg_conv3x3_fwd_first_pair(B.F32, 1, 16, 32, *args) == -7       # fp32
    assert L.vgg_conv3x3_fwd_first_pair(B.BF16, 1, 16, 32, x.data_ptr(), w.data_ptr(), None, w.data_ptr(), None, None, None, None) == -1


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv3x3_bwd_data(dtype, shape):
    N, H, W, Cin, Cout = shape
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=sum(shape) + 1)
    ref = R.conv3x3_bwd_data(d["dy"], d["w"])
    g = to_nhwc(d["dy"], dtype)
    dx = torch.empty((N, H, W, Cin), dtype=TDT[dtype], device="cuda")
    ws = ws_bytes(B.vgg_conv3x3_bwd_data_workspace_bytes(dtype, N, H, W, Cin, Cout))
    wtf = _pack(dtype, d["w"], flip=1)
    B.vgg_conv3x3_bwd_data(dtype, N, H, W, Cin, Cout, g, wtf, None, dx, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(dx), ref) <= TOL[dtype]
    # fused ReLU backward of the producer of x: dx * (x > 0)
    xsrc = to_nhwc(d["x"], dtype)
    B.vgg_conv3x3_bwd_data(dtype, N, H, W, Cin, Cout, g, wtf, xsrc, dx, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(dx), ref * (from_nhwc(xsrc) > 0)) <= TOL[dtype]


# The convolution layers of the batch-100 benchmark whose launches take kernels that the small shapes above
# never reach (bf16: weights in registers, with 256- and with 320-pixel tiles).  (N, H, W, Cin, Cout,
# expected kernel of the forward call, expected kernel of the data gradient with a mask.)
FULL_SIZE_LAYERS = [
    (100, 112, 112, 64, 128, 4, 1),
    (100, 56, 56, 128, 256, 5, 5),
    (100, 56, 56, 256, 256, 5, 5),
    (100, 28, 28, 256, 512, 4, 4),
    (100, 28, 28, 512, 512, 4, 4),
    (100, 14, 14, 512, 512, 7, 7),
]


def _sample_pixels(N, H, W, tile_rows, count, seed):
    """Pixels (n, h, w) to check at full size: the tensor's first and last pixels, the corners of an image,
    both sides of the first, a middle and the last tile boundary, and `count` random ones."""
    M = N * H * W
    flat = {0, 1, W - 1, W, H * W - 1, H * W, M - 1, M - W, M - H * W}
    for t in (1, (M // tile_rows) // 2, M // tile_rows):
        for d in (-1, 0, 1):
            flat.add(min(max(t * tile_rows + d, 0), M - 1))
    rng = np.random.default_rng(np.random.PCG64(seed))
    flat.update(int(v) for v in rng.integers(0, M, size=count))
    flat = np.array(sorted(flat))
    return flat // (H * W), (flat % (H * W)) // W, flat % W


def _patches(t_nchw, n, h, w):
    """The zero-padded 3x3 neighbourhoods [S, C, 3, 3] of the pixels (n[i], h[i], w[i])."""
    _, C, H, W = t_nchw.shape
    out = np.zeros((len(n), C, 3, 3), dtype=np.float64)
    for dh in range(3):
        for dw in range(3):
            hh, ww = h + dh - 1, w + dw - 1
            ok = (hh >= 0) & (hh < H) & (ww >= 0) & (ww < W)
            out[ok, :, dh, dw] = t_nchw[n[ok], :, hh[ok], ww[ok]]
    return out


@pytest.mark.parametrize("shape,kernel", [((42, 28, 28, 64, 512), 4), ((11, 56, 56, 64, 512), 5), ((33, 32, 32, 64, 512), 4)])
def test_conv3x3_bf16_weights_in_registers_element_by_element(shape, kernel):
    """The weights-in-registers kernel at sizes the oracle computes whole: just over 512 tiles of 256 pixels x 128
    channels (the smallest launches that take it), consecutive-pixel tiles with both halo sizes and patch tiles.
    Forward (plain stores straight from registers), forward with the fused pool where the size allows it, and
    the data gradient of the mirrored layer with its mask."""
    dtype = B.BF16
    N, H, W, Cin, Cout = shape
    assert B.vgg_conv3x3_plan(B.PLAN_FWD, dtype, N, H, W, Cin, Cout)[0] == kernel
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=sum(shape))
    ref = R.conv3x3_fwd(d["x"], d["w"], d["b"], relu=True)
    x = to_nhwc(d["x"], dtype)
    wp = _pack(dtype, d["w"])
    y = torch.empty((N, H, W, Cout), dtype=TDT[dtype], device="cuda")
    ws = ws_bytes(B.vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, Cin, Cout))
    B.vgg_conv3x3_fwd(dtype, N, H, W, Cin, Cout, x, wp, dev(d["b"]), y, 1, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(y), ref) <= TOL[dtype]
    if H % 16 == 0 and W % 16 == 0:
        assert B.vgg_conv3x3_plan(B.PLAN_FWD_POOL, dtype, N, H, W, Cin, Cout)[0] == kernel
        y2 = torch.empty_like(y)
        po = torch.empty((N, H // 2, W // 2, Cout), dtype=TDT[dtype], device="cuda")
        arg = torch.empty((N, H // 2, W // 2, Cout), dtype=torch.uint8, device="cuda")
        B.vgg_conv3x3_fwd_pool(dtype, N, H, W, Cin, Cout, x, wp, dev(d["b"]), y2, po, 1, ws, argmax=arg)
        torch.cuda.synchronize()
        assert torch.equal(y2.view(torch.int16), y.view(torch.int16))
        po_chk = torch.empty_like(po)
        arg_chk = torch.empty_like(arg)
        B.vgg_maxpool2x2(dtype, N, H, W, Cout, y, po_chk, arg_chk)
        torch.cuda.synchronize()
        assert torch.equal(po.view(torch.int16), po_chk.view(torch.int16)) and torch.equal(arg, arg_chk)
    # data gradient of the layer with the channel counts swapped: the same implicit GEMM on the flipped packing
    assert B.vgg_conv3x3_plan(B.PLAN_BWD_DATA, dtype, N, H, W, Cout, Cin)[0] == kernel
    d = synth.conv_layer_inputs(N, H, W, Cout, Cin, seed=sum(shape) + 1)
    refd = R.conv3x3_bwd_data(d["dy"], d["w"])
    g = to_nhwc(d["dy"], dtype)
    dx = torch.empty((N, H, W, Cout), dtype=TDT[dtype], device="cuda")
    wsd = ws_bytes(B.vgg_conv3x3_bwd_data_workspace_bytes(dtype, N, H, W, Cout, Cin))
    wtf = _pack(dtype, d["w"], flip=1)
    xsrc = to_nhwc(d["x"], dtype)
    B.vgg_conv3x3_bwd_data(dtype, N, H, W, Cout, Cin, g, wtf, xsrc, dx, wsd)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(dx), refd * (from_nhwc(xsrc) > 0)) <= TOL[dtype]


@pytest.mark.parametrize("cout", [200, 196, 132])
def test_conv3x3_bf16_weights_in_registers_ragged_channels(cout):
    """The weights-in-registers kernel with a last column tile that is only partly there: 200 channels (16-byte
    stores, the last 16-channel blocks of the tile missing), 196 (not a multiple of eight: the element-wise
    epilogue) and 132 (four channels into the second tile); 32 input channels make the contraction a single
    chunk.  Forward against the oracle, element by element; nothing may be written past the tensor."""
    dtype = B.BF16
    N, H, W, Cin = 84, 28, 28, 32
    assert B.vgg_conv3x3_plan(B.PLAN_FWD, dtype, N, H, W, Cin, cout)[0] == 4
    d = synth.conv_layer_inputs(N, H, W, Cin, cout, seed=cout)
    ref = R.conv3x3_fwd(d["x"], d["w"], d["b"], relu=True)
    x = to_nhwc(d["x"], dtype)
    wp = _pack(dtype, d["w"])
    n = N * H * W * cout
    buf = torch.full((n + 4096,), -7.0, dtype=TDT[dtype], device="cuda")      # (guard behind the tensor)
    y = buf[:n].view(N, H, W, cout)
    ws = ws_bytes(B.vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, Cin, cout))
    B.vgg_conv3x3_fwd(dtype, N, H, W, Cin, cout, x, wp, dev(d["b"]), y, 1, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(y), ref) <= TOL[dtype]
    assert (buf[n:] == -7.0).all()


def test_conv3x3_bf16_320_pixel_tiles_element_by_element():
    """The 320-pixel tiles (one workgroup per compute unit) at a size the oracle computes whole: 84 images of
    14x14 give 52 such tiles x 4 column tiles, tiles that cross image rows and images, and a ragged last tile.
    Forward on 128 -> 512 channels, data gradient (with and without mask) on 512 -> 128, each checked to be
    the launch that takes that kernel."""
    dtype = B.BF16
    N, H, W = 84, 14, 14
    # forward
    Cin, Cout = 128, 512
    assert B.vgg_conv3x3_plan(B.PLAN_FWD, dtype, N, H, W, Cin, Cout)[:2] in ([6, 320], [7, 320])
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=8414)
    x = to_nhwc(d["x"], dtype)
    y = torch.empty((N, H, W, Cout), dtype=TDT[dtype], device="cuda")
    ws = ws_bytes(B.vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, Cin, Cout))
    B.vgg_conv3x3_fwd(dtype, N, H, W, Cin, Cout, x, _pack(dtype, d["w"]), dev(d["b"]), y, 1, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(y), R.conv3x3_fwd(d["x"], d["w"], d["b"], relu=True)) <= TOL[dtype]
    # data gradient
    Cin, Cout = 512, 128
    assert B.vgg_conv3x3_plan(B.PLAN_BWD_DATA, dtype, N, H, W, Cin, Cout)[:2] in ([6, 320], [7, 320])
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=8415)
    ref = R.conv3x3_bwd_data(d["dy"], d["w"])
    g = to_nhwc(d["dy"], dtype)
    dx = torch.empty((N, H, W, Cin), dtype=TDT[dtype], device="cuda")
    ws = ws_bytes(B.vgg_conv3x3_bwd_data_workspace_bytes(dtype, N, H, W, Cin, Cout))
    wtf = _pack(dtype, d["w"], flip=1)
    B.vgg_conv3x3_bwd_data(dtype, N, H, W, Cin, Cout, g, wtf, None, dx, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(dx), ref) <= TOL[dtype]
    xsrc = to_nhwc(d["x"], dtype)
    B.vgg_conv3x3_bwd_data(dtype, N, H, W, Cin, Cout, g, wtf, xsrc, dx, ws)
    torch.cuda.synchronize()
    assert max_rel_err(from_nhwc(dx), ref * (from_nhwc(xsrc) > 0)) <= TOL[dtype]


@pytest.mark.parametrize("shape", FULL_SIZE_LAYERS)
def test_conv3x3_bf16_full_size_on_sampled_pixels(shape):
    """Forward and data gradient at the benchmark's sizes, in the launch configuration it times; the oracle
    computes the sampled pixels one neighbourhood at a time (all channels of each)."""
    N, H, W, Cin, Cout, kernel_fwd, kernel_bwd = shape
    dtype = B.BF16
    plan = B.vgg_conv3x3_plan(B.PLAN_FWD, dtype, N, H, W, Cin, Cout)
    assert plan[0] == kernel_fwd, plan
    assert B.vgg_conv3x3_plan(B.PLAN_BWD_DATA, dtype, N, H, W, Cin, Cout)[0] == kernel_bwd
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=sum(shape[:5]))
    n, h, w = _sample_pixels(N, H, W, plan[1], 400, seed=H + Cin)
    x = to_nhwc(d["x"], dtype)
    # forward (bias, ReLU): the centre of the oracle's output over each 3x3 neighbourhood
    y = torch.empty((N, H, W, Cout), dtype=TDT[dtype], device="cuda")
    ws = ws_bytes(B.vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, Cin, Cout))
    B.vgg_conv3x3_fwd(dtype, N, H, W, Cin, Cout, x, _pack(dtype, d["w"]), dev(d["b"]), y, 1, ws)
    torch.cuda.synchronize()
    ref = R.conv3x3_fwd(_patches(d["x"], n, h, w), d["w"], d["b"], relu=True)[:, :, 1, 1]
    got = y[torch.from_numpy(n).cuda(), torch.from_numpy(h).cuda(), torch.from_numpy(w).cuda()].float().cpu().numpy()
    assert max_rel_err(got, ref) <= TOL[dtype]
    del y
    # data gradient, without and with the (x > 0) factor of the layer below
    g = to_nhwc(d["dy"], dtype)
    dx = torch.empty((N, H, W, Cin), dtype=TDT[dtype], device="cuda")
    ws = ws_bytes(B.vgg_conv3x3_bwd_data_workspace_bytes(dtype, N, H, W, Cin, Cout))
    wtf = _pack(dtype, d["w"], flip=1)
    ref = R.conv3x3_bwd_data(_patches(d["dy"], n, h, w), d["w"])[:, :, 1, 1]
    idx = (torch.from_numpy(n).cuda(), torch.from_numpy(h).cuda(), torch.from_numpy(w).cuda())
    B.vgg_conv3x3_bwd_data(dtype, N, H, W, Cin, Cout, g, wtf, None, dx, ws)
    torch.cuda.synchronize()
    assert max_rel_err(dx[idx].float().cpu().numpy(), ref) <= TOL[dtype]
    B.vgg_conv3x3_bwd_data(dtype, N, H, W, Cin, Cout, g, wtf, x, dx, ws)
    torch.cuda.synchronize()
    keep = x[idx].float().cpu().numpy() > 0
    assert max_rel_err(dx[idx].float().cpu().numpy(), ref * keep) <= TOL[dtype]


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv3x3_bwd_weight(dtype, shape):
    _check_bwd_weight(dtype, shape, seed=sum(shape) + 2)


def _check_bwd_weight(dtype, shape, seed):
    """fp32, or bf16 operands (x and g rounded to bf16, fp32 sums and fp32 result)."""
    N, H, W, Cin, Cout = shape
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=seed)
    dw_ref, db_ref = R.conv3x3_bwd_weight(d["x"], d["dy"])
    x = to_nhwc(d["x"], dtype)
    g = to_nhwc(d["dy"], dtype)
    cp = B.vgg_padded_channels(dtype, Cin)
    dwp = torch.full((9, Cout, cp), float("nan"), device="cuda")
    db = torch.empty((Cout,), device="cuda")
    ws = ws_bytes(B.vgg_conv3x3_bwd_weight_workspace_bytes(dtype, N, H, W, Cin, Cout))
    if dtype == B.BF16 and Cout % 8:
        with pytest.raises(B.VggError):      # 16-byte channel segments of g
            B.vgg_conv3x3_bwd_weight(dtype, N, H, W, Cin, Cout, x, g, dwp, db, ws)
        return
    B.vgg_conv3x3_bwd_weight(dtype, N, H, W, Cin, Cout, x, g, dwp, db, ws)
    torch.cuda.synchronize()
    dw = dwp[:, :, :Cin].reshape(3, 3, Cout, Cin).permute(2, 3, 0, 1)    # [t][co][ci] -> [co][ci][kh][kw]
    assert max_rel_err(dw.cpu().numpy(), dw_ref) <= TOL[dtype]
    assert max_rel_err(db.cpu().numpy(), db_ref) <= TOL[dtype]
    assert (dwp[:, :, Cin:] == 0).all()     # padding channels get exact zeros
    if dtype == B.F32:
        dw2 = torch.empty((Cout, Cin, 3, 3), device="cuda")
        B.vgg_conv_unpack_weights(Cin, Cout, dwp, dw2)
        torch.cuda.synchronize()
        assert torch.equal(dw2, dw)
    # run-to-run reproducibility of the split reduction
    dwp2 = torch.empty_like(dwp)
    B.vgg_conv3x3_bwd_weight(dtype, N, H, W, Cin, Cout, x, g, dwp2, db, ws)
    torch.cuda.synchronize()
    assert torch.equal(dwp, dwp2)


@pytest.mark.parametrize("shape", [(37, 55, 16, 3, 8), (57, 9, 42, 3, 64), (9, 16, 48, 2, 16), (2, 224, 224, 3, 64)])
def test_conv3x3_bwd_weight_thin_layers_stay_inside_their_workspace(shape):
    # At most three input channels: fp32 takes a kernel with its own pixel tiling, hence its own number of
    # partial sums.  The workspace is exactly what the query asks for, followed by a guard that must survive.
    N, H, W, Cin, Cout = shape
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=sum(shape) + 3)
    dw_ref, db_ref = R.conv3x3_bwd_weight(d["x"], d["dy"])
    for dtype in (B.F32, B.BF16):
        need = B.vgg_conv3x3_bwd_weight_workspace_bytes(dtype, N, H, W, Cin, Cout)
        buf = torch.full((need + 4096,), 0xA5, dtype=torch.uint8, device="cuda")
        cp = B.vgg_padded_channels(dtype, Cin)
        dwp = torch.full((9, Cout, cp), float("nan"), device="cuda")
        db = torch.empty((Cout,), device="cuda")
        B.vgg_conv3x3_bwd_weight(dtype, N, H, W, Cin, Cout, to_nhwc(d["x"], dtype), to_nhwc(d["dy"], dtype), dwp, db, buf[:need])
        torch.cuda.synchronize()
        assert (buf[need:] == 0xA5).all(), dtype
        dw = dwp[:, :, :Cin].reshape(3, 3, Cout, Cin).permute(2, 3, 0, 1)
        assert max_rel_err(dw.cpu().numpy(), dw_ref) <= TOL[dtype]
        assert max_rel_err(db.cpu().numpy(), db_ref) <= TOL[dtype]
        with pytest.raises(B.VggError):
            B.vgg_conv3x3_bwd_weight(dtype, N, H, W, Cin, Cout, to_nhwc(d["x"], dtype), to_nhwc(d["dy"], dtype), dwp, db,
                                     buf[:need - 256])


def test_paper_dense_and_softmax_examples():
    # The paper's two introductory functions at the sizes its compiled listings show: dense on a 10 x 10
    # matrix, a 10-vector and a 10-vector bias; softmax of a 10-vector (section "Two simple examples").
    rng = np.random.default_rng(1810)
    W = rng.standard_normal((10, 10)).astype(np.float32)
    x = rng.standard_normal((1, 10)).astype(np.float32)
    b = rng.standard_normal(10).astype(np.float32)
    z = torch.empty((1, 10), device="cuda")
    B.vgg_fc(B.F32, 1, 10, 10, dev(x), dev(W), dev(b), z, B.F32, 0, ws_bytes(B.vgg_fc_workspace_bytes(B.F32, 1, 10, 10)))
    p = torch.empty((1, 10), device="cuda")
    B.vgg_softmax(1, 10, z, p)
    torch.cuda.synchronize()
    zr = R.fc(x, W, b, relu=False)
    assert max_rel_err(z.cpu().numpy(), zr) <= 1e-6
    assert np.abs(z.cpu().numpy().astype(np.float64) - (W.astype(np.float64) @ x[0].astype(np.float64) + b)).max() <= 1e-5
    assert max_rel_err(p.cpu().numpy(), R.softmax(zr)) <= 1e-6
    assert abs(float(p.sum()) - 1.0) <= 1e-6


@pytest.mark.parametrize("shape", RANDOM_CONV_SHAPES)
def test_conv3x3_random_shapes(shape):
    for dtype in (B.F32, B.BF16):
        test_conv3x3_fwd(dtype, shape)
        test_conv3x3_bwd_data(dtype, shape)
    if shape[4] % 4 == 0:
        _check_bwd_weight(B.F32, shape, seed=sum(shape) + 2)
        _check_bwd_weight(B.BF16, shape, seed=sum(shape) + 2)


def test_pack_unpack_roundtrip_and_flip_layout():
    rng = np.random.default_rng(3)
    Cin, Cout = 5, 12
    w = rng.standard_normal((Cout, Cin, 3, 3)).astype(np.float32)
    p = _pack(B.F32, w)
    back = torch.empty((Cout, Cin, 3, 3), device="cuda")
    B.vgg_conv_unpack_weights(Cin, Cout, p, back)
    assert np.array_equal(back.cpu().numpy(), w)
    pf = _pack(B.F32, w, flip=1).cpu().numpy()       # [9][Cin][CoutP]
    for t in range(9):
        assert np.array_equal(pf[t, :, :Cout], w.reshape(Cout, Cin, 9)[:, :, 8 - t].T)
    assert not pf[:, :, Cout:].any()


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("shape", [(2, 8, 12, 64), (3, 2, 2, 8), (1, 14, 14, 512)])
def test_maxpool_fwd_bwd(dtype, shape):
    N, H, W, Cc = shape
    rng = np.random.default_rng(sum(shape))
    x = rng.standard_normal((N, Cc, H, W)).astype(np.float32)
    xd = to_nhwc(x, dtype)
    xq = from_nhwc(xd)                        # what the kernel sees (bf16-rounded for BF16)
    p_ref, a_ref = R.maxpool2x2(xq)
    y = torch.empty((N, H // 2, W // 2, Cc), dtype=TDT[dtype], device="cuda")
    arg = torch.empty((N, H // 2, W // 2, Cc), dtype=torch.uint8, device="cuda")
    B.vgg_maxpool2x2(dtype, N, H, W, Cc, xd, y, arg)
    torch.cuda.synchronize()
    assert np.array_equal(from_nhwc(y), p_ref)                 # selection only: bit-exact
    a_gpu = arg.permute(0, 3, 1, 2).cpu().numpy()
    if dtype == B.F32:
        assert np.array_equal(a_gpu, a_ref)                    # random fp32 data has no ties
    else:
        # bf16 rounding creates ties; the oracle consumed the same rounded values, first-max rule applies
        assert np.array_equal(a_gpu, a_ref)
    dp = rng.standard_normal(p_ref.shape).astype(np.float32)
    dpd = to_nhwc(dp, dtype)
    dx = torch.full((N, H, W, Cc), float("nan"), dtype=TDT[dtype], device="cuda")
    B.vgg_maxpool2x2_bwd(dtype, N, H, W, Cc, dpd, arg, dx)
    torch.cuda.synchronize()
    assert np.array_equal(from_nhwc(dx), R.maxpool2x2_bwd(from_nhwc(dpd), a_ref))


def test_maxpool_ties_pick_first():
    x = np.zeros((1, 8, 4, 4), dtype=np.float32)
    x[0, 1] = 3.0
    x[0, 2, 1, 1] = 1.0
    xd = to_nhwc(x, B.F32)
    y = torch.empty((1, 2, 2, 8), device="cuda")
    arg = torch.empty((1, 2, 2, 8), dtype=torch.uint8, device="cuda")
    B.vgg_maxpool2x2(B.F32, 1, 4, 4, 8, xd, y, arg)
    _, a_ref = R.maxpool2x2(x)
    assert np.array_equal(arg.permute(0, 3, 1, 2).cpu().numpy(), a_ref)


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("shape", [(100, 512, 1000), (2, 512, 10), (7, 2048, 96), (130, 64, 200),
                                   # rows that are not whole 64-byte units: the paper's own dense example
                                   # (a 10 x 10 matrix times a 10-vector, here also on ten vectors), odd
                                   # lengths, a last unit holding one element
                                   (1, 10, 10), (10, 10, 10), (3, 50, 7), (5, 37, 130), (129, 1, 3), (4, 8200, 40), (6, 2052, 9)])
def test_fc_forward(dtype, shape):
    N, In, Out = shape
    rng = np.random.default_rng(sum(shape))
    a = rng.standard_normal((N, In)).astype(np.float32)
    w = (rng.standard_normal((Out, In)) * np.sqrt(2.0 / In)).astype(np.float32)
    b = rng.standard_normal(Out).astype(np.float32)
    ws = ws_bytes(B.vgg_fc_workspace_bytes(dtype, N, In, Out))
    for relu, zdt in ((1, dtype), (0, B.F32)):
        ref = R.fc(a, w, b, relu=bool(relu))
        z = torch.empty((N, Out), dtype=TDT[zdt], device="cuda")
        B.vgg_fc(dtype, N, In, Out, dev(a, TDT[dtype]), dev(w, TDT[dtype]), dev(b), z, zdt, relu, ws)
        torch.cuda.synchronize()
        assert max_rel_err(z.float().cpu().numpy(), ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("shape", [(100, 512, 1000), (2, 512, 10), (7, 2048, 96), (130, 64, 200), (113, 160, 33), (250, 96, 72),
                                   (1, 10, 10), (10, 10, 10), (5, 37, 130), (9, 50, 64), (3, 1030, 5), (10, 24, 10)])
def test_fc_backward(dtype, shape):
    # bf16: a and w are bf16, dz fp32 (rounded to bf16 inside, except for db); all results fp32
    N, In, Out = shape
    if dtype == B.BF16 and In % 8:
        a = torch.zeros((64,), device="cuda")
        with pytest.raises(B.VggError):      # 16-byte segments of bf16 rows
            B.vgg_fc_bwd(dtype, N, In, Out, a, a, a, a, None, None, 0, a)
        return
    rng = np.random.default_rng(sum(shape) + 5)
    a = rng.standard_normal((N, In)).astype(np.float32)
    w = (rng.standard_normal((Out, In)) * np.sqrt(2.0 / In)).astype(np.float32)
    dz = rng.standard_normal((N, Out)).astype(np.float32)
    dw_ref, db_ref, da_ref = R.fc_bwd(a, w, dz)
    dw = torch.full((Out, In), float("nan"), device="cuda")
    db = torch.empty((Out,), device="cuda")
    da = torch.full((N, In), float("nan"), device="cuda")
    ws = ws_bytes(B.vgg_fc_bwd_workspace_bytes(dtype, N, In, Out))
    ad, wd = dev(a, TDT[dtype]), dev(w, TDT[dtype])
    B.vgg_fc_bwd(dtype, N, In, Out, ad, wd, dev(dz), dw, db, da, 0, ws)
    torch.cuda.synchronize()
    assert max_rel_err(dw.cpu().numpy(), dw_ref) <= TOL[dtype]
    assert max_rel_err(db.cpu().numpy(), db_ref) <= TOL[B.F32]         # a plain fp32 sum in both
    assert max_rel_err(da.cpu().numpy(), da_ref) <= TOL[dtype]
    B.vgg_fc_bwd(dtype, N, In, Out, ad, wd, dev(dz), dw, None, da, 1, ws)
    torch.cuda.synchronize()
    assert max_rel_err(da.cpu().numpy(), da_ref * (ad.float().cpu().numpy() > 0)) <= TOL[dtype]
    with pytest.raises(B.VggError):
        B.vgg_fc_bwd(dtype, N, In, Out, ad, wd, dev(dz), dw, None, da, 1, None)


@pytest.mark.parametrize("shape", [(100, 1000), (2, 10), (5, 64), (3, 129), (1, 10), (1, 1), (4, 5000)])
def test_softmax_xent_sgd(shape):
    N, K = shape
    rng = np.random.default_rng(N * K)
    z = (rng.standard_normal((N, K)) * 3).astype(np.float32)
    labels = rng.integers(0, K, size=N).astype(np.int32)
    p_ref = R.softmax(z)
    p = torch.empty((N, K), device="cuda")
    B.vgg_softmax(N, K, dev(z), p)
    torch.cuda.synchronize()
    assert max_rel_err(p.cpu().numpy(), p_ref) <= 1e-5
    loss_ref, dz_ref = R.softmax_xent(p.cpu().numpy().astype(np.float64), labels)
    loss = torch.empty((1,), device="cuda")
    dz = torch.empty((N, K), device="cuda")
    B.vgg_softmax_xent_bwd(N, K, p, dev(labels), loss, dz, ws_bytes(N * 4))
    torch.cuda.synchronize()
    assert abs(loss.item() - loss_ref) <= 1e-5 * abs(loss_ref)
    assert max_rel_err(dz.cpu().numpy(), dz_ref) <= 1e-6
    n = N * K + 3 if (N * K) % 4 else N * K - 1      # exercise the scalar tail
    theta = rng.standard_normal(n).astype(np.float32)
    grad = rng.standard_normal(n).astype(np.float32)
    th = dev(theta)
    B.vgg_sgd_update(n, th, dev(grad), 0.01)
    torch.cuda.synchronize()
    ref = R.sgd(theta, grad, 0.01)
    assert np.abs(th.cpu().numpy() - ref).max() <= 1e-6


def test_layout_roundtrip_and_convert():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2, 3, 6, 10)).astype(np.float32)
    y = torch.empty((2, 6, 10, 16), device="cuda")
    B.vgg_nchw_to_nhwc(B.F32, 2, 3, 6, 10, 16, dev(x), y)
    assert np.array_equal(y[..., :3].permute(0, 3, 1, 2).cpu().numpy(), x) and not y[..., 3:].any()
    back = torch.empty((2, 3, 6, 10), device="cuda")
    B.vgg_nhwc_to_nchw(B.F32, 2, 3, 6, 10, 16, y, back)
    assert np.array_equal(back.cpu().numpy(), x)
    # fp32 -> bf16 is round-to-nearest-even: torch implements the same IEEE rule
    v = dev(rng.standard_normal(1000).astype(np.float32))
    out = torch.empty((1000,), dtype=torch.bfloat16, device="cuda")
    B.vgg_convert(B.F32, B.BF16, 1000, v, out)
    assert torch.equal(out, v.to(torch.bfloat16))
    halfway = torch.tensor([1.00390625, 1.01171875], device="cuda")   # exactly between two bf16 values
    o2 = torch.empty((2,), dtype=torch.bfloat16, device="cuda")
    B.vgg_convert(B.F32, B.BF16, 2, halfway, o2)
    assert o2.float().tolist() == [1.0, 1.015625]                     # ties go to the even mantissa


def test_conv3x3_split_contraction_needs_its_workspace():
    # a shape whose contraction is split reports a workspace for the partial sums and refuses to run without it
    N, H, W, Cin, Cout = 1, 14, 14, 512, 512
    for dtype in (B.F32, B.BF16):
        need = B.vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, Cin, Cout)
        assert need >= 2 * N * H * W * Cout * 4
        assert B.vgg_conv3x3_bwd_data_workspace_bytes(dtype, N, H, W, Cin, Cout) == need
        x = torch.zeros((N, H, W, Cin), dtype=TDT[dtype], device="cuda")
        w = torch.zeros((9, Cout, Cin), dtype=TDT[dtype], device="cuda")
        y = torch.empty((N, H, W, Cout), dtype=TDT[dtype], device="cuda")
        for ws in (None, ws_bytes(need - 256)):
            with pytest.raises(B.VggError):
                B.vgg_conv3x3_fwd(dtype, N, H, W, Cin, Cout, x, w, None, y, 1, ws)
            with pytest.raises(B.VggError):
                B.vgg_conv3x3_bwd_data(dtype, N, H, W, Cin, Cout, x, w, None, y, ws)
    # the batch-100 shapes keep every contraction in one workgroup: no workspace
    assert B.vgg_conv3x3_fwd_workspace_bytes(B.BF16, 100, 14, 14, 512, 512) == 0


def test_mfma_probe_runs_and_reports_flops():
    sink = torch.empty((B.vgg_mfma_probe_sink_bytes(),), dtype=torch.uint8, device="cuda")
    for dt, per in ((B.BF16, 2 * 32 * 32 * 16), (B.F32, 2 * 32 * 32 * 2)):
        flops = B.vgg_mfma_probe(dt, True, 10, sink)
        torch.cuda.synchronize()
        assert flops > 0 and flops % (10 * 8 * per) == 0
    # constant operands: every accumulator element is the contraction length times the MFMA count
    B.vgg_mfma_probe(B.BF16, False, 3, sink)
    torch.cuda.synchronize()
    vals = sink.view(torch.float32)[:256]
    assert torch.all(vals == 4 * 16 * (3 * 8 // 4) * 16.0)
    # the 16x16x32 shape: twice the instructions, each half the size, the same sums and the same operation count
    sink.zero_()
    assert B.vgg_mfma_probe(B.BF16, False, 3, sink, True) == B.vgg_mfma_probe(B.BF16, False, 3, sink)
    B.vgg_mfma_probe(B.BF16, False, 3, sink, True)
    torch.cuda.synchronize()
    assert torch.all(sink.view(torch.float32)[:256] == 4 * 16 * (3 * 8 // 4) * 16.0)
    with pytest.raises(B.VggError):
        B.vgg_mfma_probe(B.F32, False, 3, sink, True)
    small = torch.empty((16,), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.VggError):
        B.vgg_mfma_probe(B.BF16, False, 3, small)
