"""Host-only checks of the C-ABI library: it loads, exports every symbol the
header declares, rejects bad arguments before touching the device, and its
launch plan has the structure the paper's instruction counts imply."""
import ctypes as C
import os
import re

import pytest

from paper_1810_09868_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "vgg_mi355x.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(vgg(?:19)?_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared()
    assert len(names) >= 28
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names


def test_strerror_and_padded_channels():
    L = B.lib()
    assert L.vgg_strerror(0) == b"ok"
    for code in range(-8, 0):
        assert L.vgg_strerror(code) not in (b"ok", b"unknown status")
    assert B.vgg_padded_channels(B.F32, 3) == 16
    assert B.vgg_padded_channels(B.BF16, 3) == 32
    assert B.vgg_padded_channels(B.BF16, 64) == 64
    assert B.vgg_padded_channels(7, 64) == 0


def test_argument_validation_happens_on_the_host():
    L = B.lib()
    a = 4096  # a 16-byte aligned fake address; validation must fail before it is ever used
    assert L.vgg_conv3x3_fwd(0, 1, 4, 4, 16, 16, None, a, None, a, 1, None, 0, None) == -1
    assert L.vgg_conv3x3_fwd(5, 1, 4, 4, 16, 16, a, a, None, a, 1, None, 0, None) == -3
    assert L.vgg_conv3x3_fwd(0, 0, 4, 4, 16, 16, a, a, None, a, 1, None, 0, None) == -2
    assert L.vgg_conv3x3_fwd(0, 1, 4, 4, 16, 16, a + 4, a, None, a, 1, None, 0, None) == -4
    assert L.vgg_conv3x3_fwd(0, 1, 4, 4, 3, 16, a, a, None, a, 1, None, 0, None) == -5   # needs a padded copy
    assert L.vgg_conv3x3_bwd_weight(1, 1, 4, 4, 16, 20, a, a, a, None, a, 1 << 30, None) == -7  # bf16: Cout % 8
    assert L.vgg_conv3x3_bwd_weight(0, 1, 4, 4, 16, 18, a, a, a, None, a, 1 << 30, None) == -7  # fp32: Cout % 4
    assert L.vgg_conv3x3_bwd_weight(1, 1, 4, 4, 16, 16, a, a, a, None, None, 0, None) == -5
    assert L.vgg_conv3x3_bwd_weight(0, 1, 4, 4, 16, 16, a, a, a, None, None, 0, None) == -5
    assert L.vgg_maxpool2x2(0, 1, 5, 4, 8, a, a, None, None) == -2                        # odd H
    assert L.vgg_maxpool2x2(0, 1, 4, 4, 8, None, a, None, None) == -1
    assert L.vgg_fc(0, 2, 0, 8, a, a, None, a, 0, 0, a, 1 << 30, None) == -2
    assert L.vgg_fc(0, 10, 10, 10, a, a, None, a, 0, 0, None, 0, None) == -5             # any In is a valid shape
    assert L.vgg_fc_bwd(1, 2, 12, 8, a, a, a, a, None, None, 0, a, 1 << 30, None) == -7  # bf16 backward: In % 8
    assert L.vgg_fc(0, 2, 64, 8, a, a, None, a, 0, 0, None, 0, None) == -5
    # the variant without a workspace argument: what exceeds its built-in buffer is refused on the host
    assert B.vgg_fc_workspace_bytes(B.F32, 1100, 8192, 4096) > B.FC_STATIC_SCRATCH_BYTES
    assert L.vgg_fc_static(0, 1100, 8192, 4096, a, a, None, a, 0, 0, None) == -8
    assert L.vgg_fc_static(0, 0, 8192, 4096, a, a, None, a, 0, 0, None) == -2
    assert L.vgg_fc_static(0, 4, 64, 8, a + 8, a, None, a, 0, 0, None) == -4
    assert B.vgg_fc_workspace_bytes(B.F32, 100, 25088, 4096) <= B.FC_STATIC_SCRATCH_BYTES
    # the first two convolutions as one call: bf16 only, H % 16 == 0 and W % 32 == 0, at least one output
    assert L.vgg_conv3x3_fwd_first_pair(1, 1, 16, 32, a, a, None, a, None, None, None, None) == -1
    assert L.vgg_conv3x3_fwd_first_pair(1, 1, 16, 32, None, a, None, a, None, a, None, None) == -1
    assert L.vgg_conv3x3_fwd_first_pair(7, 1, 16, 32, a, a, None, a, None, a, None, None) == -3
    assert L.vgg_conv3x3_fwd_first_pair(1, 0, 16, 32, a, a, None, a, None, a, None, None) == -2
    assert L.vgg_conv3x3_fwd_first_pair(0, 1, 16, 32, a, a, None, a, None, a, None, None) == -7
    assert L.vgg_conv3x3_fwd_first_pair(1, 1, 16, 48, a, a, None, a, None, a, None, None) == -7
    assert L.vgg_conv3x3_fwd_first_pair(1, 1, 24, 32, a, a, None, a, None, a, None, None) == -7
    assert L.vgg_conv3x3_fwd_first_pair(1, 1, 16, 32, a, a + 2, None, a, None, a, None, None) == -4
    assert L.vgg_softmax(0, 10, a, a, None) == -2
    assert L.vgg_sgd_update(0, a, a, 0.1, None) == -2
    assert L.vgg_sgd_update(4, None, a, 0.1, None) == -1


def test_model_level_validation_and_sizes():
    cfg = B.make_config(B.F32, 2, 32, 32, 512, 10)
    bad = B.make_config(B.F32, 2, 30, 32, 512, 10)
    assert B.vgg19_packed_bytes(bad) == 0 and B.vgg19_forward_workspace_bytes(bad) == 0
    nparams = sum(9 * ci * co + co for ci, co in
                  [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256)] + [(256, 256)] * 3 + [(256, 512)] +
                  [(512, 512)] * 7) + 512 * 512 + 512 + 512 * 512 + 512 + 512 * 10 + 10
    pb = B.vgg19_packed_bytes(cfg)
    assert nparams * 4 <= pb <= nparams * 4 + 9 * 64 * 13 * 4 + 64 * 256      # padding of conv1_1 + alignment
    assert B.vgg19_forward_workspace_bytes(cfg) > 2 * 2 * 32 * 32 * 64 * 4
    assert B.vgg19_train_workspace_bytes(cfg) > B.vgg19_forward_workspace_bytes(cfg)
    bf = B.make_config(B.BF16, 2, 32, 32, 512, 10)
    assert B.vgg19_train_workspace_bytes(bf) == 0
    L = B.lib()
    a = 4096
    assert L.vgg19_forward(C.byref(cfg), a, a, a, a, None, 0, None) == -5
    assert L.vgg19_forward(C.byref(bad), a, a, a, a, a, 1 << 40, None) == -2
    assert L.vgg19_forward(None, a, a, a, a, a, 1 << 40, None) == -1
    assert L.vgg19_train_step(C.byref(bf), a, a, a, 1 << 40, None, a, a, a, 1 << 40, None) == -7      # no master copy
    bfm = B.make_config(B.BF16, 2, 32, 32, 512, 10, 0.01, B.FLAG_FP32_MASTER)
    assert B.vgg19_train_workspace_bytes(bfm) > 0
    assert B.vgg19_packed_bytes(bfm) > B.vgg19_packed_bytes(bf) + B.vgg19_packed_bytes(cfg) - 9 * 64 * 32 * 4
    assert L.vgg19_train_step(C.byref(bfm), a, a, a, B.vgg19_packed_bytes(bf), None, a, a, a, 1 << 40, None) == -5
    assert B.vgg19_packed_bytes(B.make_config(B.F32, 2, 32, 32, 512, 10, 0.01, B.FLAG_FP32_MASTER)) == 0
    assert B.vgg19_packed_bytes(B.make_config(B.BF16, 2, 32, 32, 512, 10, 0.01, 2)) == 0
    full = B.make_config(B.F32, 100, 224, 224, 4096, 1000)
    assert B.vgg19_packed_bytes(full) >= 143667240 * 4


def test_launch_plan_matches_paper_op_counts():
    gold = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "hlo_counts.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, f, b = line.split()
        gold[name] = (int(f), int(b))
    cfg = B.make_config(B.F32, 100, 224, 224, 4096, 1000)
    fwd = B.vgg19_plan(cfg, False)
    assert fwd.count(1) == gold["convolution"][0] == 16
    assert fwd.count(4) == gold["reduce-window"][0] == 5
    assert fwd.count(6) == gold["dot"][0] == 3
    # bf16 forward: the first two convolutions and the first pool are one launch, still listed as three steps
    fwd16 = B.vgg19_plan(B.make_config(B.BF16, 100, 224, 224, 4096, 1000), False)
    assert fwd16 == fwd
    tr = B.vgg19_plan(cfg, True)
    # 47 convolutions = 16 forward + 16 weight gradients + 15 data gradients (none for the first layer)
    assert tr.count(1) + tr.count(2) + tr.count(3) == gold["convolution"][1] == 47
    assert tr.count(2) == 15 and tr.count(3) == 16
    assert tr.count(5) == gold["select-and-scatter"][1] == 5
    assert tr.count(6) + tr.count(7) + tr.count(8) == gold["dot"][1] == 9


def test_bench_refuses_more_than_one_gpu():
    # one GPU only: no collectives, no sharding; the benchmark says so instead of starting
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def _ru(v, a=256):
    return (v + a - 1) // a * a


def test_weight_gradient_workspace_query_covers_the_plan_that_runs():
    # The partial sums of the weight gradient are [partials][9][Cout][CinP] and [partials][Cout]; the
    # workspace query must be sized for the kernel that the launch picks for the same arguments (layers
    # with at most three input channels take a kernel with its own pixel tiling and split count).
    shapes = [(37, 55, 16, 3, 8), (57, 9, 42, 3, 64), (100, 224, 224, 3, 64), (2, 32, 32, 3, 64), (1, 7, 5, 1, 4),
              (3, 20, 28, 2, 12), (5, 56, 56, 3, 32), (2, 14, 14, 512, 512), (3, 30, 18, 17, 24), (100, 14, 14, 512, 512),
              (40, 28, 28, 256, 512), (9, 16, 48, 3, 16)]
    for n in range(1, 60, 7):
        for h in (3, 9, 16, 55):
            for w in (5, 16, 42, 56):
                shapes.append((n, h, w, 3, 8 * (1 + n % 5)))
    for dtype in (B.F32, B.BF16):
        for (n, h, w, ci, co) in shapes:
            if dtype == B.BF16 and co % 8:
                continue
            info = B.vgg_conv3x3_plan(B.PLAN_BWD_WEIGHT, dtype, n, h, w, ci, co)
            cp = B.vgg_padded_channels(dtype, ci)
            partials = info[5]
            assert partials >= 1 and info[6] >= 1
            pad = 0 if cp == ci else _ru(n * h * w * cp * (4 if dtype == B.F32 else 2))
            need = pad + _ru(partials * 9 * co * cp * 4) + _ru(partials * co * 4)
            assert B.vgg_conv3x3_bwd_weight_workspace_bytes(dtype, n, h, w, ci, co) == need, (dtype, n, h, w, ci, co, info)
            # one byte less is refused on the host, before anything is launched
            a = 4096
            assert B.lib().vgg_conv3x3_bwd_weight(dtype, n, h, w, ci, co, a, a, a, None, a, need - 1, None) == -5
    # the kernel for thin layers is the one the plan names for the network's first layer
    assert B.vgg_conv3x3_plan(B.PLAN_BWD_WEIGHT, B.F32, 100, 224, 224, 3, 64)[0] == 103
    assert B.vgg_conv3x3_plan(B.PLAN_BWD_WEIGHT, B.F32, 100, 224, 224, 64, 64)[0] == 116
    assert B.vgg_conv3x3_plan(B.PLAN_BWD_WEIGHT, B.F32, 100, 56, 56, 256, 256)[0] == 114
    # bf16: the thin kernel needs a width that is a multiple of 16; otherwise the 32-channel variant of the general one
    assert B.vgg_conv3x3_plan(B.PLAN_BWD_WEIGHT, B.BF16, 100, 224, 224, 3, 64)[0] == 118
    assert B.vgg_conv3x3_plan(B.PLAN_BWD_WEIGHT, B.BF16, 57, 9, 42, 3, 64)[0] == 117
    assert B.vgg_conv3x3_plan(B.PLAN_BWD_WEIGHT, B.BF16, 100, 224, 224, 64, 64)[0] == 116


def test_convolution_plan_query():
    L = B.lib()
    buf = (C.c_int * 7)()
    assert L.vgg_conv3x3_plan(0, 0, 1, 4, 4, 16, 16, None, 7) == -1
    assert L.vgg_conv3x3_plan(9, 0, 1, 4, 4, 16, 16, buf, 7) == -2
    assert L.vgg_conv3x3_plan(0, 0, 1, 4, 4, 16, 16, buf, 3) == -2
    assert L.vgg_conv3x3_plan(0, 4, 1, 4, 4, 16, 16, buf, 7) == -3
    assert L.vgg_conv3x3_plan(B.PLAN_FWD_POOL, 0, 1, 14, 14, 16, 16, buf, 7) == -7     # pool fusion needs 16-pixel patches
    # batch 100: 256-pixel tiles, contraction never split; the 14x14 layers take 128-pixel tiles with 64-wide column
    # tiles (fp32) or 320-pixel tiles, one per compute unit (bf16)
    for dtype in (B.F32, B.BF16):
        for (h, ci, co) in ((224, 64, 64), (112, 128, 128), (56, 256, 256), (28, 512, 512), (14, 512, 512)):
            for op in (B.PLAN_FWD, B.PLAN_BWD_DATA):
                info = B.vgg_conv3x3_plan(op, dtype, 100, h, h, ci, co)
                assert info[5] == 1
                assert info[1] == ((128 if dtype == B.F32 else 320) if h == 14 else 256)
                assert info[2] == (64 if (co == 64 or (h == 14 and dtype == B.F32)) else 128)
                if dtype == B.BF16 and h == 14:
                    assert info[0] in (6, 7) and info[6] <= 256
                assert info[1] * info[4] >= 100 * h * h
    # a single image: the last stages split their contraction over several workgroups
    assert B.vgg_conv3x3_plan(B.PLAN_FWD, B.BF16, 1, 14, 14, 512, 512)[5] > 1
    assert B.vgg_conv3x3_fwd_workspace_bytes(B.BF16, 1, 14, 14, 512, 512) > 0
    assert B.vgg_conv3x3_fwd_workspace_bytes(B.BF16, 100, 14, 14, 512, 512) == 0
