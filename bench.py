#!/usr/bin/env python3
"""Benchmark: VGG19 forward images/s at batch 100, 224x224, on one MI355X.

One step = one whole forward pass (NCHW->NHWC transform, 16 convolutions with
bias+ReLU, 5 max-pools, 3 dense layers, softmax) over one batch of synthetic
images that is already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--dtype bf16|f32]

The roofline figures come from a second pass of the same K steps in which the
library brackets every launch with HIP events on the launch stream
(vgg19_timed); doing that inside the main timed loop would perturb `value`.
The CPU baseline is the fp64 oracle timed on a few images of the same batch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

CONV = [(3, 64, 224), (64, 64, 224), (64, 128, 112), (128, 128, 112), (128, 256, 56), (256, 256, 56),
        (256, 256, 56), (256, 256, 56), (256, 512, 28), (512, 512, 28), (512, 512, 28), (512, 512, 28),
        (512, 512, 14), (512, 512, 14), (512, 512, 14), (512, 512, 14)]
PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # MI355X dense MFMA peaks
HBM_GBS = 8000.0


def recorded_traffic(dtype_name, N):
    """HBM-side bytes per launch of the roofline kernel from the committed rocprofv3 counter summary,
    or None when there is none for this workload or the kernel sources changed since it was taken."""
    import hashlib
    import re
    if N != 100:
        return None
    path = os.path.join(ROOT, "profiles", "vgg19_fwd_%s_batch100_rocprofv3.md" % dtype_name)
    try:
        text = open(path).read()
        h = hashlib.sha256()
        for fn in ("paper_1810_09868_amd/csrc/conv_igemm.hip", "paper_1810_09868_amd/csrc/common.h"):
            h.update(open(os.path.join(ROOT, fn), "rb").read())
        sha = re.search(r"kernel_source_sha256: ([0-9a-f]+)", text).group(1)
        if sha != h.hexdigest():
            return None
        return float(re.search(r"traffic_bytes_per_launch: ([0-9.]+)", text).group(1))
    except (OSError, AttributeError):
        return None


def conv_flops(N, l):
    ci, co, hw = CONV[l]
    return 2.0 * N * hw * hw * 9 * ci * co


def run_forward_bench(dtype_name, N, steps, warmup, inp):
    import torch
    from paper_1810_09868_amd import binding as B
    from paper_1810_09868_amd.model import Vgg19
    dtype = B.BF16 if dtype_name == "bf16" else B.F32
    m = Vgg19(dtype, N, 224, 224, 4096, 1000)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    x = torch.from_numpy(inp.x).cuda()
    for _ in range(warmup):
        m.forward(x)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        m.forward(x)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    # per-launch pass (HIP events inside the library, on the launch stream)
    conv_ms = [0.0] * 16
    other_ms = {"pool": 0.0, "fc": 0.0, "other": 0.0}
    for _ in range(steps):
        kinds, ms = B.vgg19_timed(m.cfg, False, x, None, m.packed, m.logits, m.ws)
        ci = 0
        for k, t in zip(kinds, ms):
            if k == 1:
                conv_ms[ci] += t / steps
                ci += 1
            elif k == 4:
                other_ms["pool"] += t / steps
            elif k == 6:
                other_ms["fc"] += t / steps
            else:
                other_ms["other"] += t / steps
    total_conv_ms = sum(conv_ms)
    total_conv_flops = sum(conv_flops(N, l) for l in range(16))
    # dominant kernel: the 256x128-tile instantiation, used by every layer with Cout > 64 whose grid
    # of such tiles can give each of the 256 CUs two workgroups (not the 14x14 layers)
    def n_tiles(l):
        hw = CONV[l][2]
        return N * (hw // 16) ** 2 if hw % 16 == 0 else -(-N * hw * hw // 256)
    wide = [l for l in range(16) if CONV[l][1] > 64 and n_tiles(l) * -(-CONV[l][1] // 128) >= 512]
    wide_flops = sum(conv_flops(N, l) for l in wide) / len(wide)       # algorithmic flops per launch
    wide_ms = sum(conv_ms[l] for l in wide) / len(wide)                # average launch duration
    achieved = wide_flops / (wide_ms * 1e-3) / 1e12
    peak = PEAK_TFLOPS[dtype_name]
    # The bf16 forward pass runs the first two convolutions and the first pool as one launch: the plan still
    # lists the second convolution, with no launch behind it (its interval is the gap between two events).
    fused01 = conv_ms[1] < 0.02 * conv_ms[0]
    per_layer = []
    for l in range(16):
        if fused01 and l == 1:
            per_layer.append({"layer": 1, "ms": 0.0, "tflops": None, "note": "in the launch of layer 0"})
            continue
        fl = conv_flops(N, l) + (conv_flops(N, 1) if fused01 and l == 0 else 0.0)
        per_layer.append({"layer": l, "ms": round(conv_ms[l], 4), "tflops": round(fl / (conv_ms[l] * 1e-3) / 1e12, 1)})
    res = {
        "ms_per_step": dt * 1e3,
        "images_per_s": N / dt,
        "conv_ms_per_step": total_conv_ms,
        "conv_tflops": total_conv_flops / (total_conv_ms * 1e-3) / 1e12,
        "pct_mfma_peak_conv": 100.0 * total_conv_flops / (total_conv_ms * 1e-3) / 1e12 / peak,
        "other_ms_per_step": other_ms,
        "per_layer": per_layer,
        "roofline": {"bound": "mfma", "kernel": ("conv3x3_igemm_wreg_kernel<2,2,*,4,2>" if dtype_name == "bf16"
                                                  else "conv3x3_igemm_dma_kernel<float,256,128,4,2,*>"),
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "launches_per_step": len(wide), "avg_launch_ms": wide_ms,
                     "traffic": recorded_traffic(dtype_name, N)},
    }
    del m
    torch.cuda.empty_cache()
    return res


def run_train_bench(N, steps, inp_seed=0, dtype_name="f32", extras=True, graph=True):
    """Training step (forward, cross-entropy, backward, SGD) at the same shapes: extra context.  bf16: bf16
    operands, fp32 sums, fp32 master parameters."""
    import torch
    from paper_1810_09868_amd import binding as B
    from paper_1810_09868_amd import synth
    from paper_1810_09868_amd.model import Vgg19
    inp = synth.full_config(N, seed=inp_seed)
    m = Vgg19(B.BF16 if dtype_name == "bf16" else B.F32, N, 224, 224, 4096, 1000, lr=0.01, training=True)
    m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    x = torch.from_numpy(inp.x).cuda()
    lab = torch.from_numpy(inp.labels).cuda()
    for _ in range(2):
        m.train_step(x, lab)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        m.train_step(x, lab)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    dt_graph = None
    if graph:
        # the same steps as one HIP graph: the training loop replayed by a single launch
        g = m.capture_train_steps(x, lab, steps)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        dt_graph = (time.perf_counter() - t0) / steps
        del g
    kinds, ms = B.vgg19_timed(m.cfg, True, x, lab, m.packed, m.logits, m.ws)
    names = {1: "conv_fwd", 2: "conv_dgrad", 3: "conv_wgrad", 4: "pool", 5: "pool_bwd", 6: "fc", 7: "fc_bwd", 9: "other"}
    by_kind = {}
    for k, t in zip(kinds, ms):
        if k in names:
            by_kind[names[k]] = round(by_kind.get(names[k], 0.0) + t, 3)
    conv = sum(conv_flops(N, l) for l in range(16))
    fc = 2.0 * N * (25088 * 4096 + 4096 * 4096 + 4096 * 1000)
    flops = 3 * conv - conv_flops(N, 0) + 3 * fc   # no data gradient for the first convolution
    del m
    torch.cuda.empty_cache()
    res = {"workload": ("configs[4]: fp32 training step" if dtype_name == "f32" else
                        "configs[4] with bf16 operands, fp32 sums and fp32 master parameters: training step") +
                       ", batch %d, 3x224x224 (forward, mean cross-entropy, backward, SGD lr 0.01)" % N,
           "dtype": dtype_name, "ms_per_step": dt * 1e3, "images_per_s": N / dt, "tflops": flops / dt / 1e12,
           "pct_mfma_peak": 100.0 * flops / dt / 1e12 / PEAK_TFLOPS[dtype_name], "ms_by_kind": by_kind,
           "as_one_graph": {"steps_per_graph": steps, "ms_per_step": dt_graph * 1e3} if graph else None}
    if extras:
        res["tiny_config_loop"] = tiny_loop_bench()
    return res


def tiny_loop_bench(K=50):
    """configs[0] (batch 2, 32x32) training loop, where launches rather than arithmetic set the pace: K eager
    steps against K steps recorded into one HIP graph."""
    import torch
    from paper_1810_09868_amd import binding as B
    from paper_1810_09868_amd import synth
    from paper_1810_09868_amd.model import Vgg19
    cfg = synth.tiny_config(seed=0)
    m = Vgg19(B.F32, 2, 32, 32, 512, 10, lr=0.01, training=True)
    m.pack(cfg.conv_w, cfg.conv_b, cfg.fc_w, cfg.fc_b)
    x = torch.from_numpy(cfg.x).cuda()
    lab = torch.from_numpy(cfg.labels).cuda()
    for _ in range(3):
        m.train_step(x, lab)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        m.train_step(x, lab)
    torch.cuda.synchronize()
    eager = (time.perf_counter() - t0) / K
    g = m.capture_train_steps(x, lab, K)
    g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g.replay()
    torch.cuda.synchronize()
    graph = (time.perf_counter() - t0) / K
    return {"steps": K, "eager_ms_per_step": round(eager * 1e3, 4), "graph_ms_per_step": round(graph * 1e3, 4)}


def batch_sweep(dtype_name, batches, steps):
    """Forward pass at the other batch sizes of the paper's timing table (1 and 10 images): ms and images/s."""
    import torch
    from paper_1810_09868_amd import binding as B
    from paper_1810_09868_amd import synth
    from paper_1810_09868_amd.model import Vgg19
    dtype = B.BF16 if dtype_name == "bf16" else B.F32
    res = []
    for N in batches:
        inp = synth.full_config(N, seed=0, with_labels=False)
        m = Vgg19(dtype, N, 224, 224, 4096, 1000)
        m.pack(inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
        x = torch.from_numpy(inp.x).cuda()
        for _ in range(3):
            m.forward(x)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            m.forward(x)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        # the same passes recorded once and replayed as a single HIP graph
        g = m.capture_forward(x, steps)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        dtg = (time.perf_counter() - t0) / steps
        del g
        res.append({"batch": N, "ms_per_step": round(dt * 1e3, 4), "images_per_s": round(N / dt, 1),
                    "as_one_graph_ms_per_step": round(dtg * 1e3, 4)})
        del m
        torch.cuda.empty_cache()
    return res


def conv_microbench(steps):
    """configs[1]: one conv3_1-style layer, fp32, 128 -> 256 channels, 56x56, batch 100, bias + ReLU, through the
    single-operation entry point; N(0,1) inputs, He-normal weights.  ms, TFLOP/s and share of the fp32 MFMA peak."""
    import torch
    from paper_1810_09868_amd import binding as B
    from paper_1810_09868_amd import synth
    N, H, W, Cin, Cout = 100, 56, 56, 128, 256
    d = synth.conv_layer_inputs(N, H, W, Cin, Cout, seed=0)
    xs = torch.from_numpy(d["x"]).cuda()
    x = torch.empty((N, H, W, Cin), dtype=torch.float32, device="cuda")
    B.vgg_nchw_to_nhwc(B.F32, N, Cin, H, W, Cin, xs, x)
    wp = torch.empty((9, Cout, Cin), dtype=torch.float32, device="cuda")
    B.vgg_conv_pack_weights(B.F32, Cin, Cout, torch.from_numpy(d["w"]).cuda(), wp, 0)
    bias = torch.from_numpy(d["b"]).cuda()
    y = torch.empty((N, H, W, Cout), dtype=torch.float32, device="cuda")
    for _ in range(3):
        B.vgg_conv3x3_fwd(B.F32, N, H, W, Cin, Cout, x, wp, bias, y, 1, None)
    # (the binding launches on torch's current stream, which is the stream these events are recorded on)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        B.vgg_conv3x3_fwd(B.F32, N, H, W, Cin, Cout, x, wp, bias, y, 1, None)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    flops = 2.0 * N * H * W * 9 * Cin * Cout
    tf = flops / (ms * 1e-3) / 1e12
    byts = 4.0 * (N * H * W * (Cin + Cout) + 9 * Cin * Cout)
    return {"workload": "configs[1]: 3x3 conv 128->256, 56x56, batch 100, fp32, bias+ReLU (vgg_conv3x3_fwd)",
            "dtype": "f32", "ms": round(ms, 4), "gflop": round(flops / 1e9, 2), "tflops": round(tf, 2),
            "pct_fp32_mfma_peak": round(100.0 * tf / PEAK_TFLOPS["f32"], 2),
            "min_bytes_mb": round(byts / 1e6, 1), "gbs_at_min_bytes": round(byts / (ms * 1e-3) / 1e9, 1)}


def mfma_loop_ceiling():
    """TFLOP/s of a loop of nothing but MFMAs (register operands), constant and random operands: what the chip
    sustains at the clock it holds under matrix load, next to the data-sheet peak used for `roofline.peak`."""
    import torch
    from paper_1810_09868_amd import binding as B
    sink = torch.empty((B.vgg_mfma_probe_sink_bytes(),), dtype=torch.uint8, device="cuda")
    out = {}
    # (bf16: the 32x32x16 shape, and the 16x16x32 shape that the roofline kernel uses; about 10 ms per launch)
    for name, dt, iters, m16 in (("bf16", B.BF16, 20000, False), ("bf16_16x16x32", B.BF16, 20000, True), ("f32", B.F32, 10000, False)):
        for rnd in (False, True):
            B.vgg_mfma_probe(dt, rnd, iters // 2, sink, m16)   # warm-up: the clock settles under load
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = B.vgg_mfma_probe(dt, rnd, iters, sink, m16)
            e1.record()
            torch.cuda.synchronize()
            out["%s_%s_operands_tflops" % (name, "random" if rnd else "constant")] = round(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    return out


def operand_sensitivity(steps):
    """The forward benchmark's dominant kernel on one layer (bf16, 512 -> 512 channels, 28x28, batch 100, bias + ReLU,
    through vgg_conv3x3_fwd) with three kinds of operand values: N(0,1) activations with He-normal weights, the same
    activations after a ReLU (half of them zero, as inside the network) and one constant everywhere.  Same launches,
    same instruction stream: the spread is what the chip's power management does with the switching activity of
    the data, and it bounds what `roofline.frac` can reach on real values."""
    import torch
    from paper_1810_09868_amd import binding as B
    N, H, W, Cin, Cout = 100, 28, 28, 512, 512
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    x0 = torch.randn((N, H, W, Cin), device="cuda", generator=gen)
    w0 = torch.randn((Cout, Cin, 3, 3), device="cuda", generator=gen) * (2.0 / (9 * Cin)) ** 0.5
    bias = torch.full((Cout,), 0.01, device="cuda")
    y = torch.empty((N, H, W, Cout), dtype=torch.bfloat16, device="cuda")
    wsb = B.vgg_conv3x3_fwd_workspace_bytes(B.BF16, N, H, W, Cin, Cout)
    ws = torch.empty((max(wsb, 256),), dtype=torch.uint8, device="cuda") if wsb else None
    flops = 2.0 * N * H * W * 9 * Cin * Cout
    out = {"workload": "3x3 conv 512->512, 28x28, batch 100, bf16, bias+ReLU (vgg_conv3x3_fwd)",
           "kernel": B.vgg_conv3x3_plan(B.PLAN_FWD, B.BF16, N, H, W, Cin, Cout)[0]}
    cases = (("normal_activations", x0, w0), ("relu_activations", x0.clamp(min=0), w0),
             ("constant", torch.full_like(x0, 1.0), torch.full_like(w0, 1.0 / (9 * Cin))))
    for name, xf, wf in cases:
        x = xf.to(torch.bfloat16)
        w = torch.empty((9, Cout, Cin), dtype=torch.bfloat16, device="cuda")
        B.vgg_conv_pack_weights(B.BF16, Cin, Cout, wf, w, 0)
        for _ in range(3):
            B.vgg_conv3x3_fwd(B.BF16, N, H, W, Cin, Cout, x, w, bias, y, 1, ws)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            B.vgg_conv3x3_fwd(B.BF16, N, H, W, Cin, Cout, x, w, bias, y, 1, ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        out[name + "_tflops"] = round(flops / (ms * 1e-3) / 1e12, 1)
    return out


def cpu_baseline(inp, images):
    from oracle import vgg_ref as R
    t0 = time.perf_counter()
    R.vgg19_forward(inp.x[:images], inp.conv_w, inp.conv_b, inp.fc_w, inp.fc_b)
    dt = time.perf_counter() - t0
    return {"value": images / dt, "unit": "images/s", "cores": R.num_threads(), "kind": "oracle",
            "sample": "fp64 oracle forward pass on the first %d of the 100 images (%.1f s)" % (images, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--batch", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true")
    ap.add_argument("--cpu-images", type=int, default=24)
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also launch one plain 256 MiB device copy (convert_kernel<float,float>, 2^26 elements) "
                         "so that hardware byte counters can be scaled against a kernel of known traffic")
    ap.add_argument("--train-only", action="store_true",
                    help="profiling aid: time only the training step of --dtype (eager launches, no HIP graph) and "
                         "print its record instead of the forward benchmark's line")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this library runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library is the only implementation", file=sys.stderr)
        sys.exit(1)
    from paper_1810_09868_amd import binding as B
    from paper_1810_09868_amd import synth
    B.lib()
    if a.pmc_calibration:
        src = torch.zeros((1 << 26,), dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        B.vgg_convert(B.F32, B.F32, 1 << 26, src, dst)
        torch.cuda.synchronize()
        del src, dst
    if a.train_only:
        print(json.dumps(run_train_bench(a.batch, a.steps, dtype_name=a.dtype, extras=False, graph=False)))
        return
    inp = synth.full_config(a.batch, seed=0, with_labels=False)
    main_res = run_forward_bench(a.dtype, a.batch, a.steps, a.warmup, inp)
    out = {
        "metric": "VGG19 fwd images/s at batch 100, 224x224; conv TFLOP/s and % MFMA peak",
        "value": main_res["images_per_s"],
        "unit": "images/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if a.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": ("configs[3]: full VGG19 forward, bf16 weights/activations, fp32 MFMA accumulation, "
                                if a.dtype == "bf16" else "configs[2]: full VGG19 forward, fp32, ") +
                               "batch %d, 3x224x224, classifier 25088-4096-4096-1000" % a.batch,
                   "batch": a.batch, "image": "3x224x224"},
        "conv_tflops": main_res["conv_tflops"],
        "conv_ms_per_step": main_res["conv_ms_per_step"],
        "pct_mfma_peak_conv": main_res["pct_mfma_peak_conv"],
        "other_ms_per_step": main_res["other_ms_per_step"],
        "per_layer": main_res["per_layer"],
        "roofline": main_res["roofline"],
        "paper_context": {"tpu_v2_core_compute_s_batch100": 0.23, "flux_cpu_s_batch100": 52.4},
    }
    if not a.no_secondary:
        other = "f32" if a.dtype == "bf16" else "bf16"
        sec = run_forward_bench(other, a.batch, max(3, a.steps // 4), 2, inp)
        out["secondary"] = {"workload": "configs[2] fp32" if other == "f32" else "configs[3] bf16",
                            "dtype": other, "images_per_s": sec["images_per_s"], "ms_per_step": sec["ms_per_step"],
                            "conv_tflops": sec["conv_tflops"], "pct_mfma_peak_conv": sec["pct_mfma_peak_conv"],
                            "conv_ms_per_step": sec["conv_ms_per_step"], "other_ms_per_step": sec["other_ms_per_step"],
                            "per_layer": sec["per_layer"], "roofline": sec["roofline"]}
        out["conv_microbenchmark"] = conv_microbench(max(5, a.steps))
    if not a.no_secondary:
        out["train_step"] = run_train_bench(a.batch, max(2, a.steps // 5))
        out["train_step_bf16"] = run_train_bench(a.batch, max(2, a.steps // 2), dtype_name="bf16", extras=False)
        out["batch_sweep"] = batch_sweep(a.dtype, (1, 10), max(5, a.steps))
    out["mfma_loop_ceiling"] = mfma_loop_ceiling()
    if not a.no_secondary:
        out["operand_sensitivity"] = operand_sensitivity(max(10, a.steps))
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, min(a.cpu_images, a.batch))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
