#!/usr/bin/env python3
"""Benchmark of the stage hot path on one MI355X.

One "step" is one steady-state mini-batch at a pipeline stage: the backward pass of the oldest
mini-batch in flight (dgrad + wgrad on the prescribed weights), the fused update that also builds
the intermediate weights of the next backward and writes the new version into the stash ring, and
the n micro-batch forwards of the mini-batch that enters.  The workload is the interior stage
(stage 1 of 4) of the 8-layer GELU MLP of width 4096, bf16 activations with fp32 master weights,
micro-batch 256 x 8, I-TiMePReSt blend, staleness 2 in steady state.  Inputs are seeded synthetic
tensors resident in HBM before the timed region.

Prints ONE JSON line: stage throughput in samples/s, the roofline of the dominant kernel (timed
with HIP events inside the timed region) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# Figures of the default workload taken with rocprofv3 on the library at commit 11d5330 (kernel sources of the three
# GEMMs and the update unchanged since); commands and raw counts in profiles/.
#   traffic: HBM-side bytes per launch from two --pmc runs (FETCH_SIZE, then WRITE_SIZE) scaled by what the same
#            counters read for a plain 1 GiB copy (FETCH_SIZE reports half the bytes, WRITE_SIZE all of them):
#            profiles/bench_mlp4096_stage1_hbm_traffic.md
#   rocprof_avg_us: average kernel duration from --kernel-trace --stats (no event brackets):
#            profiles/bench_mlp4096_stage1_kernel_stats.md
MEASURED_TRAFFIC_BYTES = {"fprop": 56.1e6, "dgrad": 159.5e6, "wgrad": 168.0e6, "update": 940.1e6,
                          "act_bwd": 52.5e6, "colsum": 19.0e6}
ROCPROF_AVG_US = {"fprop": 18.51, "dgrad": 68.31, "wgrad": 66.57, "update": 162.72, "act_bwd": 12.89}
PROFILED_AT = "8a38374"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--policy", default="convex", choices=["latest", "eq1", "convex", "stashed"])
    ap.add_argument("--workload", default="mlp", choices=["mlp", "vgg", "tfm", "bneck"],
                    help="mlp: interior stage of the width-4096 GELU MLP (the configuration the metric is quoted on); "
                         "vgg: stage 0 of the VGG-16-style net on 32x32x3 images (implicit-GEMM convolutions); "
                         "tfm: interior stage of the decoder-only transformer (4 blocks, d_model 2048, 1024 tokens); "
                         "bneck: the conv4_x group of the ResNet-50-style net (six bottlenecks, 8x8 -> 4x4 maps; "
                         "--stage 1: its conv3_x group, four bottlenecks, 16x16 -> 8x8; --stage 0: stem and conv2_x; "
                         "--stage 3: conv5_x, average pooling, classifier)")
    ap.add_argument("--blocks", type=int, default=4, help="transformer blocks in the tfm stage")
    ap.add_argument("--stage", type=int, default=None)
    ap.add_argument("--width", type=int, default=4096)
    ap.add_argument("--mb", type=int, default=None, help="micro-batch size (default 256 mlp, 64 vgg, 8 tfm)")
    ap.add_argument("--n", type=int, default=None, help="micro-batches per mini-batch (default 8 mlp, 4 vgg, 4 tfm)")
    ap.add_argument("--repeats", type=int, default=5,
                    help="timed blocks of --steps steps each; the line reports the median block (and all of them)")
    ap.add_argument("--forward-streams", type=int, default=None, choices=[0, 1, 2, 3],
                    help="streams of their own for the forward passes: micro-batch ub runs on stream ub mod N, beside the "
                         "backward pass of an earlier mini-batch on the stage's stream; 0: everything on the stage's "
                         "stream (default 2; 3 for a last stage, whose own stream takes a turn; stages with attention layers: 0)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-minibatches", type=int, default=3)
    ap.add_argument("--copy-probe", type=int, default=0, metavar="BYTES",
                    help="only run a plain device copy of BYTES bytes (5 untimed, 10 timed) and exit (calibration of the "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def layer_work(cls, layer, rows, mb):
    """Algorithmic (flops, bytes) of ONE launch of kernel class `cls` for one layer; rows = samples of a
    mini-batch (backward kernels), mb = samples of a micro-batch (forward kernels)."""
    if layer.kind == "pool":
        return 0.0, 0.0
    if layer.kind in ("ln", "attn", "res", "bn", "sub", "swap", "avg"):
        return 0.0, 0.0
    # GEMM rows per sample (output pixels of a convolution) and input pixels per sample (more with stride 2)
    px = layer.ho * layer.wo if layer.kind == "conv" else getattr(layer, "tokens", 1)
    pin = layer.h * layer.w if layer.kind == "conv" else px
    fin = (layer.k * layer.k * layer.cin) if layer.kind == "conv" else layer.in_features
    cin = layer.cin if layer.kind == "conv" else layer.in_features
    fout = layer.cout if layer.kind == "conv" else layer.out_features
    if cls == "fprop":                 # x, W in; act'(z), a out
        return 2.0 * mb * px * fin * fout, 2.0 * (mb * pin * cin + fin * fout + 2 * mb * px * fout)
    if cls == "dgrad":                 # dz, W_b, act'(z_prev) in; dz_prev out
        return 2.0 * rows * px * fin * fout, 2.0 * (rows * px * fout + fin * fout + 2 * rows * pin * cin)
    if cls == "wgrad":                 # dz, x in; dW (fp32) out
        return 2.0 * rows * px * fin * fout, 2.0 * (rows * px * fout + rows * pin * cin) + 4.0 * fin * fout
    if cls == "colsum":
        return 0.0, 2.0 * rows * px * fout
    return 0.0, 0.0


def kernel_work(cls, w, s, needs_dx):
    """Algorithmic work of one STEP in kernel class cls at stage s: (flops, bytes), summed over the
    launches of the step; divided by the launches it is the per-launch figure."""
    layers = w.stages[s]
    rows = w.n * w.mb
    P = sum(int(np_prod(sh)) for l in layers for sh in l.param_shapes())
    if cls == "update":                # g, m, W[v], W[v_f] in; m, W[v+1] fp32 + two bf16 copies out
        return 8.0 * P, 28.0 * P
    if cls == "act_bwd":               # dy (.) act'(z) at the stage output and behind every pool
        tot = 0.0
        for i, l in enumerate(layers):
            if l.kind in ("dense", "conv") and (i == len(layers) - 1 or layers[i + 1].kind != "dense" and
                                                 layers[i + 1].kind != "conv") and l.act != "none":
                tot += 3 * 2.0 * rows * l.out_dim()
        return 0.0, tot
    if cls == "pool":                  # forward: in + out; backward: in, out, dy in, dx out
        tot = 0.0
        for l in layers:
            if l.kind == "pool":
                e = l.c * l.h * l.w
                tot += 2.0 * rows * (e + e / 4) + 2.0 * rows * (2 * e + 2 * e / 4)
            if l.kind == "sub":        # forward: a quarter in, a quarter out; backward: a quarter in, all out
                e = l.c * l.h * l.w
                tot += 2.0 * rows * (e / 2) + 2.0 * rows * (e / 4 + e)
            if l.kind == "avg":        # forward: all positions in, the means out; backward: their gradients in, all out
                tot += 2 * 2.0 * rows * (l.c * l.tokens + l.c)
        return 0.0, tot
    if cls == "norm":                  # forward: x in, y out; backward: dy, x in, dx out
        tot = sum(2.0 * rows * l.out_dim() * 5 for l in layers if l.kind == "ln")
        # batch norm, every operand once: forward x in, a out (a ReLU's derivative is read off a); backward dy, x in,
        # dx out; the tensor a fused residual add reads is left out
        tot += sum(2.0 * rows * l.out_dim() * (2 + 3) for l in layers if l.kind == "bn")
        return 0.0, tot
    if cls == "add":                   # forward a + b -> out; backward the same on gradients
        tot = sum(2.0 * rows * l.out_dim() * 3 * 2 for l in layers if l.kind == "res" and l.mark == "add")
        return 0.0, tot
    if cls == "attn":                  # causal: half of the S x S scores; QK^T and PV forward, five products backward
        fl = by = 0.0
        for l in layers:
            if l.kind == "attn":
                fl += rows * 7 * 2.0 * l.tokens * l.tokens * l.d / 2
                by += 2.0 * rows * l.tokens * l.d * (4 + 8)
        return fl, by
    if cls == "copy":                  # stage input saved for the backward where no GEMM can fuse it
        l = layers[0]
        return 0.0, (2 * 2.0 * rows * np_prod(l.in_shape())) if l.kind in ("conv", "res", "ln", "bn") else 0.0
    flops = nbytes = 0.0
    for i, l in enumerate(layers):
        if l.kind in ("pool", "ln", "attn", "res", "bn", "sub", "swap", "avg"):
            continue
        if cls == "dgrad" and i == 0 and not needs_dx:
            continue
        if cls == "colsum" and i == len(layers) - 1 and l.act != "none" and w.dtype == "bf16" and l.out_dim() % 8 == 0:
            continue   # the stage's last layer: its column sums come out of the kernel that forms dz = dy (.) act'(z)
        if cls == "colsum" and i + 1 < len(layers) and layers[i + 1].kind == "bn" and l.act == "none":
            # the bias gradient comes out of the normalisation's backward kernel (layers of up to 2048 rows per
            # micro-batch, whole 16-byte units of channels): no pass over dz of its own
            px = l.ho * l.wo if l.kind == "conv" else getattr(l, "tokens", 1)
            if w.mb * px <= 2048 and (l.cout if l.kind == "conv" else l.out_features) % 8 == 0:
                continue
        f, b = layer_work(cls, l, rows, w.mb)
        mult = w.n if cls == "fprop" else 1
        flops += mult * f
        nbytes += mult * b
    return flops, nbytes


def np_prod(shape):
    out = 1
    for v in shape:
        out *= int(v)
    return out


def cpu_baseline(w, s, policy, minibatches):
    """The oracle as it stands, timed on the host: the same stage, the same step, fp64 numpy.  The transformer
    stage is timed on mini-batches of one sequence (the oracle's cost is linear in the number of sequences)."""
    from dataclasses import replace
    if w.name.startswith("tfm"):
        w = replace(w, mb=1, n=1)
        minibatches = 1
    if w.name.startswith("resnet"):
        minibatches = 1
    import numpy as np
    from oracle.stage import Stage
    from synth_inputs import workloads as W
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    params = W.init_params(w, s)
    st = Stage(w.stages[s], params, policy=policy, lam=w.lam, lr=w.lr, momentum=w.momentum, n=w.n,
               first_stage=(s == 0))
    depth = w.K - s
    xs = [W.stage_input(w, s, j) for j in range(2)]
    dys = [W.stage_upstream_grad(w, s, j, mean_loss=True) for j in range(2)]

    def fwd(j):
        x = xs[j % 2]
        for ub in range(w.n):
            st.forward(j, ub, x[ub * w.mb:(ub + 1) * w.mb])

    for j in range(depth):
        fwd(j)
    t0 = time.perf_counter()
    for j in range(minibatches):
        st.backward(j, dys[j % 2])
        st.update(j)
        fwd(j + depth)
    dt = time.perf_counter() - t0
    return {"value": minibatches * w.n * w.mb / dt, "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{minibatches} steady-state mini-batches of {w.n} x {w.mb} samples ({minibatches * w.n * w.mb} samples) "
                      f"of the same stage, numpy fp64, {dt:.1f} s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (one pipeline stage per GPU; no collectives are part "
              "of it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    if args.copy_probe:
        src = torch.ones(args.copy_probe // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 100.0
        print(json.dumps({"copy_probe_bytes": args.copy_probe, "copies": 15, "avg_us": round(us, 1),
                          "gbs_read_plus_write": round(2 * args.copy_probe / us * 1e-3, 1)}))
        return
    from paper_2509_23241_amd import binding as B
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple
    from synth_inputs import workloads as W

    if args.workload == "mlp":
        w = W.mlp_wide(width=args.width, mb=args.mb or 256, n=args.n or 8)
        s = 1 if args.stage is None else args.stage
        what = f"stage {s} of the 4-stage 8-layer GELU MLP width {args.width}"
    elif args.workload == "vgg":
        w = W.vgg_stage0(mb=args.mb or 64, n=args.n or 4)
        s = 0
        if args.stage not in (None, 0):
            sys.exit("bench.py: the vgg workload describes stage 0 only")
        what = ("stage 0 (conv3-64, conv3-64, pool, conv3-128, conv3-128, pool; ReLU) of the 4-stage VGG-16-style "
                "net on 32x32x3 images")
    elif args.workload == "bneck":
        s = 2 if args.stage is None else args.stage
        if s not in (0, 1, 2, 3):
            sys.exit("bench.py: the bneck workload has stages 0 .. 3")
        w = (W.resnet_middle_stages if s in (1, 2) else W.resnet_stages)(mb=args.mb or 128, n=args.n or 4)
        what = {0: "stage 0 (7x7 stride-2 stem 3 -> 64 channels, batch normalisation, ReLU, 2x2 max pooling, then the "
                   "conv2_x group on 16x16 maps: a projection bottleneck 64 -> 256 and two identity bottlenecks "
                   "256-64-64-256",
                1: "stage 1 (the conv3_x group: first bottleneck 256 -> 512 channels with the 3x3 at stride 2, 16x16 -> 8x8 "
                   "feature maps, and a projection shortcut, then three identity bottlenecks 512-128-128-512",
                2: "stage 2 (the conv4_x group: first bottleneck 512 -> 1024 channels with the 3x3 at stride 2, 8x8 -> 4x4 "
                   "feature maps, and a projection shortcut, then five identity bottlenecks 1024-256-256-1024",
                3: "stage 3 (the conv5_x group: first bottleneck 1024 -> 2048 channels with the 3x3 at stride 2, 4x4 -> 2x2 "
                   "feature maps, and a projection shortcut, then two identity bottlenecks 2048-512-512-2048, global "
                   "average pooling and the classifier 2048 -> 200"}[s]
        what += ("; batch normalisation per micro-batch, ReLU) of the 4-stage ResNet-50-style net on 64x64x3 images")
    else:
        w = W.transformer_stage(layers=args.blocks, mb=args.mb or 8, n=args.n or 4)
        s = 1
        if args.stage not in (None, 1):
            sys.exit("bench.py: the tfm workload describes stage 1 only")
        what = (f"stage 1 ({args.blocks} pre-norm decoder blocks, d_model 2048, 16 heads, FFN 8192, 1024 tokens; a sample "
                "is one sequence) of the 4-stage decoder-only transformer")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    depth = w.K - s
    layers = [layer_tuple(l) for l in w.stages[s]]
    # micro-batch forwards on two streams where the stage's forward kernels share no scratch memory
    # a stage that holds one mini-batch at a time (the last one) cannot run forwards beside a backward pass; its own
    # stream then takes a turn with the forward streams: three of them make four in all
    fstreams = args.forward_streams if args.forward_streams is not None else \
        (3 if w.K - s == 1 else {"mlp": 2, "vgg": 2, "bneck": 2}.get(args.workload, 0))
    if any(l.kind == "attn" for l in w.stages[s]):
        fstreams = 0
    two_streams = fstreams > 0
    st = GpuStage(layers, W.init_params(w, s), dtype=w.dtype, mb=w.mb, n=w.n, stage_index=s, num_stages=w.K,
                  policy=args.policy, lam=w.lam, lr=w.lr, momentum=w.momentum, needs_dx=(s > 0), device=dev,
                  forward_stream=fstreams)
    tdt = st.tdtype
    rows = w.n * w.mb
    nbuf = 2                                       # distinct synthetic mini-batches, resident in HBM
    xs = [torch.from_numpy(W.stage_input(w, s, j).reshape(rows, -1)).to(dev).to(tdt) for j in range(nbuf)]
    dys = [torch.from_numpy(W.stage_upstream_grad(w, s, j, mean_loss=True).reshape(rows, -1)).to(dev).to(tdt) for j in range(nbuf)]
    y = torch.empty(rows, st.out_elems, dtype=tdt, device=dev)
    dx = torch.empty(rows, st.in_elems, dtype=tdt, device=dev) if st.needs_dx else None

    def forward(j):
        x = xs[j % nbuf]
        for ub in range(w.n):
            st.forward(j, ub, x[ub * w.mb:(ub + 1) * w.mb], y[ub * w.mb:(ub + 1) * w.mb])

    def step(j):
        st.backward(j, dys[j % nbuf], dx)
        st.blend_update(j, j + 1 if depth > 1 else B.TP_NONE)
        forward(j + depth)

    for j in range(depth):                         # fill the stage: K - s mini-batches in flight
        forward(j)
    j = 0
    for _ in range(args.warmup):
        step(j)
        j += 1
    # pass 1: blocks of EXACTLY `steps` steps, nothing but the path itself on the stream, each bracketed by a
    # device synchronisation on both sides -> value from the median block, the others reported beside it
    block_ms = []
    for _ in range(max(1, args.repeats)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(j)
            j += 1
        torch.cuda.synchronize()
        block_ms.append((time.perf_counter() - t0) / args.steps * 1e3)
    dt = sorted(block_ms)[len(block_ms) // 2] * 1e-3 * args.steps
    # what an event pair with nothing between it reads on this stream (reported only: an event-bracketed kernel
    # duration carries part of it -- about 2 us against rocprofv3's kernel durations, which are in profiles/ and
    # quoted beside the roofline below)
    pairs = []
    for _ in range(200):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        e1.record()
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    event_pair_us = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)[len(pairs) // 2]
    # pass 2: the same `steps` steps again with every kernel bracketed by HIP events on the stage's
    # stream -> per-kernel durations for the roofline.  (The event pairs cost several microseconds of
    # pipeline bubble each, which is why they are kept out of the pass that `value` comes from.)
    B.stage_profile_begin(st.handle, args.steps * (8 + 2 * len(layers) * (w.n + 2)) + 64)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step(j)
        j += 1
    torch.cuda.synchronize()
    dt_prof = time.perf_counter() - t1
    prof = B.stage_profile_end(st.handle)
    q = st.query()
    delta_steady = min(depth - 1, int(q.latest_version))

    ms_per_step = dt / args.steps * 1e3
    value = rows / (dt / args.steps)
    kernels = {}
    for cls in B.KERNEL_CLASSES:
        launches, ms = prof[cls]
        if launches == 0:
            continue
        per_step = launches / args.steps
        flops, nbytes = (v / per_step for v in kernel_work(cls, w, s, st.needs_dx))
        avg_us = ms / launches * 1e3
        kernels[cls] = {"launches_per_step": launches / args.steps, "avg_us": round(avg_us, 2),
                        "share_of_step": round(ms / args.steps / (dt_prof / args.steps * 1e3), 4),
                        "tflops": round(flops / (avg_us * 1e-6) / 1e12, 2) if flops else None,
                        "gbs": round(nbytes / (avg_us * 1e-6) / 1e9, 1) if nbytes else None}
    dominant = max(kernels, key=lambda c: kernels[c]["share_of_step"])
    dk = kernels[dominant]
    flops, nbytes = (v / dk["launches_per_step"] for v in kernel_work(dominant, w, s, st.needs_dx))
    # the roofline that bounds one launch: matrix cores or HBM, whichever takes longer at peak
    t_mfma = flops / (PEAK_BF16_TFLOPS * 1e12)
    t_hbm = nbytes / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        achieved = flops / (dk["avg_us"] * 1e-6) / 1e12
        roofline = {"kernel": dominant, "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": None}
    else:
        achieved = nbytes / (dk["avg_us"] * 1e-6) / 1e9
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None}
    default_workload = (args.workload, args.width, w.mb, w.n, s, args.policy) == ("mlp", 4096, 256, 8, 1, "convex")
    roofline["traffic"] = MEASURED_TRAFFIC_BYTES.get(dominant) if default_workload else None
    if default_workload and dominant in ROCPROF_AVG_US:
        # the same ratio from rocprofv3's kernel duration (another run, another box of the pool): no event brackets
        work = nbytes if roofline["bound"] == "hbm" else flops
        peak = PEAK_HBM_GBS * 1e9 if roofline["bound"] == "hbm" else PEAK_BF16_TFLOPS * 1e12
        roofline["rocprof_avg_us"] = ROCPROF_AVG_US[dominant]
        roofline["frac_rocprof"] = round(work / (ROCPROF_AVG_US[dominant] * 1e-6) / peak, 4)
        roofline["profiled_at_commit"] = PROFILED_AT
    roofline["algorithmic"] = nbytes if roofline["bound"] == "hbm" else flops
    roofline["avg_us"] = dk["avg_us"]
    roofline["launches_per_step"] = dk["launches_per_step"]
    out = {
        "metric": "stage fwd+bwd samples/s on 1 MI355X; MFMA util %; blend/update HBM GB/s",
        "value": round(value, 1), "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "repeats": len(block_ms),
        "ms_per_step_blocks": [round(v, 4) for v in block_ms],
        "ms_per_step_spread_pct": round(100 * (max(block_ms) - min(block_ms)) / ms_per_step, 2),
        "ms_per_step_with_events": round(dt_prof / args.steps * 1e3, 4), "event_pair_us": round(event_pair_us, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{what}: bf16 activations, "
                               f"fp32 master weights, micro-batch {w.mb} x {w.n}, policy {args.policy}, "
                               f"lambda {w.lam}, staleness {delta_steady}, one step = 1 backward + 1 fused update/blend "
                               f"+ {w.n} micro-batch forwards"
                               + (f" (the forwards on {fstreams} streams of their own, beside the backward pass of the "
                                  "next mini-batch on the stage's stream; the per-kernel durations below are taken with "
                                  "everything on the stage's stream)" if two_streams else ""),
                   "params_per_stage": int(st.P), "ring_slots": int(st.C), "forward_streams": fstreams},
        "roofline": roofline,
        "kernels": kernels,
        "mfma_util_pct": {c: round(100 * kernels[c]["tflops"] / PEAK_BF16_TFLOPS, 2)
                          for c in ("fprop", "dgrad", "wgrad") if c in kernels},
        "update_hbm_gbs": kernels.get("update", {}).get("gbs"),
        "profile_dropped": prof["dropped"],
    }
    st.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, s, args.policy, args.cpu_minibatches)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
