"""Statistical efficiency of the weight policies under the emulated K-stage nF1B schedule.

The paper's central claim (Sections "Results", "Memory Overhead") is a trade: V-TiMePReSt keeps one
weight version per stage and needs more mini-batches to converge; I-TiMePReSt stashes the forward
versions (K - s per stage) and converges in fewer, by running the backward pass on an intermediate
weight.  Its datasets are not used here.  This module reproduces the *experiment* on synthetic
teacher-student data that needs none: a fixed random teacher network labels Gaussian inputs, a student
MLP split into K stages is trained through the stage library with real staleness from the schedule,
once per policy, and the loss per mini-batch and the stash memory per stage are tabulated.

    python -m paper_2509_23241_amd.convergence [--minibatches 600] [--width 256] [--stages 4] ...

Everything runs through the same C-ABI calls as the benchmark (stage_forward / stage_loss_softmax_ce /
stage_backward / stage_blend_update); this file only generates data and prints tables.
"""
from __future__ import annotations

import argparse
import json
import math
import sys
from typing import Dict, List

import numpy as np
import torch

import synth_inputs as S
from synth_inputs import workloads as W

from . import binding as B
from .runner import GpuPipeline


def student(width: int, in_dim: int, classes: int, stages: int, layers_per_stage: int, mb: int, n: int, lr: float,
            lam: float, dtype: str) -> W.Workload:
    specs = []
    fin = in_dim
    total = stages * layers_per_stage
    for i in range(total):
        last = i == total - 1
        specs.append(W.Dense(fin, classes if last else width, "none" if last else "gelu"))
        fin = width
    st = tuple(tuple(specs[s * layers_per_stage:(s + 1) * layers_per_stage]) for s in range(stages))
    return W.Workload(name=f"student{width}x{total}", dtype=dtype, stages=st, mb=mb, n=n, classes=classes, lr=lr, lam=lam)


class TeacherData:
    """x ~ N(0, 1); label = argmax of a fixed random two-layer tanh network.  Seeded, generated on the host."""

    def __init__(self, in_dim: int, hidden: int, classes: int, rows: int, device, dtype):
        self.in_dim, self.rows, self.device, self.dtype = in_dim, rows, device, dtype
        self.w1 = S.normal("teacher/w1", (in_dim, hidden), std=1.0 / math.sqrt(in_dim))
        self.w2 = S.normal("teacher/w2", (hidden, classes), std=4.0 / math.sqrt(hidden))
        self.cache: Dict[int, tuple] = {}

    def host(self, j: int):
        """(inputs in the storage type's values, labels) of mini-batch j as host arrays."""
        x = S.normal(f"teacher/x/{j}", (self.rows, self.in_dim))
        y = np.argmax(np.tanh(x @ self.w1) @ self.w2, axis=1).astype(np.int32)
        return (S.round_bf16(x) if self.dtype == torch.bfloat16 else S.round_f32(x)), y

    def _make(self, j: int):
        if j not in self.cache:
            x, y = self.host(j)
            self.cache[j] = (torch.from_numpy(x).to(self.device).to(self.dtype), torch.from_numpy(y).to(self.device))
        return self.cache[j]

    def inputs(self, j: int):
        return self._make(j)[0]

    def labels(self, j: int):
        return self._make(j)[1]


def run_policy(w: W.Workload, policy: str, data: TeacherData, minibatches: int, mid_pass_updates: bool = False):
    """Train through the stage library; TiMePReSt and mid-pass updates run on the micro-batch-granular clock."""
    params = [W.init_params(w, s) for s in range(w.K)]
    pipe = GpuPipeline(w, params, policy=policy)
    stash = [(st.C, int(st.C) * int(st.P) * 4) for st in pipe.stages]
    if policy == "timeprest" or mid_pass_updates:
        _, losses = pipe.run_microbatches(minibatches, data.inputs, data.labels, mid_pass_updates=mid_pass_updates)
    else:
        _, losses = pipe.run(minibatches, data.inputs, data.labels)
    out = torch.cat([losses[j] for j in range(minibatches)]).cpu().numpy().astype(np.float64)
    pipe.close()
    return out, stash


def first_below(loss: np.ndarray, threshold: float, window: int = 20):
    if len(loss) < window:
        return None
    avg = np.convolve(loss, np.ones(window) / window, mode="valid")
    hit = np.nonzero(avg < threshold)[0]
    return int(hit[0]) + window if len(hit) else None


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--minibatches", type=int, default=600)
    ap.add_argument("--width", type=int, default=256)
    ap.add_argument("--in-dim", type=int, default=64)
    ap.add_argument("--classes", type=int, default=16)
    ap.add_argument("--stages", type=int, default=4)
    ap.add_argument("--layers-per-stage", type=int, default=2)
    ap.add_argument("--mb", type=int, default=32)
    ap.add_argument("--n", type=int, default=4)
    ap.add_argument("--lr", type=float, default=0.02)
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--threshold", type=float, default=None, help="loss level for the 'mini-batches to reach' column "
                    "(default: 1.25 x the best final loss among the runs)")
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args(argv)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    tdt = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    rows = args.mb * args.n
    data = TeacherData(args.in_dim, 2 * args.in_dim, args.classes, rows, dev, tdt)

    def wl(stages, lam):
        lps = args.layers_per_stage * args.stages // stages
        return student(args.width, args.in_dim, args.classes, stages, lps, args.mb, args.n, args.lr, lam, args.dtype)

    runs = [("sequential SGD (1 stage, no staleness)", 1, "latest", 0.1),
            ("V-TiMePReSt (latest, no stash)", args.stages, "latest", 0.1),
            ("V-TiMePReSt, updates also in the middle of a pass", args.stages, "latest-mid", 0.1),
            ("TiMePReSt (versions of the pass start)", args.stages, "timeprest", 0.1),
            ("I-TiMePReSt Eq. 1, lambda 0.1", args.stages, "eq1", 0.1),
            ("I-TiMePReSt convex, lambda 0.1", args.stages, "convex", 0.1),
            ("I-TiMePReSt convex, lambda ln 2", args.stages, "convex", math.log(2.0)),
            ("I-TiMePReSt convex, lambda 2", args.stages, "convex", 2.0),
            ("stashed (backward on the forward version)", args.stages, "stashed", 0.1)]
    results = []
    for name, stages, policy, lam in runs:
        loss, stash = run_policy(wl(stages, lam), policy.replace("-mid", ""), data, args.minibatches,
                                 mid_pass_updates=policy.endswith("-mid"))
        results.append({"name": name, "stages": stages, "policy": policy, "lambda": lam, "loss": loss, "stash": stash})
        print(f"ran {name}: first {loss[:10].mean():.4f} last {loss[-50:].mean():.4f}", file=sys.stderr, flush=True)
    best_final = min(float(r["loss"][-50:].mean()) for r in results if np.isfinite(r["loss"][-50:].mean()))
    thr = args.threshold if args.threshold is not None else 1.25 * best_final
    marks = [m for m in (50, 100, 200, 400, args.minibatches) if m <= args.minibatches]
    if args.json:
        print(json.dumps([{k: (v.tolist() if isinstance(v, np.ndarray) else v) for k, v in r.items()} for r in results]))
        return
    print(f"student: {args.stages * args.layers_per_stage}-layer GELU MLP width {args.width}, {args.in_dim} -> {args.classes} classes, "
          f"{args.dtype}, micro-batch {args.mb} x {args.n}, SGD lr {args.lr} momentum 0.9, {args.minibatches} mini-batches; "
          f"loss = mean over the 50 mini-batches before the mark")
    print("| policy | " + " | ".join(f"loss @{m}" for m in marks) + f" | mini-batches to loss < {thr:.3f} | ring slots per stage | stash MB (all stages) |")
    print("|---|" + "---|" * (len(marks) + 3))
    for r in results:
        cells = [f"{r['loss'][max(0, m - 50):m].mean():.4f}" for m in marks]
        fb = first_below(r["loss"], thr)
        slots = "/".join(str(c) for c, _ in r["stash"])
        mbytes = sum(b for _, b in r["stash"]) / 1e6
        print(f"| {r['name']} | " + " | ".join(cells) + f" | {fb if fb is not None else 'not reached'} | {slots} | {mbytes:.2f} |")


if __name__ == "__main__":
    main()
