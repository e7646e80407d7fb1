"""Device memory a stage holds, by weight policy (Section "Memory Overhead"; the paper's Figures 6 and 8 plot it
per worker): V-TiMePReSt keeps one weight version and never builds intermediate weights; the stashing policies keep
K - s versions at stage s plus the compute copy of the intermediate weights.  Everything comes from the library's own
stage_workspace_query (host only, no GPU): ring, momentum, gradient, compute copies, saved activations of the
mini-batches in flight, scratch.

    python -m paper_2509_23241_amd.footprint
"""
from __future__ import annotations

from typing import Dict, List

from synth_inputs import workloads as W

from . import binding as B
from .runner import layer_tuple

PARTS = ("ring_bytes", "momentum_bytes", "grad_bytes", "wfwd_bytes", "wbwd_bytes", "act_bytes", "scratch_bytes")


def timeprest_versions(K: int, n: int, s: int, num_mb: int = 16) -> int:
    """How many consecutive weight versions stage s must be able to hold under TiMePReSt: the latest one and those
    that passes under way still read (pinned when a pass starts at its first stage, dropped when the pass has left
    this stage), replayed on the library's micro-batch clock."""
    events = B.tp_schedule_microbatch_events(K, num_mb, n, False)
    version = [0] * K
    fwd, bwd, pins, widest = {}, {}, {}, 1
    for (t, kind, st, j, ub) in events:
        if kind == "F":
            if st == 0 and ub == 0:
                fwd[j] = list(version)
                pins[("f", j)] = fwd[j][s]
            if st == s and ub == n - 1:
                pins.pop(("f", j))
        else:
            if st == K - 1:
                bwd[j] = list(version)
                pins[("b", j)] = bwd[j][s]
            if st == s:
                pins.pop(("b", j))
            version[st] += 1
        held = set(pins.values()) | {version[s]}
        widest = max(widest, max(held) - min(held) + 1)
    return widest


def stage_bytes(w: W.Workload, s: int, policy: str) -> Dict[str, int]:
    """Bytes per buffer of stage s of workload w under `policy`, with the ring and in-flight depth of the nF1B schedule."""
    depth = w.K - s
    ring = 1 if policy == "latest" else timeprest_versions(w.K, w.n, s) if policy == "timeprest" else depth
    d = B.make_desc([layer_tuple(l) for l in w.stages[s]], dtype=w.dtype, mb=w.mb, n=w.n, stage_index=s, num_stages=w.K,
                    ring_capacity=ring, max_in_flight=depth, policy=policy,
                    needs_dx=s > 0, lam=w.lam, lr=w.lr, momentum=w.momentum)
    sz = B.stage_workspace_query(d)
    out = {k: int(getattr(sz, k)) for k in PARTS}
    out["params"] = int(sz.param_count)
    out["versions"] = ring
    out["total"] = sum(out[k] for k in PARTS)
    return out


def table(rows: List[tuple]) -> str:
    lines = ["| workload, stage | policy | parameters | ring (versions) | momentum + gradient | compute copies | saved activations | scratch | total MB |",
             "|---|---|---|---|---|---|---|---|---|"]
    for name, w, s in rows:
        for policy, label in (("latest", "V-TiMePReSt"), ("timeprest", "TiMePReSt"), ("convex", "I-TiMePReSt / stashed")):
            b = stage_bytes(w, s, policy)
            versions = b["versions"]
            mb = lambda v: f"{v / 1e6:.1f}"
            lines.append(f"| {name}, stage {s} | {label} | {b['params'] / 1e6:.2f} M | {mb(b['ring_bytes'])} ({versions}) | "
                         f"{mb(b['momentum_bytes'] + b['grad_bytes'])} | {mb(b['wfwd_bytes'] + b['wbwd_bytes'])} | "
                         f"{mb(b['act_bytes'])} | {mb(b['scratch_bytes'])} | {mb(b['total'])} |")
    return "\n".join(lines)


def default_rows() -> List[tuple]:
    mlp = W.mlp_wide()
    rows = [("MLP width 4096", mlp, s) for s in range(mlp.K)]
    rows.append(("VGG-style 32x32", W.vgg_stage0(), 0))
    res = W.resnet_middle_stages()
    rows += [("ResNet-style conv3_x", res, 1), ("ResNet-style conv4_x", res, 2)]
    rows.append(("transformer d 2048", W.transformer_stage(), 1))
    return rows


if __name__ == "__main__":
    print(table(default_rows()))
