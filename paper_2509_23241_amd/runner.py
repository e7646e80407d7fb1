"""Torch-side plumbing around the C ABI: device buffers, streams, and the one-GPU emulation of
the K-stage nF1B schedule.  No arithmetic of the method happens here -- every step runs in the
library's kernels; this module only allocates memory, uploads inputs and calls the ABI in the
order the library's own schedule generator gives.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def layer_tuple(spec) -> tuple:
    """Workload layer description -> the tuple format of binding.make_desc."""
    kind = getattr(spec, "kind", "dense")
    if kind == "conv":
        assert spec.k in (1, 3, 5, 7) and spec.pad == (spec.k - 1) // 2 and spec.stride in (1, 2), \
            "convolutions are built for kernels 1, 3, 5, 7 with stride 1 or 2 and pad (kernel-1)/2"
        return ("conv", spec.cin, spec.cout, spec.h, spec.w, spec.act, spec.stride, spec.k)
    if kind == "pool":
        return ("pool", spec.c, spec.h, spec.w)
    if kind == "sub":
        return ("sub", spec.c, spec.h, spec.w)
    if kind == "avg":
        return ("avg", spec.c, spec.tokens)
    if kind == "swap":
        return ("swap", spec.d, spec.tokens, spec.out_d, spec.out_tokens)
    if kind == "ln":
        return ("ln", spec.d, spec.tokens)
    if kind == "attn":
        return ("attn", spec.d, spec.heads, spec.tokens)
    if kind == "res":
        return ("res", spec.d, spec.tokens, spec.mark, spec.act)
    if kind == "bn":
        return ("bn", spec.c, spec.tokens, spec.act)
    return (spec.in_features, spec.out_features, spec.act, getattr(spec, "tokens", 1))


def _torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


class GpuStage:
    """One pipeline stage on the current device; owns the torch tensors the library works in."""

    def __init__(self, layers: Sequence[tuple], params: Optional[List[np.ndarray]], *, dtype: str, mb: int, n: int,
                 stage_index: int, num_stages: int, policy: str, lam: float, lr: float, momentum: float,
                 ring_capacity: Optional[int] = None, max_in_flight: Optional[int] = None,
                 needs_dx: Optional[bool] = None, device="cuda:0", stream: Optional[torch.cuda.Stream] = None,
                 forward_stream=False):
        """forward_stream: False / 0, or how many streams (default priority; True = 1) the stage gets for the forward
        passes; what runs there is ordered on the stage's stream by forward_join() or any later call other than a
        forward or a backward (a backward waits for the forwards of its own mini-batch only)."""
        self.layers = [tuple(l) for l in layers]
        self.in_elems = B.layer_in_elems(self.layers[0])      # values per sample in / out of the stage
        self.out_elems = B.layer_out_elems(self.layers[-1])
        self.dtype, self.mb, self.n = dtype, mb, n
        self.s, self.K = stage_index, num_stages
        depth = num_stages - stage_index
        if ring_capacity is None:
            # TiMePReSt: a pass under way may still read a version up to K - 1 updates older than the latest
            ring_capacity = 1 if policy == "latest" else (num_stages if policy == "timeprest" else depth)
        if max_in_flight is None:
            max_in_flight = depth
        if needs_dx is None:
            needs_dx = stage_index > 0
        self.needs_dx = needs_dx
        self.desc = B.make_desc(self.layers, dtype=dtype, mb=mb, n=n, stage_index=stage_index,
                                num_stages=num_stages, ring_capacity=ring_capacity, max_in_flight=max_in_flight,
                                policy=policy, needs_dx=needs_dx, lam=lam, lr=lr, momentum=momentum)
        self.sizes = B.stage_workspace_query(self.desc)
        self.P = self.sizes.param_count
        self.C = ring_capacity
        self.device = torch.device(device)
        self.tdtype = _torch_dtype(dtype)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        dev = self.device

        def raw(nbytes):
            return torch.zeros(max(int(nbytes), 256), dtype=torch.uint8, device=dev)

        self.ring = torch.zeros(self.C * self.P, dtype=torch.float32, device=dev)
        self.momentum = torch.zeros(self.P, dtype=torch.float32, device=dev)
        self.grad = torch.zeros(self.P, dtype=torch.float32, device=dev)
        self.wfwd = torch.zeros(self.P if dtype == "bf16" else 64, dtype=torch.bfloat16, device=dev)
        self.wbwd = torch.zeros(max(self.sizes.wbwd_bytes // (2 if dtype == "bf16" else 4), 64), dtype=self.tdtype, device=dev)
        self.act = raw(self.sizes.act_bytes)
        self.scratch = raw(self.sizes.scratch_bytes)
        self.diag = torch.zeros(B.TP_DIAG_COUNT, dtype=torch.float64, device=dev)
        if params is not None:
            self.ring[: self.P].copy_(torch.from_numpy(self.pack(params)).to(dev))
        bufs = B.tp_buffers(self.ring.data_ptr(), self.momentum.data_ptr(), self.grad.data_ptr(),
                            self.wfwd.data_ptr(), self.wbwd.data_ptr(), self.act.data_ptr(),
                            self.scratch.data_ptr(), self.diag.data_ptr())
        with torch.cuda.stream(self.stream):
            self.handle = B.stage_init(self.desc, bufs, self.stream.cuda_stream)
        self.fwd_streams = [torch.cuda.Stream(self.device) for _ in range(int(forward_stream))]
        if self.fwd_streams:
            B.stage_set_forward_streams(self.handle, [q.cuda_stream for q in self.fwd_streams])

    # -- parameter arena <-> per-layer arrays (pure indexing) -----------------
    def pack(self, params: List[np.ndarray]) -> np.ndarray:
        """Flat list [W, b, W, b, ...] over the layers that have parameters -> padded arena."""
        flat = np.zeros(self.P, dtype=np.float32)
        pi = 0
        for l, spec in enumerate(self.layers):
            shapes = B.layer_param_shapes(spec)
            if not shapes:
                continue
            wo, bo = self.sizes.w_offset[l], self.sizes.b_offset[l]
            nw, nb = int(np.prod(shapes[0])), int(np.prod(shapes[1]))
            flat[wo: wo + nw] = np.asarray(params[pi], dtype=np.float32).reshape(-1)
            flat[bo: bo + nb] = np.asarray(params[pi + 1], dtype=np.float32).reshape(-1)
            pi += 2
        return flat

    def unpack(self, flat) -> List[np.ndarray]:
        flat = np.asarray(flat)
        out = []
        for l, spec in enumerate(self.layers):
            shapes = B.layer_param_shapes(spec)
            if not shapes:
                continue
            wo, bo = self.sizes.w_offset[l], self.sizes.b_offset[l]
            out.append(flat[wo: wo + int(np.prod(shapes[0]))].reshape(shapes[0]))
            out.append(flat[bo: bo + int(np.prod(shapes[1]))])
        return out

    # -- calls ----------------------------------------------------------------
    def forward(self, mb_id: int, ub: int, x: torch.Tensor, y: Optional[torch.Tensor] = None):
        if y is None:
            y = torch.empty(self.mb, self.out_elems, dtype=self.tdtype, device=self.device)
        assert x.is_contiguous() and y.is_contiguous() and x.dtype == self.tdtype and y.dtype == self.tdtype
        assert x.shape[0] == self.mb and x.numel() == self.mb * self.in_elems
        assert y.shape[0] == self.mb and y.numel() == self.mb * self.out_elems
        v = B.stage_forward(self.handle, mb_id, ub, x.data_ptr(), y.data_ptr())
        return y, v

    def forward_join(self):
        B.stage_forward_join(self.handle)

    def forward_on(self, mb_id: int, ub: int, version: int, x: torch.Tensor, y: torch.Tensor):
        """Forward on a retained version (TP_TIMEPREST)."""
        assert x.is_contiguous() and y.is_contiguous() and x.dtype == self.tdtype and y.dtype == self.tdtype
        assert x.numel() == self.mb * self.in_elems and y.numel() == self.mb * self.out_elems
        B.stage_forward_on(self.handle, mb_id, ub, version, x.data_ptr(), y.data_ptr())
        return y

    def backward_on(self, mb_id: int, version: int, dy: torch.Tensor, dx: Optional[torch.Tensor] = None):
        """Backward on a retained version (TP_TIMEPREST)."""
        rows = self.mb * self.n
        assert dy.numel() == rows * self.out_elems and dy.is_contiguous() and dy.dtype == self.tdtype
        if self.needs_dx and dx is None:
            dx = torch.empty(rows, self.in_elems, dtype=self.tdtype, device=self.device)
        B.stage_backward_on(self.handle, mb_id, version, dy.data_ptr(), dx.data_ptr() if dx is not None else 0)
        return dx

    def input_view(self, mb_id: int, ub: int) -> torch.Tensor:
        """Tensor view of the workspace rows where the input of (mb_id, ub) belongs."""
        ptr = B.stage_input_ptr(self.handle, mb_id, ub)
        off = ptr - self.act.data_ptr()
        nbytes = self.mb * self.in_elems * self.act_elt()
        return self.act[off: off + nbytes].view(self.tdtype).view(self.mb, self.in_elems)

    def saved_input(self, mb_id: int, ub: int, layer: int) -> torch.Tensor:
        """Tensor view [mb, values per sample] of the input the stage saved for `layer` (inspection only)."""
        ptr, nbytes = B.stage_saved_input_ptr(self.handle, mb_id, ub, layer)
        off = ptr - self.act.data_ptr()
        return self.act[off: off + nbytes].view(self.tdtype).view(self.mb, -1)

    def act_elt(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    def loss(self, mb_id: int, logits: torch.Tensor, labels: torch.Tensor):
        rows = self.mb * self.n
        assert logits.shape == (rows, self.out_elems) and logits.is_contiguous() and logits.dtype == self.tdtype
        assert labels.dtype == torch.int32 and labels.shape == (rows,)
        dlogits = torch.empty_like(logits)
        loss = torch.empty(1, dtype=torch.float32, device=self.device)
        B.stage_loss_softmax_ce(self.handle, mb_id, logits.data_ptr(), labels.data_ptr(), dlogits.data_ptr(),
                                loss.data_ptr())
        return loss, dlogits

    def backward(self, mb_id: int, dy: torch.Tensor, dx: Optional[torch.Tensor] = None):
        rows = self.mb * self.n
        assert dy.shape[0] == rows and dy.numel() == rows * self.out_elems and dy.is_contiguous()
        assert dy.dtype == self.tdtype
        if self.needs_dx and dx is None:
            dx = torch.empty(rows, self.in_elems, dtype=self.tdtype, device=self.device)
        if dx is not None:
            assert dx.numel() == rows * self.in_elems and dx.is_contiguous() and dx.dtype == self.tdtype
        delta = B.stage_backward(self.handle, mb_id, dy.data_ptr(), dx.data_ptr() if dx is not None else 0)
        return dx, delta

    def blend_update(self, mb_done: int, mb_next: int = B.TP_NONE) -> int:
        return B.stage_blend_update(self.handle, mb_done, mb_next)

    def blend_update_noalloc(self, mb_done: int, mb_next: int = B.TP_NONE) -> int:
        return B.stage_blend_update_noalloc(self.handle, mb_done, mb_next)

    def query(self):
        return B.stage_query(self.handle)

    def export(self, version: int) -> torch.Tensor:
        out = torch.empty(self.P, dtype=torch.float32, device=self.device)
        B.stage_export_params(self.handle, version, out.data_ptr())
        return out

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize(self.device)
            B.stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class GpuPipeline:
    """K stages on one GPU driven through the library's own nF1B event list."""

    def __init__(self, workload, stage_params: List[List[np.ndarray]], *, policy: str, device="cuda:0",
                 fuse_next_blend: bool = True):
        self.w = workload
        self.K = workload.K
        self.fuse = fuse_next_blend
        self.stages = [GpuStage([layer_tuple(l) for l in workload.stages[s]], stage_params[s],
                                dtype=workload.dtype, mb=workload.mb, n=workload.n, stage_index=s, num_stages=self.K,
                                policy=policy, lam=workload.lam, lr=workload.lr, momentum=workload.momentum,
                                device=device) for s in range(self.K)]
        self.device = torch.device(device)

    def run(self, num_mb: int, get_input: Callable[[int], torch.Tensor], get_labels: Callable[[int], torch.Tensor],
            on_event=None):
        w = self.w
        events = B.tp_schedule_events(self.K, num_mb)
        # per stage: mini-batches in backward order, to name the next backward for the fused update
        acts: Dict[tuple, torch.Tensor] = {}
        grads: Dict[tuple, torch.Tensor] = {}
        losses: Dict[int, torch.Tensor] = {}
        rows = w.n * w.mb
        for (t, kind, s, j) in events:
            st = self.stages[s]
            info = {}
            if kind == "F":
                x = get_input(j) if s == 0 else acts.pop((s - 1, j))
                y = torch.empty(rows, st.out_elems, dtype=st.tdtype, device=self.device)
                for ub in range(w.n):
                    _, v = st.forward(j, ub, x[ub * w.mb:(ub + 1) * w.mb], y[ub * w.mb:(ub + 1) * w.mb])
                acts[(s, j)] = y
                info.update(y=y, v_f=v)
            else:
                if s == self.K - 1:
                    logits = acts.pop((s, j))
                    loss, dy = st.loss(j, logits, get_labels(j))
                    losses[j] = loss
                    info["loss"] = loss
                else:
                    dy = grads.pop((s + 1, j))
                info["dy"] = dy
                info["latest_before"] = st.query().latest_version
                dx, delta = st.backward(j, dy)
                if s > 0:
                    grads[(s, j)] = dx
                nxt = j + 1 if (self.fuse and j + 1 < num_mb) else B.TP_NONE
                if nxt != B.TP_NONE:
                    q = st.query()
                    known = [q.in_flight_mb[i] for i in range(q.num_in_flight)]
                    if nxt not in known:
                        nxt = B.TP_NONE
                info.update(dx=dx, delta=delta)
                if on_event is not None:
                    on_event("pre_update", (t, kind, s, j), self, info)
                info["new_version"] = st.blend_update(j, nxt)
            if on_event is not None:
                on_event("done", (t, kind, s, j), self, info)
        return events, losses

    def run_microbatches(self, num_mb: int, get_input, get_labels, *, mid_pass_updates: bool = False, on_event=None):
        """The micro-batch-granular clock of the library (tp_schedule_microbatch_events).  Under TP_TIMEPREST the
        versions every stage holds when a pass starts are read off the stages (stage_query), pinned (stash_push),
        named in stage_forward_on / stage_backward_on and dropped (stash_evict) as the pass leaves each stage."""
        w = self.w
        n, mb, K = w.n, w.mb, self.K
        rows = n * mb
        timeprest = self.stages[0].desc.policy == B.TP_TIMEPREST
        events = B.tp_schedule_microbatch_events(K, num_mb, n, mid_pass_updates)
        outs: Dict[tuple, torch.Tensor] = {}
        grads: Dict[tuple, torch.Tensor] = {}
        inputs: Dict[int, torch.Tensor] = {}
        fwd_v: Dict[int, list] = {}
        bwd_v: Dict[int, list] = {}
        losses: Dict[int, torch.Tensor] = {}
        for (t, kind, s, j, ub) in events:
            st = self.stages[s]
            info = {}
            if kind == "F":
                if timeprest and s == 0 and ub == 0:
                    fwd_v[j] = [int(r.query().latest_version) for r in self.stages]
                    for r, v in zip(self.stages, fwd_v[j]):
                        B.stash_push(r.handle, v)
                if s == 0 and j not in inputs:
                    inputs[j] = get_input(j)
                x = (inputs[j] if s == 0 else outs[(s - 1, j)])[ub * mb:(ub + 1) * mb]
                if (s, j) not in outs:
                    outs[(s, j)] = torch.empty(rows, st.out_elems, dtype=st.tdtype, device=self.device)
                y = outs[(s, j)][ub * mb:(ub + 1) * mb]
                if timeprest:
                    st.forward_on(j, ub, fwd_v[j][s], x, y)
                    v = fwd_v[j][s]
                else:
                    _, v = st.forward(j, ub, x, y)
                info.update(y=y, version=v)
                if ub == n - 1:
                    if s == 0:
                        inputs.pop(j)
                    else:
                        outs.pop((s - 1, j))
                    if timeprest:
                        B.stash_evict(st.handle, fwd_v[j][s])
            else:
                if timeprest and s == K - 1:
                    bwd_v[j] = [int(r.query().latest_version) for r in self.stages]
                    for r, v in zip(self.stages, bwd_v[j]):
                        B.stash_push(r.handle, v)
                if s == K - 1:
                    loss, dy = st.loss(j, outs.pop((s, j)), get_labels(j))
                    losses[j] = loss
                    info["loss"] = loss
                else:
                    dy = grads.pop((s + 1, j))
                info["dy"] = dy
                if timeprest:
                    dx = st.backward_on(j, bwd_v[j][s], dy)
                    B.stash_evict(st.handle, bwd_v[j][s])
                    info["version"] = bwd_v[j][s]
                else:
                    dx, info["delta"] = st.backward(j, dy)
                if s > 0:
                    grads[(s, j)] = dx
                info["dx"] = dx
                if on_event is not None:
                    on_event("pre_update", (t, kind, s, j, ub), self, info)
                info["new_version"] = st.blend_update(j, B.TP_NONE)
            if on_event is not None:
                on_event("done", (t, kind, s, j, ub), self, info)
        return events, losses

    def close(self):
        for st in self.stages:
            st.close()
