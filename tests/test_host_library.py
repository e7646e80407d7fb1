"""Host-side checks of the HIP library that need no GPU: it loads, exports every symbol the
header declares, and its integer bookkeeping (schedule, versions, ring slots, reference
counts, delta, coefficients, error codes) equals the oracle's bit for bit.  Stages are created
without device buffers, a mode in which the library launches nothing."""
import os
import re

import numpy as np
import pytest

from oracle.pipeline import Pipeline
from oracle.schedule import closed_form, simulate
from oracle.significance import POLICIES, coefficients
from paper_2509_23241_amd import binding as B
from synth_inputs.workloads import Dense

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "timeprest_stage.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*|int)\s+(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 15
    assert sorted(B.EXPORTS) == names
    for name in names:
        assert hasattr(B.lib, name), name


def test_struct_sizes_match_header_layout():
    import ctypes as C
    assert C.sizeof(B.tp_layer_desc) == 64
    assert C.sizeof(B.tp_stage_desc) == 10 * 4 + 3 * 8 + B.TP_MAX_LAYERS * 64
    assert B.TP_MAX_LAYERS == int(re.search(r"#define TP_MAX_LAYERS (\d+)", open(HEADER).read()).group(1))
    assert C.sizeof(B.tp_profile) == len(B.KERNEL_CLASSES) * 16 + 8
    assert C.sizeof(B.tp_event) == 24


@pytest.mark.parametrize("K,num", [(1, 5), (2, 8), (3, 7), (4, 12), (6, 9), (4, 2)])
def test_schedule_events_equal_oracle(K, num):
    ref = [(e.t, e.kind, e.s, e.j) for e in simulate(K, num)[0]]
    assert B.tp_schedule_events(K, num) == ref


def test_blend_coefficients_equal_oracle():
    for policy in POLICIES:
        for lam in (0.01, 0.1, float(np.log(2)), 1.0):
            for delta in range(0, 6):
                got = B.tp_blend_coefficients(policy, delta, lam)
                ref = coefficients(policy, delta, lam)
                assert np.allclose(got, ref, rtol=1e-15, atol=1e-16), (policy, lam, delta)
    assert B.tp_blend_coefficients("eq1", 0, 0.3) == (1.0, 0.0)
    assert B.tp_blend_coefficients("convex", 0, 0.3) == (1.0, 0.0)


def _dry_stage(K, s, policy, n=2, C=None, in_flight=None):
    depth = K - s
    d = B.make_desc([(5, 5, "relu")], dtype="f32", mb=2, n=n, stage_index=s, num_stages=K,
                    ring_capacity=C if C is not None else (1 if policy == "latest" else depth),
                    max_in_flight=in_flight if in_flight is not None else depth, policy=policy,
                    needs_dx=s > 0, lam=0.1, lr=0.01, momentum=0.9)
    return B.stage_init(d, None, 0)


def _live(q):
    return {q.slot_version[i]: q.slot_refcnt[i] for i in range(q.ring_capacity) if q.slot_occupied[i]}


@pytest.mark.parametrize("policy", POLICIES)
@pytest.mark.parametrize("K", [1, 2, 4])
def test_bookkeeping_equals_oracle_under_full_schedule(policy, K):
    n, num = 2, 11
    specs = tuple((Dense(5, 5, "relu"),) for _ in range(K - 1)) + ((Dense(5, 3, "none"),),)
    rng = np.random.default_rng(3)
    params = [[rng.standard_normal((l.out_features, l.in_features)) * 0.3, np.zeros(l.out_features)]
              for st in specs for l in st]
    pipe = Pipeline(specs, [params[s] for s in range(K)], policy=policy, lam=0.1, lr=0.01, momentum=0.9, n=n, mb=2)
    handles = [_dry_stage(K, s, policy, n=n) for s in range(K)]
    checked = []

    def on_event(ev, p, info):
        h, ost = handles[ev.s], p.stages[ev.s]
        if ev.kind == "F":
            for ub in range(n):
                v = B.stage_forward(h, ev.j, ub, 0, 0)
                assert v == info["v_f"]
        else:
            delta = B.stage_backward(h, ev.j, 0, 0)
            _, _, v_f, v_now, d_ref = info["trace"]
            assert delta == d_ref
            assert delta == (0 if policy == "latest" else closed_form(K, ev.s, ev.j)[2])
            new_v = B.stage_blend_update(h, ev.j, B.TP_NONE)
            assert new_v == ost.latest
        q = B.stage_query(h)
        assert q.latest_version == ost.latest
        live = _live(q)
        assert sorted(live) == ost.live_versions()
        for v, rc in live.items():
            assert rc == ost.refcnt[v]
            assert q.slot_version[v % q.ring_capacity] == v        # slot = version mod C
        assert sorted(q.in_flight_mb[i] for i in range(q.num_in_flight)) == sorted(ost.inflight)
        for i in range(q.num_in_flight):
            assert q.in_flight_vf[i] == ost.inflight[q.in_flight_mb[i]]["v_f"]
        checked.append(ev)

    pipe.run(num, lambda j: np.zeros((2 * n, 5)), lambda j: np.zeros(2 * n, dtype=int), on_event=on_event)
    assert len(checked) == 2 * K * num
    for h in handles:
        B.stage_destroy(h)


def test_fused_lookahead_marks_the_next_backward():
    K, s = 4, 1                                  # paper's example: machine 2 of 4
    h = _dry_stage(K, s, "eq1")
    for j in range(3):                           # K - s = 3 mini-batches enter
        for ub in range(2):
            B.stage_forward(h, j, ub, 0, 0)
    assert B.stage_backward(h, 0, 0, 0) == 0
    assert B.stage_blend_update(h, 0, 1) == 1    # builds W_b for mini-batch 1 on the fly
    assert B.stage_query(h).wb_ready_mb == 1
    for ub in range(2):
        B.stage_forward(h, 3, ub, 0, 0)          # mini-batch 4 (1-indexed) forwards on version 1
    assert B.stage_backward(h, 1, 0, 0) == 1
    assert B.stage_query(h).wb_ready_mb == B.TP_NONE
    B.stage_blend_update(h, 1, 2)
    assert B.stage_backward(h, 2, 0, 0) == 2
    B.stage_blend_update(h, 2, 3)
    q = B.stage_query(h)
    assert q.latest_version == 3 and _live(q) == {1: 1, 3: 0}
    assert B.stage_backward(h, 3, 0, 0) == 2     # W_2(1|3): stale 1, latest 3, delta 2
    B.stage_destroy(h)


def test_error_codes():
    h = _dry_stage(2, 0, "eq1")
    def code(fn, *a):
        with pytest.raises(B.StageLibError) as ei:
            fn(*a)
        return ei.value.code
    assert code(B.stage_forward, h, 0, 1, 0, 0) == B.TP_ESTATE            # first forward must be ub 0
    B.stage_forward(h, 0, 0, 0, 0)
    assert code(B.stage_forward, h, 0, 0, 0, 0) == B.TP_ESTATE            # repeated micro-batch
    assert code(B.stage_backward, h, 0, 0, 0) == B.TP_ESTATE              # not all forwards seen
    assert code(B.stage_backward, h, 7, 0, 0) == B.TP_ESTATE              # unknown mini-batch
    assert code(B.stage_blend_update, h, 0, B.TP_NONE) == B.TP_ESTATE     # no gradient pending
    B.stage_forward(h, 0, 1, 0, 0)
    B.stage_forward(h, 1, 0, 0, 0)
    B.stage_forward(h, 1, 1, 0, 0)
    assert code(B.stage_forward, h, 2, 0, 0, 0) == B.TP_ESTATE            # more than K-s in flight
    B.stage_backward(h, 0, 0, 0)
    assert code(B.stage_backward, h, 1, 0, 0) == B.TP_ESTATE              # previous gradient not applied
    assert code(B.stage_blend_update, h, 0, 5) == B.TP_ESTATE             # look-ahead for unknown mini-batch
    B.stage_blend_update(h, 0, 1)
    assert code(B.stash_push, h, 9) == B.TP_ENOVERSION
    assert code(B.stash_evict, h, 9) == B.TP_ENOVERSION
    assert code(B.stage_export_params, h, 9, 0) == B.TP_ENOVERSION
    assert B.stash_evict(h, 1) == B.TP_EBUSY                              # the latest version stays
    assert B.stash_push(h, 0) == 0                                        # version 0 sits in slot 0
    assert B.stash_evict(h, 0) == B.TP_EBUSY                              # still used by mini-batch 1
    assert "users" in B.tp_last_error()
    B.stage_destroy(h)
    # an update with the forward version still pinned and nowhere to keep it
    h = _dry_stage(2, 0, "stashed", C=1, in_flight=2)
    for j in range(2):
        for ub in range(2):
            B.stage_forward(h, j, ub, 0, 0)
    B.stage_backward(h, 0, 0, 0)
    assert code(B.stage_blend_update, h, 0, B.TP_NONE) == B.TP_EFULL
    B.stage_destroy(h)
    # a version held by a mini-batch in flight cannot be evicted from outside (Section "Memory Overhead": it stays
    # until that mini-batch has built its intermediate weights); forward -> evict -> update -> backward works
    h = _dry_stage(2, 0, "eq1", C=2)
    for ub in range(2):
        B.stage_forward(h, 0, ub, 0, 0)
    for ub in range(2):
        B.stage_forward(h, 1, ub, 0, 0)
    assert B.stash_evict(h, 0) == B.TP_EBUSY                              # two mini-batches forwarded on version 0
    assert _live(B.stage_query(h)) == {0: 2}                              # and the count is untouched
    B.stage_backward(h, 0, 0, 0)
    B.stage_blend_update(h, 0, B.TP_NONE)
    assert B.stash_evict(h, 0) == B.TP_EBUSY                              # still mini-batch 1's forward version
    assert "in flight" in B.tp_last_error()
    assert _live(B.stage_query(h)) == {0: 1, 1: 0}
    # an outside user on top of the stage's own: its pin can be dropped, the stage's cannot
    assert B.stash_push(h, 0) == 0
    assert _live(B.stage_query(h)) == {0: 2, 1: 0}
    assert B.stash_evict(h, 0) == B.TP_EBUSY and _live(B.stage_query(h)) == {0: 1, 1: 0}
    assert B.stash_evict(h, 0) == B.TP_EBUSY and _live(B.stage_query(h)) == {0: 1, 1: 0}
    assert B.stage_backward(h, 1, 0, 0) == 1                              # delta 1 on the stashed version 0
    assert _live(B.stage_query(h)) == {1: 0}                              # last user gone: evicted
    B.stage_destroy(h)
    # an outside pin alone keeps a version, and dropping it frees the slot
    h = _dry_stage(2, 0, "eq1", C=2)
    B.stash_push(h, 0)
    for ub in range(2):
        B.stage_forward(h, 0, ub, 0, 0)
    B.stage_backward(h, 0, 0, 0)
    B.stage_blend_update(h, 0, B.TP_NONE)
    assert _live(B.stage_query(h)) == {0: 1, 1: 0}
    assert B.stash_evict(h, 0) == B.TP_OK and _live(B.stage_query(h)) == {1: 0}
    B.stage_destroy(h)


def test_noalloc_update_bookkeeping_and_size_limit():
    # without device buffers the call is the bookkeeping of stage_blend_update, no kernel, no scratch lookup
    h = _dry_stage(2, 0, "convex")
    for j in range(2):
        for ub in range(2):
            B.stage_forward(h, j, ub, 0, 0)
    B.stage_backward(h, 0, 0, 0)
    assert B.stage_blend_update_noalloc(h, 0, 1) == 1
    q = B.stage_query(h)
    assert q.latest_version == 1 and q.wb_ready_mb == 1 and _live(q) == {0: 1, 1: 0}
    with pytest.raises(B.StageLibError) as ei:
        B.stage_blend_update_noalloc(h, 0, B.TP_NONE)                      # no gradient pending
    assert ei.value.code == B.TP_ESTATE
    B.stage_destroy(h)
    # a stage beyond the stated maximum is refused before anything else happens
    limit = int(re.search(r"#define TP_NOALLOC_MAX_PARAMS \(1ull << (\d+)\)", open(HEADER).read()).group(1))
    d = B.make_desc([(65536, 65536, "none")], dtype="f32", mb=1, n=1, stage_index=0, num_stages=1, ring_capacity=1,
                    max_in_flight=1, policy="latest", needs_dx=False, lam=0.1, lr=0.01, momentum=0.9)
    assert B.stage_workspace_query(d).param_count > (1 << limit)
    h = B.stage_init(d, None, 0)
    B.stage_forward(h, 0, 0, 0, 0)
    B.stage_backward(h, 0, 0, 0)
    with pytest.raises(B.StageLibError) as ei:
        B.stage_blend_update_noalloc(h, 0, B.TP_NONE)
    assert ei.value.code == B.TP_EINVAL and "at most" in str(ei.value)
    assert B.stage_blend_update(h, 0, B.TP_NONE) == 1                     # the workspace-based call has no such limit
    B.stage_destroy(h)


def test_invalid_descriptions():
    good = dict(dtype="f32", mb=2, n=2, stage_index=0, num_stages=2, ring_capacity=2, max_in_flight=2,
                policy="eq1", needs_dx=False, lam=0.1, lr=0.01, momentum=0.9)
    for bad in (dict(lam=0.0), dict(mb=0), dict(ring_capacity=0), dict(ring_capacity=17), dict(stage_index=2),
                dict(policy=9), dict(dtype=5), dict(max_in_flight=0)):
        d = B.make_desc([(4, 4, "relu")], **{**good, **bad})
        with pytest.raises(B.StageLibError) as ei:
            B.stage_workspace_query(d)
        assert ei.value.code == B.TP_EINVAL
    d = B.make_desc([(4, 8, "relu"), (4, 4, "none")], **good)             # layer shapes do not chain
    with pytest.raises(B.StageLibError):
        B.stage_workspace_query(d)
    d = B.make_desc([], **good)
    with pytest.raises(B.StageLibError):
        B.stage_workspace_query(d)


def test_transformer_layer_descriptions():
    good = dict(dtype="bf16", mb=2, n=2, stage_index=1, num_stages=4, ring_capacity=3, max_in_flight=3,
                policy="convex", needs_dx=True, lam=0.1, lr=0.01, momentum=0.9)
    D, T = 32, 8
    block = [("res", D, T, "begin"), ("ln", D, T), (D, 3 * D, "none", T), ("attn", D, 4, T), (D, D, "none", T),
             ("res", D, T, "add")]
    s = B.stage_workspace_query(B.make_desc(block, **good))
    # parameters: gamma/beta of the norm, then W/b of the two dense layers, each padded to 64 elements
    assert s.w_offset[1] == 0 and s.b_offset[1] == 64
    assert s.w_offset[2] == 128 and s.b_offset[2] == 128 + 3 * D * D
    assert s.param_count == 128 + 3 * D * D + 128 + D * D + 64
    bad_cases = [
        block[:4],                                                            # attention last, skip left open
        [("res", D, T, "begin"), ("ln", D, T)],                               # begin without add
        [("ln", D, T), ("res", D, T, "add")],                                 # add without begin
        [("res", D, T, "begin"), ("res", D, T, "begin"), ("res", D, T, "add"), ("res", D, T, "add")],   # nested
        [("res", D, T, "begin"), (D, 2 * D, "none", T), ("res", 2 * D, T, "add")],                     # shapes differ
        [(D, 3 * D, "none", T), ("attn", D, 5, T), (D, D, "none", T)],        # heads do not divide the width
        [(D, 3 * D, "none", T), ("attn", D, 4, T + 1), (D, D, "none", T)],    # token counts do not chain
        [(D, 3 * D, "none", T), ("attn", D, 4, T)],                           # attention as the last layer
    ]
    for layers in bad_cases:
        with pytest.raises(B.StageLibError) as ei:
            B.stage_workspace_query(B.make_desc(layers, **good))
        assert ei.value.code == B.TP_EINVAL, layers
    with pytest.raises(ValueError):
        B.make_desc([(4, 4, "none")] * (B.TP_MAX_LAYERS + 1), **good)


def test_projection_shortcut_descriptions():
    from paper_2509_23241_amd.runner import layer_tuple
    from synth_inputs import workloads as W
    good = dict(dtype="bf16", mb=2, n=2, stage_index=1, num_stages=4, ring_capacity=3, max_in_flight=3,
                policy="convex", needs_dx=True, lam=0.1, lr=0.01, momentum=0.9)
    block = [layer_tuple(l) for l in W.bottleneck_down_block(16, 8, 32, 4, 4)]
    s = B.stage_workspace_query(B.make_desc(block, **good))
    assert B.layer_in_elems(block[0]) == 16 * 16 and B.layer_out_elems(block[-1]) == 4 * 32
    # parameters: 1x1 (16 -> 8), bn 8, 3x3 stride 2 (8 -> 8), bn 8, 1x1 (8 -> 32), bn 32, projection 1x1 (16 -> 32), bn 32
    assert s.param_count == (128 + 64) + 128 + (576 + 64) + 128 + (256 + 64) + 128 + (512 + 64) + 128
    swap = block.index(("swap", 32, 4, 16, 16))
    bad_cases = [
        block[swap:],                                                        # swap without a begin
        block[:swap] + [("swap", 32, 4, 16, 4)] + block[swap + 1:],          # does not give back the remembered shape
        block[:swap + 1] + [("swap", 16, 16, 16, 16)] + block[swap + 1:],    # second swap before the add
        block[:-1] + [("res", 16, 16, "add")],                               # add with the begin's shape, not the kept one
        [("conv", 8, 8, 4, 4, "none", 3)],                                   # stride 3
        [("conv", 8, 8, 5, 4, "none", 2)],                                   # stride 2 on an odd height
        [("sub", 8, 4, 3)],                                                  # odd width
        [("sub", 4, 4, 4)],                                                  # bf16 pixels of 8 bytes
    ]
    for layers in bad_cases:
        with pytest.raises(B.StageLibError) as ei:
            B.stage_workspace_query(B.make_desc(layers, **good))
        assert ei.value.code == B.TP_EINVAL, layers
    # a stride-2 convolution quarters the sample: its output chains into a layer on the smaller grid only
    B.stage_workspace_query(B.make_desc([("conv", 8, 8, 4, 4, "none", 2), (8, 8, "none", 4)], **good))
    with pytest.raises(B.StageLibError):
        B.stage_workspace_query(B.make_desc([("conv", 8, 8, 4, 4, "none", 2), (8, 8, "none", 16)], **good))


def test_stem_and_head_descriptions():
    """Kernel sizes other than 3 and global average pooling: accepted geometries, parameter counts, chaining."""
    from paper_2509_23241_amd.runner import layer_tuple
    from synth_inputs import workloads as W
    good = dict(dtype="bf16", mb=2, n=2, stage_index=0, num_stages=4, ring_capacity=4, max_in_flight=4,
                policy="convex", needs_dx=False, lam=0.1, lr=0.01, momentum=0.9)
    w = W.resnet_stages(mb=2, n=2)
    for stage in range(4):
        layers = [layer_tuple(l) for l in w.stages[stage]]
        s = B.stage_workspace_query(B.make_desc(layers, **{**good, "stage_index": stage, "needs_dx": stage > 0}))
        padded = sum((int(np.prod(sh)) + 63) // 64 * 64 for l in w.stages[stage] for sh in l.param_shapes())
        assert s.param_count == padded
        assert B.layer_in_elems(layers[0]) == w.stage_in_dim(stage) and B.layer_out_elems(layers[-1]) == w.stage_out_dim(stage)
        assert [tuple(sh) for l in layers for sh in B.layer_param_shapes(l)] == \
            [tuple(sh) for l in w.stages[stage] for sh in l.param_shapes()]
    stem = layer_tuple(w.stages[0][0])
    assert stem == ("conv", 3, 64, 64, 64, "none", 2, 7)
    assert B.layer_out_elems(stem) == 32 * 32 * 64 and B.layer_param_shapes(stem)[0] == (64, 7, 7, 3)
    for k in (1, 3, 5, 7):
        B.stage_workspace_query(B.make_desc([("conv", 3, 8, 6, 4, "relu", 1, k)], **good))
    d = B.make_desc([("conv", 3, 8, 6, 4, "relu", 1, 7)], **good)
    d.layers[0].geom[4] = 1                                                  # pad that does not centre the kernel
    bad = [d, B.make_desc([("conv", 3, 8, 6, 4, "relu", 1, 4)], **good),     # even kernel
           B.make_desc([("conv", 3, 8, 6, 4, "relu", 1, 9)], **good),        # kernel larger than what is built
           B.make_desc([("avg", 8, 0)], **good),                             # no positions
           B.make_desc([("avg", 8, 4), (8 * 4, 4, "none")], **good)]         # the pooled sample has 8 values, not 32
    d2 = B.make_desc([("avg", 8, 4)], **good)
    d2.layers[0].act = B.ACT["relu"]                                         # pooling has no activation
    for desc in bad + [d2]:
        with pytest.raises(B.StageLibError) as ei:
            B.stage_workspace_query(desc)
        assert ei.value.code == B.TP_EINVAL
    B.stage_workspace_query(B.make_desc([("avg", 8, 4), (8, 4, "none")], **good))


def test_forward_streams_need_a_stage_that_launches():
    h = _dry_stage(2, 0, "convex")
    with pytest.raises(B.StageLibError) as ei:
        B.stage_set_forward_streams(h, [1234])
    assert ei.value.code == B.TP_ESTATE
    B.stage_forward_join(h)                                   # nothing to wait for: accepted
    B.stage_destroy(h)


def test_workspace_layout():
    d = B.make_desc([(256, 512, "relu"), (512, 10, "none")], dtype="bf16", mb=32, n=4, stage_index=0, num_stages=2,
                    ring_capacity=2, max_in_flight=2, policy="convex", needs_dx=False, lam=0.1, lr=0.01, momentum=0.9)
    s = B.stage_workspace_query(d)
    assert s.w_offset[0] == 0 and s.b_offset[0] == 256 * 512
    assert s.w_offset[1] == 256 * 512 + 512 and s.b_offset[1] == s.w_offset[1] + 5120
    assert s.param_count == s.b_offset[1] + 64 and s.param_count % 64 == 0
    assert s.ring_bytes == 2 * s.param_count * 4 and s.wfwd_bytes == 2 * s.param_count
    assert s.momentum_bytes == s.grad_bytes == 4 * s.param_count


def test_memory_per_stage_and_policy_follows_the_papers_ordering():
    # Section "Memory Overhead": V-TiMePReSt holds the least (one weight version, no intermediate weights), the
    # stashing policies hold K - s versions at stage s; momentum, gradient and saved activations do not depend on
    # the policy.  Sizes are the library's own workspace figures.
    from paper_2509_23241_amd import footprint as F
    from synth_inputs import workloads as W
    w = W.mlp_wide()
    for s in range(w.K):
        v = F.stage_bytes(w, s, "latest")
        P4 = 4 * v["params"]
        assert v["ring_bytes"] == P4 and v["wbwd_bytes"] == 0 and v["wfwd_bytes"] == P4 // 2
        for policy in ("eq1", "convex", "stashed"):
            i = F.stage_bytes(w, s, policy)
            assert i["ring_bytes"] == (w.K - s) * P4 and i["wbwd_bytes"] == P4 // 2
            for k in ("momentum_bytes", "grad_bytes", "act_bytes", "scratch_bytes", "wfwd_bytes", "params"):
                assert i[k] == v[k], k
            assert i["total"] - v["total"] == (w.K - s - 1) * P4 + P4 // 2
            assert i["total"] > v["total"]
        assert v["act_bytes"] % (w.K - s) == 0                           # K - s mini-batches in flight
        # the parent method sits between the two at the first stages: it keeps the versions passes under way read
        t = F.stage_bytes(w, s, "timeprest")
        assert 1 <= t["versions"] <= w.K and v["total"] < t["total"]
        if s == 0:
            assert t["versions"] < w.K - s and t["total"] < F.stage_bytes(w, s, "convex")["total"]
    assert "| MLP width 4096, stage 0 | V-TiMePReSt |" in F.table(F.default_rows())
    # a V-TiMePReSt stage can be created without a buffer for intermediate weights, a stashing one cannot
    d = B.make_desc([(8, 8, "relu")], dtype="f32", mb=2, n=2, stage_index=0, num_stages=2, ring_capacity=1,
                    max_in_flight=2, policy="latest", needs_dx=False, lam=0.1, lr=0.01, momentum=0.9)
    assert B.stage_workspace_query(d).wbwd_bytes == 0


@pytest.mark.parametrize("mid", [False, True])
@pytest.mark.parametrize("K,num,n", [(1, 4, 3), (2, 7, 4), (4, 9, 2), (4, 9, 4), (6, 8, 8), (3, 2, 1)])
def test_microbatch_schedule_events_equal_oracle(K, num, n, mid):
    from oracle.schedule import simulate_microbatches
    ref = [(e.t, e.kind, e.s, e.j, e.ub) for e in simulate_microbatches(K, num, n, mid)]
    assert B.tp_schedule_microbatch_events(K, num, n, mid) == ref


@pytest.mark.parametrize("policy,mid", [("timeprest", False), ("latest", True), ("latest", False), ("convex", False)])
def test_bookkeeping_equals_oracle_under_microbatch_schedule(policy, mid):
    # K dry stages driven through the micro-batch clock next to the oracle pipeline: versions read, live versions,
    # reference counts.  TiMePReSt: pins taken when a pass starts, versions named per call.
    from oracle.pipeline import run_microbatches
    K, n, num = 4, 4, 9
    specs = tuple((Dense(5, 5, "relu"),) for _ in range(K - 1)) + ((Dense(5, 3, "none"),),)
    rng = np.random.default_rng(3)
    params = [[rng.standard_normal((l.out_features, l.in_features)) * 0.3, np.zeros(l.out_features)]
              for st in specs for l in st]
    pipe = Pipeline(specs, [params[s] for s in range(K)], policy=policy, lam=0.1, lr=0.01, momentum=0.9, n=n, mb=2)
    C = {"latest": 1, "timeprest": K}
    handles = [_dry_stage(K, s, policy, n=n, C=C.get(policy)) for s in range(K)]
    fwd_v, bwd_v = {}, {}
    seen_split = []

    def on_event(ev, p, info):
        h, ost = handles[ev.s], p.stages[ev.s]
        if ev.kind == "F":
            if policy == "timeprest":
                if ev.s == 0 and ev.ub == 0:
                    fwd_v[ev.j] = [B.stage_query(r).latest_version for r in handles]
                    for r, v in zip(handles, fwd_v[ev.j]):
                        B.stash_push(r, v)
                B.stage_forward_on(h, ev.j, ev.ub, fwd_v[ev.j][ev.s], 0, 0)
                assert fwd_v[ev.j][ev.s] == info["version"]
                if ev.ub == n - 1:
                    B.stash_evict(h, fwd_v[ev.j][ev.s])
            else:
                assert B.stage_forward(h, ev.j, ev.ub, 0, 0) == info["version"] == ev.version
                if ev.ub > 0 and info["version"] != ost.inflight[ev.j]["versions"][0]:
                    seen_split.append((ev.s, ev.j))
        else:
            if policy == "timeprest":
                if ev.s == K - 1:
                    bwd_v[ev.j] = [B.stage_query(r).latest_version for r in handles]
                    for r, v in zip(handles, bwd_v[ev.j]):
                        B.stash_push(r, v)
                B.stage_backward_on(h, ev.j, bwd_v[ev.j][ev.s], 0, 0)
                assert bwd_v[ev.j][ev.s] == info["trace"][3]
                B.stash_evict(h, bwd_v[ev.j][ev.s])
            else:
                assert B.stage_backward(h, ev.j, 0, 0) == info["trace"][4]
            assert B.stage_blend_update(h, ev.j, B.TP_NONE) == ost.latest
        # the pins of a pass are taken at all stages at once: compare every stage after every event
        for r, ost_r in zip(handles, p.stages):
            q = B.stage_query(r)
            live = _live(q)
            assert q.latest_version == ost_r.latest
            assert sorted(live) == ost_r.live_versions(), (ev, live, ost_r.live_versions())
            assert all(live[v] == ost_r.refcnt[v] for v in live)

    events, (fv, bv) = run_microbatches(pipe, num, lambda j: np.zeros((2 * n, 5)), lambda j: np.zeros(2 * n, dtype=int),
                                        mid_pass_updates=mid, on_event=on_event)
    if policy == "timeprest":
        assert {j: list(v) for j, v in fv.items()} == fwd_v and {j: list(v) for j, v in bv.items()} == bwd_v
        for h in handles:                                              # every pin was dropped again
            assert list(_live(B.stage_query(h)).values()) == [0]
    assert bool(seen_split) == (policy == "latest" and mid)            # an update in the middle of a pass: V only
    for h in handles:
        B.stage_destroy(h)


def test_pass_versions_are_refused_outside_timeprest_and_when_not_held():
    h = _dry_stage(2, 0, "convex")
    with pytest.raises(B.StageLibError) as ei:
        B.stage_forward_on(h, 0, 0, 0, 0, 0)
    assert ei.value.code == B.TP_EINVAL
    B.stage_destroy(h)
    h = _dry_stage(2, 0, "timeprest", C=2)
    with pytest.raises(B.StageLibError) as ei:
        B.stage_forward_on(h, 0, 0, 5, 0, 0)
    assert ei.value.code == B.TP_ENOVERSION
    for ub in range(2):
        B.stage_forward_on(h, 0, ub, 0, 0, 0)
    with pytest.raises(B.StageLibError) as ei:
        B.stage_backward_on(h, 0, 3, 0, 0)
    assert ei.value.code == B.TP_ENOVERSION
    B.stage_backward_on(h, 0, 0, 0, 0)
    assert B.stage_blend_update(h, 0, B.TP_NONE) == 1
    assert _live(B.stage_query(h)) == {1: 0}                           # nothing pinned: the old version is gone
    assert B.tp_blend_coefficients("timeprest", 3, 0.5) == (1.0, 0.0)
    B.stage_destroy(h)
