"""Single-stage GPU parity driver shared by the GPU tests: one stage driven with synthetic inputs and upstream
gradients through forward, backward (with real staleness under the I-TiMePReSt blend) and update, every tensor the
stage produces OR KEEPS compared with the fp64 oracle on the same seeded inputs.

Floating point decides two things discretely on this path: which side of zero a ReLU input lies on and which
element of a pooling window is the largest.  Both sides take them on bf16-stored values (the oracle through its
storage hook), but their stored values differ by a rounding step here and there, so a decision can differ where a
pre-activation lies within rounding noise of zero or two window entries within rounding noise of each other.  This
driver MEASURES that: it reads every stored activation of the stage back (stage_saved_input_ptr), compares it with
the oracle's, counts the decisions that differ, and checks that each of them is one the noise can explain (the
oracle's value within a few bf16 steps of the threshold).  A mini-batch without a differing decision is held to the
normal tolerance on every tensor; one with a fraction e of differing decisions may move a gradient sum of
random-sign terms by about sqrt(e) of its size and is held to TOL + 4 sqrt(e) (never more than 0.25) on gradient
tensors only.  `fix_relu_masks` builds parameters with which no decision is near its threshold: such stages meet
the normal tolerance throughout, which is what pins the kernels that read a ReLU mask off a saved output."""
from __future__ import annotations

import numpy as np

from oracle import layers as OL
from oracle.stage import Stage
from parity_utils import TOL, oracle_flat_to_arena, rel_err, to_np
from synth_inputs import workloads as W

BF16_STEP = 2.0 ** -8                    # half the spacing of bfloat16 values relative to their size, at most


def _with_act(spec, act):
    return type(spec)(**{**spec.__dict__, "act": act})


def fix_relu_masks(specs, params, x, margin=4.0):
    """Parameters with which every ReLU of the stage has a fixed mask: for each layer with a ReLU, in order, the
    shift in front of it (a dense / convolution bias, the shift of a batch normalisation, for a residual add the
    shift of the normalisation feeding it) is set so that its pre-activation sits `margin` standard deviations
    above zero in even channels and below zero in odd ones (4: a normalised value lies beyond it 6e-5 of the time,
    and within rounding noise of it one time in a million; a larger shift only adds a constant part to the activations
    that the next normalisation removes again, at the price of rounding noise relative to what is left).  Uses the pure fp64 oracle on the sample input x only."""
    params = [np.array(p, dtype=np.float64) for p in params]
    pidx, nxt = [], 0
    for spec in specs:
        if spec.param_shapes():
            pidx.append(nxt)
            nxt += 2
        else:
            pidx.append(None)
    for li, spec in enumerate(specs):
        if getattr(spec, "act", "none") != "relu":
            continue
        st = Stage(specs, params, policy="latest", lam=0.1, lr=0.0, momentum=0.0, n=1)
        st.forward(0, 0, x)
        saved = st.inflight[0]["saved"][0][li]
        if spec.kind in ("dense", "conv"):
            z, shift = saved[1], pidx[li] + 1
        elif spec.kind == "bn":
            z, shift = saved[2], pidx[li] + 1
        else:                                                       # residual add: the normalisation right before it
            assert spec.kind == "res" and specs[li - 1].kind == "bn" and specs[li - 1].act == "none"
            z, shift = saved[1], pidx[li - 1] + 1
        zc = z.reshape(-1, z.shape[-1])
        sign = np.where(np.arange(zc.shape[1]) % 2 == 0, 1.0, -1.0)
        params[shift] = W.round_f32(params[shift] - zc.mean(0) + sign * margin * zc.std(0).mean())
    return params


def run_stage(specs, w_name, dtype, mb, n, policy="convex", minibatches=3, depth=2, needs_dx=True, lr=None,
              lam=0.4, params=None, mean_loss_dy=False, fixed_masks=False, pure_oracle=False, stage_index=0,
              check_saved=True, storage_floor=False, forward_stream=False, progress=None):
    """Steady schedule of a stage of pipeline depth `depth`: forwards run `depth` mini-batches ahead.

    The fp32 runs take large steps (lr 0.05): at tolerance 1e-4 any mix-up of weight versions in the
    blend shows.  The bf16 runs take small ones (lr 0.002): with unit-size synthetic upstream gradients a
    large step changes the weights by O(1) per update and the ~1 % bf16 noise of one gradient would
    compound through the following mini-batches instead of testing the kernels.  mean_loss_dy scales the
    upstream gradient like that of a loss averaged over the mini-batch (1 / (n mb) per sample): the scale at
    which the workloads' own lr 0.01 is a training step.

    storage_floor (stages without ReLU, or with ReLUs whose masks are fixed, so that the oracle takes the same ReLU
    decisions in both of its modes; a max pooling may be there -- the few windows whose routing the storage precision
    changes are part of what it does to the result; meant for stacks of dozens of layers and for gradients that are
    sums of terms which nearly cancel, such as the shift in front of a dense layer followed by a batch
    normalisation): the plain fp64 oracle runs beside the
    bf16-storing one, and a tensor's limit is the larger of the normal tolerance and the distance between the two
    ORACLES on that tensor (times sqrt 2) -- what storing every activation in bf16 does to the exact result, by the
    oracle's own account.  The GPU's bf16 execution then has to sit as close to the bf16-storing oracle as two
    independent bf16 executions of the exact computation sit to each other; on stacks where that distance is below
    the tolerance nothing changes.

    forward_stream: the stage gets a second stream for the forward passes of odd micro-batches; their results are
    read after stage_forward_join.

    progress: called with a short text after every forward, backward and update of a mini-batch (the tests that take
    a minute or more at full size report through it)."""
    if lr is None:
        lr = 0.05 if dtype == "f32" else 0.002
    import torch
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple

    specs = tuple(specs)
    w = W.Workload(name=w_name, dtype=dtype, stages=(specs,) + ((),) * (depth - 1), mb=mb, n=n, classes=2)
    if params is None:
        params = W.init_params(w, 0)
        # biases (and the scale / shift of normalisation layers) away from their initial 0 / 1, so that their
        # gradients and updates are exercised
        rng = np.random.default_rng(7)
        params = [p if p.ndim > 1 else W.round_f32(p + rng.standard_normal(p.shape) * 0.1) for p in params]
    if fixed_masks:
        params = fix_relu_masks(specs, params, W.stage_input(w, 0, 0)[:mb])
    bf16 = dtype == "bf16"
    # bf16 workloads: the oracle keeps its stored tensors in bf16 too (fp64 arithmetic), so that decisions on
    # stored values are taken in the same precision on both sides; pure_oracle (smooth stages only) compares with
    # the plain fp64 run instead
    smooth = not any(l.kind == "pool" or getattr(l, "act", "") == "relu" for l in specs)
    no_relu = not any(getattr(l, "act", "") == "relu" for l in specs)
    assert smooth or not pure_oracle
    assert no_relu or fixed_masks or not storage_floor
    ost = Stage(specs, params, policy=policy, lam=lam, lr=lr, momentum=0.9, n=n, first_stage=not needs_dx,
                storage=W.round_bf16 if (bf16 and not pure_oracle) else None)
    st = GpuStage([layer_tuple(l) for l in specs], params, dtype=dtype, mb=mb, n=n, stage_index=stage_index,
                  num_stages=stage_index + depth, policy=policy, lam=lam, lr=lr, momentum=0.9, needs_dx=needs_dx,
                  forward_stream=forward_stream)
    opure = Stage(specs, params, policy=policy, lam=lam, lr=lr, momentum=0.9, n=n, first_stage=not needs_dx) \
        if storage_floor else None
    tol = TOL[dtype]
    worst, failures = {}, []
    floors = {}                                    # tensor name -> distance between the two oracles (storage_floor)
    gtol_m = [tol]
    flipped = {}                                   # mini-batch -> sum over layers of the fraction of differing decisions
    L = len(specs)

    def note(k, e, limit=None):
        worst[k] = max(worst.get(k, 0.0), e)
        # two executions that each sit eps from the exact result are up to sqrt(2) eps apart when their roundings
        # are independent
        limit = max(tol if limit is None else limit, np.sqrt(2.0) * floors.get(k, 0.0))
        if not e <= limit:
            failures.append((k, e, limit))

    def floor_of(k, stored_ref, pure_ref):
        if opure is not None:
            floors[k] = rel_err(stored_ref, pure_ref)
            worst["oracle bf16 vs fp64 " + k] = max(worst.get("oracle bf16 vs fp64 " + k, 0.0), floors[k])

    def check_saved_and_decisions(j, y_gpu):
        """Every stored activation of mini-batch j against the oracle's, and the decisions taken on them."""
        frac = 0.0
        rec = ost.inflight[j]
        for ub in range(n):
            outs, saved = rec["outs"][ub], rec["saved"][ub]
            stored = {}                                              # layer -> its stored OUTPUT on the GPU
            for l in range(1, L):
                if specs[l].kind == "res" and specs[l].mark == "add":
                    continue                                         # may have been formed inside its producer's kernel
                stored[l - 1] = to_np(st.saved_input(j, ub, l))
            stored[L - 1] = to_np(y_gpu[ub * mb:(ub + 1) * mb])
            for l, got in sorted(stored.items()):
                ref = outs[l].reshape(mb, -1)
                if opure is not None:
                    floor_of(f"a[{l}]", ref, opure.inflight[j]["outs"][ub][l].reshape(mb, -1))
                note(f"a[{l}]", rel_err(got, ref))
                spec = specs[l]
                if getattr(spec, "act", "none") == "relu":           # which side of zero
                    diff = (got > 0) != (ref > 0)
                    if diff.any():
                        # the value on the side that is not zero, in units of the rounding noise of its channel: the
                        # typical difference between the two sides' values there, at least one bf16 step of the
                        # channel's typical PRE-activation (a value next to zero is the small remainder of terms of
                        # that size).  Typically a differing decision is a step or two from zero; a wrong mask or
                        # index would put most of them a hundred away
                        C = spec.out_shape()[-1]
                        sv = saved[l]
                        zpre = (sv[2] if spec.kind == "bn" else sv[1]).reshape(-1, C)
                        g2, r2 = got.reshape(-1, C), ref.reshape(-1, C)
                        noise = np.maximum(np.sqrt(np.mean((g2 - r2) ** 2, axis=0)),
                                           BF16_STEP * np.sqrt(np.mean(zpre ** 2, axis=0)) + 1e-30)
                        near = (np.maximum(np.abs(g2), np.abs(r2)) / noise)[diff.reshape(-1, C)]
                        if near.size >= 8:
                            note(f"relu[{l}] differing decisions: median distance from zero, in noise units", float(np.median(near)), limit=4.0)
                        note(f"relu[{l}] differing decisions: largest distance from zero, in noise units", float(near.max()), limit=64.0)
                    note(f"relu[{l}] differing", float(diff.mean()), limit=max(1e-2, 4.0 / diff.size))
                    frac += float(diff.mean())
            for l in range(1, L):                                    # which element of a window (a first-layer pool
                spec = specs[l]                                      # sees the same input on both sides)
                if spec.kind != "pool":
                    continue
                gin = to_np(st.saved_input(j, ub, l)).reshape((mb,) + tuple(spec.in_shape()))
                _, idx_gpu = OL.maxpool2_forward(gin)                # the routing the values stored on the GPU imply
                diff = idx_gpu != saved[l][1]
                if diff.any():
                    rin = outs[l - 1].reshape(gin.shape)
                    B_, H, Wd, C = rin.shape
                    win = rin.reshape(B_, H // 2, 2, Wd // 2, 2, C).transpose(0, 1, 3, 2, 4, 5).reshape(B_, H // 2, Wd // 2, 4, C)
                    top2 = np.sort(win, axis=3)[:, :, :, -2:, :]
                    # the gap between a differing window's two largest entries, in units of the typical difference
                    # between the two sides' values in that channel (at least one bf16 step of the larger entry)
                    noise = np.sqrt(np.mean((gin - rin).reshape(-1, C) ** 2, axis=0))
                    prev = specs[l - 1]
                    if prev.kind in ("dense", "conv", "bn"):         # a bf16 step of the typical pre-activation in front
                        zpre = saved[l - 1][2 if prev.kind == "bn" else 1].reshape(-1, C)
                        noise = np.maximum(noise, BF16_STEP * np.sqrt(np.mean(zpre ** 2, axis=0)))
                    floor = np.maximum(noise, BF16_STEP * np.abs(top2[:, :, :, 1, :])) + 1e-30
                    gap = ((top2[:, :, :, 1, :] - top2[:, :, :, 0, :]) / floor)[diff]
                    if gap.size >= 8:
                        note(f"pool[{l}] differing windows: median gap, in noise units", float(np.median(gap)), limit=4.0)
                    note(f"pool[{l}] differing windows: largest gap, in noise units", float(gap.max()), limit=64.0)
                note(f"pool[{l}] differing", float(diff.mean()), limit=max(0.1, 4.0 / diff.size))
                frac += float(diff.mean())
        flipped[j] = frac / n

    def forward(j):
        x = W.stage_input(w, 0, j)
        xt = torch.from_numpy(x.reshape(n * mb, -1)).cuda().to(st.tdtype)
        y = torch.empty(n * mb, st.out_elems, dtype=st.tdtype, device="cuda")
        ref, pref = [], []
        for ub in range(n):
            ref.append(ost.forward(j, ub, x[ub * mb:(ub + 1) * mb]))
            if opure is not None:
                pref.append(opure.forward(j, ub, x[ub * mb:(ub + 1) * mb]))
            _, v = st.forward(j, ub, xt[ub * mb:(ub + 1) * mb], y[ub * mb:(ub + 1) * mb])
            assert v == ost.inflight[j]["v_f"]
        if forward_stream:
            st.forward_join()
        if opure is not None:
            floor_of("y", np.concatenate(ref).reshape(n * mb, -1), np.concatenate(pref).reshape(n * mb, -1))
        ey = rel_err(to_np(y), np.concatenate(ref).reshape(n * mb, -1))
        note("y", ey)
        if check_saved:
            before = dict(worst)
            for k in [k for k in worst if k.startswith("a[")]:
                worst[k] = 0.0
            check_saved_and_decisions(j, y)
            acts = {k: v for k, v in worst.items() if k.startswith("a[")}
            kmax = max(acts, key=acts.get) if acts else None
            print(f"  forward {j}: y {ey:.1e}, largest stored-activation error {kmax} {acts.get(kmax, 0.0):.1e}, "
                  f"differing decisions {flipped[j]:.1e}", flush=True)
            for k, v in before.items():
                worst[k] = max(worst.get(k, 0.0), v)
        else:
            flipped[j] = 0.0 if smooth else 1.0

    progress = progress or (lambda msg: None)
    for j in range(depth):
        forward(j)
        progress(f"{w_name} forward {j}")
    for j in range(minibatches):
        dy = W.stage_upstream_grad(w, 0, j, mean_loss=mean_loss_dy)
        dx_ref = ost.backward(j, dy)
        if opure is not None:
            dx_pure = opure.backward(j, dy)
            if needs_dx:
                floor_of("dx", dx_ref, dx_pure)
            floor_of("g", ost.flat(ost.g), opure.flat(opure.g))
            for pi, (a, b) in enumerate(zip(ost.g, opure.g)):
                if np.linalg.norm(b) > 0:
                    floor_of(f"g[{pi}]", a, b)
        dx, delta = st.backward(j, torch.from_numpy(dy.reshape(n * mb, -1)).cuda().to(st.tdtype))
        assert delta == ost.trace[-1][4]
        progress(f"{w_name} backward {j}")
        # gradient tensors of a mini-batch in which a fraction e of the decisions differed: TOL + 4 sqrt(e)
        e = flipped.pop(j) if bf16 else 0.0
        gtol = min(0.25, tol + 4.0 * np.sqrt(e)) if e > 0 else tol
        gtol_m[0] = max(gtol_m[0], gtol)               # the momentum carries every earlier gradient
        print(f"  mini-batch {j}: delta {delta}, differing decisions {e:.1e}, gradient tolerance {gtol:.3f}",
              {k: f"{v:.1e}" for k, v in worst.items() if "[" not in k}, flush=True)
        if needs_dx:
            note("dx", rel_err(to_np(dx), dx_ref.reshape(n * mb, -1)), limit=gtol)
        note("g", rel_err(to_np(st.grad), oracle_flat_to_arena(st, ost.flat(ost.g))), limit=gtol)
        # per-tensor gradients.  A tensor whose true gradient is zero (a bias in front of a batch
        # normalisation: the mean subtraction removes it; what is left is the cancellation noise of a sum of
        # terms that add up to zero) has no scale of its own: such tensors are measured against the typical
        # gradient entry instead of their own (rounding-noise) norm.
        g_rms = float(np.sqrt(np.mean(np.concatenate([r.reshape(-1) for r in ost.g]) ** 2)))
        for pi, (got, ref) in enumerate(zip(st.unpack(to_np(st.grad)), ost.g)):
            floor = g_rms * np.sqrt(ref.size)
            if np.linalg.norm(ref) < 0.05 * floor:
                note(f"g[{pi}]", float(np.linalg.norm(got.reshape(-1) - ref.reshape(-1)) / floor), limit=gtol)
            else:
                note(f"g[{pi}]", rel_err(got, ref), limit=gtol)
        ost.update(j)
        if opure is not None:
            opure.update(j)
            for pi, (a, b) in enumerate(zip(ost.m, opure.m)):
                if np.linalg.norm(b) > 0:
                    floor_of(f"m[{pi}]", a, b)
        # with one mini-batch in flight the next one has not been forwarded yet: no look-ahead blend
        assert (st.blend_update(j, j + 1) if depth > 1 else st.blend_update(j)) == ost.latest
        m_rms = float(np.sqrt(np.mean(np.concatenate([r.reshape(-1) for r in ost.m]) ** 2)))
        for pi, (got, ref, mg, mr) in enumerate(zip(st.unpack(to_np(st.export(ost.latest))), ost.weights[ost.latest],
                                                    st.unpack(to_np(st.momentum)), ost.m)):
            note(f"W_new[{pi}]", rel_err(got, ref))
            floor = m_rms * np.sqrt(mr.size)
            if np.linalg.norm(mr) < 0.05 * floor:
                note(f"m[{pi}]", float(np.linalg.norm(mg.reshape(-1) - mr.reshape(-1)) / floor), limit=gtol_m[0])
            else:
                note(f"m[{pi}]", rel_err(mg, mr), limit=gtol_m[0])
        note("W_new", rel_err(to_np(st.export(ost.latest)), oracle_flat_to_arena(st, ost.flat(ost.weights[ost.latest]))))
        progress(f"{w_name} update {j}")
        forward(j + depth)
        progress(f"{w_name} forward {j + depth}")
    st.close()
    assert not failures, (failures, worst)
    return worst
