"""Pins for the oracle's stage and pipeline: zero-staleness identity, reduction to
sequential mini-batch SGD, finite-difference gradients, linearity of dx in the
backward weights, momentum closed form, stash invariants."""
import math

import numpy as np
import pytest

from oracle import layers as L
from oracle.pipeline import Pipeline
from oracle.schedule import closed_form
from oracle.significance import POLICIES, coefficients
from oracle.stage import Stage, StageError
from synth_inputs.workloads import Dense


def _tiny_specs(act="gelu"):
    return ((Dense(5, 7, act), Dense(7, 6, act)), (Dense(6, 3, "none"),))


def _tiny_params(specs, seed=0):
    rng = np.random.default_rng(seed)
    out = []
    for stage in specs:
        ps = []
        for l in stage:
            ps.append(rng.standard_normal((l.out_features, l.in_features)) * 0.5)
            ps.append(rng.standard_normal(l.out_features) * 0.1)
        out.append(ps)
    return out


def _data(j, rows=4, dim=5, classes=3):
    rng = np.random.default_rng(100 + j)
    return rng.standard_normal((rows, dim)), rng.integers(0, classes, rows)


# -- independent reference: plain sequential mini-batch SGD with momentum -----

def _sequential_sgd(specs, params, num_mb, lr, mu, rows):
    layers = [l for st in specs for l in st]
    P = [p.copy() for st in params for p in st]
    M = [np.zeros_like(p) for p in P]
    losses = []
    for j in range(num_mb):
        x, y = _data(j, rows)
        acts, zs, a = [], [], x
        for i, l in enumerate(layers):
            acts.append(a)
            z = a @ P[2 * i].T + P[2 * i + 1]
            zs.append(z)
            a = L.act_forward(z, l.act)
        loss, d = L.softmax_cross_entropy(a, y, rows)
        losses.append(loss)
        G = [None] * len(P)
        for i in reversed(range(len(layers))):
            dz = d * L.act_derivative(zs[i], layers[i].act)
            G[2 * i], G[2 * i + 1] = dz.T @ acts[i], dz.sum(0)
            d = dz @ P[2 * i]
        for i in range(len(P)):
            M[i] = mu * M[i] + G[i]
            P[i] = P[i] - lr * M[i]
    return P, losses


@pytest.mark.parametrize("policy", POLICIES)
def test_one_minibatch_in_flight_equals_sequential_sgd(policy):
    # With a single mini-batch in flight (flush after each) every policy is plain SGD.
    specs, rows, n = _tiny_specs(), 4, 2
    params = _tiny_params(specs)
    stages = [Stage(specs[s], params[s], policy=policy, lam=0.3, lr=0.05, momentum=0.9, n=n,
                    first_stage=(s == 0)) for s in range(2)]
    losses = []
    for j in range(5):
        x, y = _data(j, rows)
        half = rows // n
        outs = []
        for ub in range(n):
            h = stages[0].forward(j, ub, x[ub * half:(ub + 1) * half])
            outs.append(stages[1].forward(j, ub, h))
        loss, d = L.softmax_cross_entropy(np.concatenate(outs), y, rows)
        losses.append(loss)
        dx = stages[1].backward(j, d)
        stages[1].update(j)
        assert stages[0].backward(j, dx) is None
        stages[0].update(j)
    ref_P, ref_losses = _sequential_sgd(specs, params, 5, 0.05, 0.9, rows)
    got = [p for st in stages for p in st.weights[st.latest]]
    for a, b in zip(got, ref_P):
        assert np.allclose(a, b, rtol=1e-12, atol=1e-14)
    assert np.allclose(losses, ref_losses, rtol=1e-12)


@pytest.mark.parametrize("policy", POLICIES)
def test_single_stage_pipeline_is_sequential_sgd(policy):
    specs = (tuple(l for st in _tiny_specs("relu") for l in st),)
    params = [[p for st in _tiny_params(_tiny_specs("relu")) for p in st]]
    pipe = Pipeline(specs, params, policy=policy, lam=0.2, lr=0.05, momentum=0.9, n=2, mb=2)
    pipe.run(4, lambda j: _data(j)[0], lambda j: _data(j)[1])
    ref_P, ref_losses = _sequential_sgd(specs, params, 4, 0.05, 0.9, 4)
    for a, b in zip(pipe.stages[0].weights[4], ref_P):
        assert np.allclose(a, b, rtol=1e-12, atol=1e-14)
    assert np.allclose([pipe.losses[j] for j in range(4)], ref_losses, rtol=1e-12)


@pytest.mark.parametrize("act", ["gelu", "relu"])
def test_gradients_match_finite_differences(act):
    # delta = 0, so W_b = W_f and the backward is the exact gradient of the loss.
    specs = (tuple(l for st in _tiny_specs(act) for l in st),)
    params = [p for st in _tiny_params(_tiny_specs(act), seed=5) for p in st]
    x, y = _data(0)

    def loss_of(plist, xin):
        st = Stage(specs[0], plist, policy="eq1", lam=0.1, lr=0.0, momentum=0.0, n=2)
        out = np.concatenate([st.forward(0, ub, xin[ub * 2:(ub + 1) * 2]) for ub in range(2)])
        return L.softmax_cross_entropy(out, y, 4), st

    (loss, d), st = loss_of(params, x)
    dx = st.backward(0, d)
    h = 1e-6
    for pi, p in enumerate(params):
        for idx in np.ndindex(p.shape):
            hi = [q.copy() for q in params]
            lo = [q.copy() for q in params]
            hi[pi][idx] += h
            lo[pi][idx] -= h
            fd = (loss_of(hi, x)[0][0] - loss_of(lo, x)[0][0]) / (2 * h)
            assert abs(st.g[pi][idx] - fd) < 1e-7, (pi, idx)
    for idx in np.ndindex(x.shape):
        hi, lo = x.copy(), x.copy()
        hi[idx] += h
        lo[idx] -= h
        fd = (loss_of(params, hi)[0][0] - loss_of(params, lo)[0][0]) / (2 * h)
        assert abs(dx[idx] - fd) < 1e-7


def _run_stage_with_staleness(policy, lam, updates=2, seed=7):
    """One stage: forward of mini-batch 9 on version 0, then `updates` updates, then its backward."""
    specs = _tiny_specs()[0]
    params = _tiny_params(_tiny_specs(), seed)[0]
    st = Stage(specs, params, policy=policy, lam=lam, lr=0.1, momentum=0.5, n=2)
    x9 = _data(9)[0]
    for ub in range(2):
        st.forward(9, ub, x9[ub * 2:(ub + 1) * 2])
    rng = np.random.default_rng(seed)
    for j in range(updates):
        xj = _data(j)[0]
        for ub in range(2):
            st.forward(j, ub, xj[ub * 2:(ub + 1) * 2])
        st.backward(j, rng.standard_normal((4, 6)))
        st.update(j)
    dy = rng.standard_normal((4, 6))
    dx = st.backward(9, dy)
    return st, dx, dy


def test_zero_staleness_intermediate_is_latest_bit_exact():
    for policy in ("eq1", "convex", "stashed", "latest"):
        st, _, _ = _run_stage_with_staleness(policy, lam=0.7, updates=0)
        assert st.trace[-1] == ("B", 9, 0, 0, 0)
        for a, b in zip(st.last_W_b, st.weights[0]):
            assert np.array_equal(a, b)


def test_intermediate_weights_follow_the_coefficients():
    lam = 0.25
    for policy in ("eq1", "convex", "stashed"):
        st, _, _ = _run_stage_with_staleness(policy, lam, updates=2)
        assert st.trace[-1] == ("B", 9, 0, 2, 2)
        W0 = _tiny_params(_tiny_specs(), 7)[0]
        latest = st.weights[2]
        fd = math.exp(-lam * 2)
        for wb, s, l in zip(st.last_W_b, W0, latest):
            if policy == "eq1":
                ref = (2 - 1 / fd) * s
            elif policy == "convex":
                ref = fd * s + (1 - fd) * l
            else:
                ref = s
            assert np.allclose(wb, ref, rtol=1e-14, atol=1e-15)
    st, _, _ = _run_stage_with_staleness("latest", lam, updates=2)
    for wb, l in zip(st.last_W_b, st.weights[2]):
        assert np.array_equal(wb, l)


def test_eq1_sign_change_at_ln2():
    st, _, _ = _run_stage_with_staleness("eq1", math.log(2), updates=1)
    for wb in st.last_W_b:
        assert np.max(np.abs(wb)) < 1e-15                   # coefficient 2 - 1/f = 0
    st, _, _ = _run_stage_with_staleness("eq1", math.log(2), updates=2)
    W0 = _tiny_params(_tiny_specs(), 7)[0]
    assert np.allclose(st.last_W_b[0], -2.0 * W0[0])        # 2 - e^{2 ln 2} = -2


def _one_layer_run(policy, lam, updates=2):
    """Single dense layer: its weight gradient never sees W_b, so the update history
    (and with it the latest weights) is the same under every policy."""
    specs = (Dense(5, 6, "gelu"),)
    rng = np.random.default_rng(21)
    st = Stage(specs, [rng.standard_normal((6, 5)), rng.standard_normal(6)], policy=policy, lam=lam,
               lr=0.1, momentum=0.5, n=2)
    x9 = _data(9)[0]
    for ub in range(2):
        st.forward(9, ub, x9[ub * 2:(ub + 1) * 2])
    for j in range(updates):
        xj = _data(j)[0]
        for ub in range(2):
            st.forward(j, ub, xj[ub * 2:(ub + 1) * 2])
        st.backward(j, rng.standard_normal((4, 6)))
        st.update(j)
    dx = st.backward(9, rng.standard_normal((4, 6)))
    return st, dx


def test_dx_is_linear_in_backward_weights_and_dw_ignores_them():
    # Saved activations come from the forward weights; W_b enters only through dx = dz . W_b.
    lam = 0.25
    runs = {p: _one_layer_run(p, lam) for p in POLICIES}
    a, b = coefficients("convex", 2, lam)
    assert np.allclose(runs["convex"][1], a * runs["stashed"][1] + b * runs["latest"][1], rtol=1e-12, atol=1e-14)
    a1, _ = coefficients("eq1", 2, lam)
    assert np.allclose(runs["eq1"][1], a1 * runs["stashed"][1], rtol=1e-12, atol=1e-14)
    assert not np.allclose(runs["latest"][1], runs["stashed"][1])
    for p in POLICIES:                                      # dW, db identical under every policy
        assert np.array_equal(runs[p][0].g[0], runs["stashed"][0].g[0])
        assert np.array_equal(runs[p][0].g[1], runs["stashed"][0].g[1])


def test_two_layer_stage_backward_weights_reach_the_first_layer():
    # Two layers, W_b = alpha * W_stale in both: dz of the first layer and dx scale with
    # alpha and alpha^2; the last layer's gradient does not see W_b at all.
    lam = 0.25
    st_s, dx_s, _ = _run_stage_with_staleness("stashed", lam, updates=2)
    st_e, dx_e, _ = _run_stage_with_staleness("eq1", lam, updates=2)
    a1, _ = coefficients("eq1", 2, lam)
    assert np.allclose(dx_e, a1 * a1 * dx_s, rtol=1e-12, atol=1e-14)
    assert np.allclose(st_e.g[0], a1 * st_s.g[0], rtol=1e-12, atol=1e-14)
    assert np.allclose(st_e.g[1], a1 * st_s.g[1], rtol=1e-12, atol=1e-14)
    assert np.allclose(st_e.g[2], st_s.g[2], rtol=1e-13)
    assert np.allclose(st_e.g[3], st_s.g[3], rtol=1e-13)


def test_momentum_closed_form():
    # constant gradient g: W_t = W_0 - lr * g * sum_{k=1..t} (1 - mu^k)/(1 - mu)
    specs = (Dense(3, 2, "none"),)
    W0, b0 = np.arange(6.0).reshape(2, 3), np.zeros(2)
    st = Stage(specs, [W0, b0], policy="latest", lam=0.1, lr=0.01, momentum=0.9, n=1)
    x = np.array([[1.0, -2.0, 0.5]])
    dy = np.array([[0.3, -0.7]])
    g = dy.T @ x
    for t in range(1, 8):
        st.forward(t, 0, x)
        st.backward(t, dy)
        st.update(t)
        s = sum((1 - 0.9 ** k) / (1 - 0.9) for k in range(1, t + 1))
        assert np.allclose(st.weights[t][0], W0 - 0.01 * g * s, rtol=1e-13)
        assert np.allclose(st.weights[t][1], b0 - 0.01 * dy[0] * s, rtol=1e-13)


@pytest.mark.parametrize("policy", POLICIES)
@pytest.mark.parametrize("K", [2, 4])
def test_stash_invariants_under_full_schedule(policy, K):
    specs = tuple((Dense(5, 5, "relu"),) for _ in range(K - 1)) + ((Dense(5, 3, "none"),),)
    rng = np.random.default_rng(11)
    params = [[rng.standard_normal((l.out_features, l.in_features)) * 0.4, np.zeros(l.out_features)]
              for st in specs for l in st]
    params = [params[s] for s in range(K)]
    pipe = Pipeline(specs, params, policy=policy, lam=0.1, lr=0.05, momentum=0.9, n=2, mb=2)
    num = 10
    seen = []

    def check(ev, p, info):
        st = p.stages[ev.s]
        lag = K - 1 - ev.s
        live = st.live_versions()
        if policy == "latest":
            assert live == [st.latest]                      # V keeps no stale version
        else:
            assert len(live) <= K - ev.s
            assert all(st.latest - lag <= v <= st.latest for v in live)
        assert all(c >= 0 for c in st.refcnt.values())
        if ev.kind == "B":
            _, mb, v_f, v_now, delta = info["trace"]
            exp = closed_form(K, ev.s, ev.j)
            if policy == "latest":
                assert (v_now, delta) == (exp[1], 0)
            else:
                assert (v_f, v_now, delta) == exp
        seen.append(ev)

    pipe.run(num, lambda j: _data(j)[0], lambda j: _data(j)[1], on_event=check)
    assert len(seen) == 2 * K * num
    for st in pipe.stages:
        assert st.live_versions() == [num] and st.refcnt == {num: 0} and not st.inflight
        # every version but the final one was evicted exactly once (reading an evicted
        # version raises, so none was read after eviction)
        assert sorted(st.evicted) == list(range(num))


def test_last_stage_follows_exact_sgd_given_its_inputs():
    # delta is always 0 at the last stage: whatever the policy, its weights follow plain
    # SGD on the activations it was fed.
    K = 3
    specs = ((Dense(5, 5, "gelu"),), (Dense(5, 5, "gelu"),), (Dense(5, 3, "none"),))
    rng = np.random.default_rng(12)
    params = [[rng.standard_normal((l.out_features, l.in_features)) * 0.4, np.zeros(l.out_features)]
              for st in specs for l in st]
    fed = {}

    for policy in ("latest", "eq1", "convex"):
        pipe = Pipeline(specs, [list(map(np.copy, p)) for p in params], policy=policy, lam=0.5,
                        lr=0.05, momentum=0.9, n=2, mb=2)
        W, b = params[2][0].copy(), params[2][1].copy()
        mW, mb_ = np.zeros_like(W), np.zeros_like(b)
        inputs = {}

        def hook(ev, p, info):
            nonlocal W, b, mW, mb_
            if ev.s == 1 and ev.kind == "F":
                inputs[ev.j] = info["y"]
            if ev.s == 2 and ev.kind == "B":
                xin = inputs[ev.j]
                _, d = L.softmax_cross_entropy(xin @ W.T + b, _data(ev.j)[1], 4)
                mW = 0.9 * mW + d.T @ xin
                mb_ = 0.9 * mb_ + d.sum(0)
                W, b = W - 0.05 * mW, b - 0.05 * mb_
                assert np.allclose(info["W_new"], np.concatenate([W.ravel(), b]), rtol=1e-12, atol=1e-14)

        pipe.run(6, lambda j: _data(j)[0], lambda j: _data(j)[1], on_event=hook)


def test_error_paths():
    specs = (Dense(3, 2, "none"),)
    st = Stage(specs, [np.zeros((2, 3)), np.zeros(2)], policy="eq1", lam=0.1, lr=0.1, momentum=0.0, n=2)
    with pytest.raises(StageError):
        st.forward(0, 1, np.zeros((1, 3)))                  # out of order
    st.forward(0, 0, np.zeros((1, 3)))
    with pytest.raises(StageError):
        st.backward(0, np.zeros((2, 2)))                    # not all micro-batches seen
    with pytest.raises(StageError):
        st.update(0)                                        # no gradient yet


# ---- TiMePReSt (pass-consistent versions) and the micro-batch clock --------------------------------------------

def _one_layer_pipeline(policy, K=4, n=4, seed=3):
    specs = tuple((Dense(5, 5, "gelu"),) for _ in range(K - 1)) + ((Dense(5, 3, "none"),),)
    rng = np.random.default_rng(seed)
    params = [[rng.standard_normal((l.out_features, l.in_features)) * 0.4, rng.standard_normal(l.out_features) * 0.1]
              for st in specs for l in st]
    return specs, Pipeline(specs, [params[s] for s in range(K)], policy=policy, lam=0.3, lr=0.05, momentum=0.9, n=n, mb=2)


def _mb_data(j, rows=8):
    rng = np.random.default_rng(50 + j)
    return rng.standard_normal((rows, 5)), rng.integers(0, 3, rows)


def test_timeprest_reads_the_versions_its_passes_started_on():
    # every forward and backward event re-derived by hand from copies of the weight versions kept on the side:
    # y = act(x W_f^T + b_f) on the forward pass's version, dx = (dy . act'(z)) W_b on the backward pass's version,
    # dW from the saved forward activations, the update applied to the latest weights
    from oracle.pipeline import run_microbatches
    K, n = 4, 4
    specs, pipe = _one_layer_pipeline("timeprest", K, n)
    history = [{0: [p.copy() for p in st.weights[0]]} for st in pipe.stages]
    xs, zs = {}, {}
    used = {"f_stale": 0, "b_stale": 0, "differ": 0}

    def on_event(ev, p, info):
        st, act = p.stages[ev.s], specs[ev.s][0].act
        if ev.kind == "F":
            v = info["version"]
            Wf, bf = history[ev.s][v]
            x = (_mb_data(ev.j)[0] if ev.s == 0 else xs[(ev.s - 1, ev.j, ev.ub)][1])
            x = x[ev.ub * 2:(ev.ub + 1) * 2] if ev.s == 0 else x
            z = x @ Wf.T + bf
            assert np.allclose(info["y"], L.act_forward(z, act), rtol=0, atol=1e-13)
            xs[(ev.s, ev.j, ev.ub)] = (x, info["y"])
            zs[(ev.s, ev.j, ev.ub)] = z
            used["f_stale"] += v < ev.version
        else:
            _, _, v_f, v_b, delta = info["trace"]
            assert delta == 0
            Wb = history[ev.s][v_b][0]
            dW = np.zeros_like(Wb)
            for ub in range(n):
                dz = info["dy"][ub * 2:(ub + 1) * 2] * L.act_derivative(zs[(ev.s, ev.j, ub)], act)
                dW += dz.T @ xs[(ev.s, ev.j, ub)][0]
                if ev.s > 0:
                    assert np.allclose(info["dx"][ub * 2:(ub + 1) * 2], dz @ Wb, rtol=0, atol=1e-13)
            assert np.allclose(info["g"][:dW.size].reshape(dW.shape), dW, rtol=0, atol=1e-13)
            used["b_stale"] += v_b < ev.version
            used["differ"] += v_f != v_b
            latest = st.latest
            history[ev.s][latest] = [w.copy() for w in st.weights[latest]]
            old = history[ev.s][latest - 1]
            assert np.allclose(st.weights[latest][0], old[0] - 0.05 * st.m[0], rtol=0, atol=1e-13)   # update on the latest

    run_microbatches(pipe, 9, lambda j: _mb_data(j)[0], lambda j: _mb_data(j)[1], on_event=on_event)
    assert used["f_stale"] > 0 and used["b_stale"] > 0 and used["differ"] > 0
    assert all(st.live_versions() == [9] and st.refcnt == {9: 0} for st in pipe.stages)


@pytest.mark.parametrize("policy", ["latest", "convex", "timeprest"])
def test_microbatch_clock_equals_minibatch_clock_without_mid_pass_updates(policy):
    # the same versions are read either way, so the same numbers come out -- except under TiMePReSt, whose passes
    # read older versions than the stage's latest
    from oracle.pipeline import run_microbatches
    _, coarse = _one_layer_pipeline("latest" if policy == "timeprest" else policy)
    coarse.run(8, lambda j: _mb_data(j)[0], lambda j: _mb_data(j)[1])
    _, fine = _one_layer_pipeline(policy)
    run_microbatches(fine, 8, lambda j: _mb_data(j)[0], lambda j: _mb_data(j)[1])
    same = all(np.array_equal(a, b) for sa, sb in zip(coarse.stages, fine.stages)
               for a, b in zip(sa.weights[sa.latest], sb.weights[sb.latest]))
    assert same == (policy != "timeprest")
    assert (coarse.losses == fine.losses) == (policy != "timeprest")


def test_timeprest_with_one_stage_or_frozen_weights_is_plain_sgd():
    from oracle.pipeline import run_microbatches
    for K in (1,):
        _, a = _one_layer_pipeline("timeprest", K=K)
        _, b = _one_layer_pipeline("latest", K=K)
        run_microbatches(a, 6, lambda j: _mb_data(j)[0], lambda j: _mb_data(j)[1])
        b.run(6, lambda j: _mb_data(j)[0], lambda j: _mb_data(j)[1])
        assert a.losses == b.losses


def test_mid_pass_updates_change_what_later_micro_batches_read():
    from oracle.pipeline import run_microbatches
    _, strict = _one_layer_pipeline("latest")
    _, loose = _one_layer_pipeline("latest")
    run_microbatches(strict, 8, lambda j: _mb_data(j)[0], lambda j: _mb_data(j)[1], mid_pass_updates=False)
    seen = []
    run_microbatches(loose, 8, lambda j: _mb_data(j)[0], lambda j: _mb_data(j)[1], mid_pass_updates=True,
                     on_event=lambda ev, p, info: seen.append((ev.s, ev.j, ev.ub, info["version"])) if ev.kind == "F" else None)
    per_pass = {}
    for s, j, ub, v in seen:
        per_pass.setdefault((s, j), []).append(v)
    assert any(len(set(v)) > 1 for v in per_pass.values())
    assert strict.losses != loose.losses
    with pytest.raises(StageError):                                     # a stashed forward version cannot change mid-pass
        _, bad = _one_layer_pipeline("convex")
        run_microbatches(bad, 8, lambda j: _mb_data(j)[0], lambda j: _mb_data(j)[1], mid_pass_updates=True)
