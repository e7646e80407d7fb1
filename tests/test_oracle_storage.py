"""Pins of the oracle's storage hook (`Stage(storage=...)`): the mode the bf16 workloads are compared in.

The workloads keep activations in bfloat16 and master weights in fp32 ("bf16 activations with fp32 master
weights").  In that mode the oracle rounds, with its arithmetic still fp64, exactly the tensors such a workload
stores in its activation type: the compute copy of every weight MATRIX, every layer's output, and every gradient
with respect to an activation that is handed from one layer to the next.  Biases, normalisation scale/shift,
parameter gradients, momentum and master weights are never rounded.  These tests pin (a) that the hook changes
nothing but those roundings, (b) which tensors it sees, (c) that the rounded run stays within a stated distance
of the pure fp64 run on smooth nets, (d) that the two decisions taken on stored values (ReLU side, pooling
maximum) are taken on the rounded ones."""
import numpy as np
import pytest

from oracle.stage import Stage
from synth_inputs import round_bf16, workloads as W


def _cases():
    dense = (W.Dense(6, 9, "gelu"), W.Dense(9, 7, "relu"), W.Dense(7, 5, "none"))
    conv = (W.Conv2d(3, 4, 4, 6, "gelu"), W.MaxPool2(4, 4, 6), W.Conv2d(4, 5, 2, 3, "relu", stride=1))
    bneck = W.bottleneck_down_block(4, 2, 8, 4, 4) + W.bottleneck_block(8, 2, 2, 2)
    tfm = W.transformer_block(8, 2, 12, 3)
    return {"dense": dense, "conv": conv, "bottleneck": bneck, "transformer": tfm}


def _params(specs, seed):
    w = W.Workload(name="storage_pin", dtype="f32", stages=(tuple(specs),), mb=2, n=2, classes=2)
    rng = np.random.default_rng(seed)
    return [p + 0.1 * rng.standard_normal(p.shape) for p in W.init_params(w, 0)]


def _run(specs, params, storage, policy="convex", lr=0.05):
    """Two mini-batches forward, then backward 0 (delta 0), update, backward 1 (delta 1), update."""
    st = Stage(specs, params, policy=policy, lam=0.4, lr=lr, momentum=0.9, n=2, storage=storage)
    rng = np.random.default_rng(11)
    in_shape = tuple(specs[0].in_shape())
    out = {}
    for j in range(2):
        x = rng.standard_normal((4,) + in_shape)
        out[f"y{j}"] = np.concatenate([st.forward(j, ub, x[2 * ub:2 * ub + 2]).reshape(2, -1) for ub in range(2)])
    for j in range(2):
        dy = rng.standard_normal(out[f"y{j}"].shape) / np.sqrt(out[f"y{j}"].shape[1])
        out[f"dx{j}"] = st.backward(j, dy).reshape(4, -1)
        assert st.trace[-1][4] == j                                # delta 0, then 1
        out[f"g{j}"] = st.flat(st.g)
        st.update(j)
        out[f"W{j + 1}"] = st.flat(st.weights[st.latest])
    return out


@pytest.mark.parametrize("name", sorted(_cases()))
def test_identity_storage_is_the_pure_oracle_bit_for_bit(name):
    specs = _cases()[name]
    params = _params(specs, 1)
    a = _run(specs, params, None)
    b = _run(specs, params, lambda t: t)
    c = _run(specs, params, lambda t: np.array(t, copy=True))      # the hook's result is used, never the argument mutated
    for k in a:
        assert np.array_equal(a[k], b[k]), k
        assert np.array_equal(a[k], c[k]), k


def test_which_tensors_the_hook_sees():
    # distinct sizes everywhere, so a shape names a tensor: x [3 x 4], layer 0: 4 -> 5 (GELU), layer 1: 5 -> 6 (none)
    specs = (W.Dense(4, 5, "gelu"), W.Dense(5, 6, "none"))
    rng = np.random.default_rng(2)
    params = [rng.standard_normal(s) for l in specs for s in l.param_shapes()]
    seen = []

    def hook(t):
        seen.append(tuple(np.shape(t)))
        return t

    st = Stage(specs, params, policy="latest", lam=0.1, lr=0.1, momentum=0.0, n=1, storage=hook)
    st.forward(0, 0, rng.standard_normal((3, 4)))
    # forward: the two weight matrices (not the biases), then each layer's output
    assert seen == [(5, 4), (6, 5), (3, 5), (3, 6)]
    del seen[:]
    st.backward(0, rng.standard_normal((3, 6)))
    # backward: the backward copies of the weight matrices, the gradient entering each layer's product
    # (dz of layer 1, dz of layer 0), and the gradient handed to the previous stage
    assert seen == [(5, 4), (6, 5), (3, 6), (3, 5), (3, 4)]
    del seen[:]
    st.update(0)
    assert seen == []                                              # master weights, momentum, gradient: never


def test_what_is_never_rounded():
    # a hook that would wreck anything it touches: biases, parameter gradients of the last layer's bias,
    # momentum and the master weights come out the same as in the pure run when weights and activations
    # are such that the hook has nothing to change (all values already on the coarse grid)
    specs = (W.Dense(3, 2, "none"),)
    Wm = np.array([[1.0, -2.0, 0.5], [0.25, 4.0, -1.0]])
    b = np.array([0.1234567, -0.7654321])                          # not bf16 values
    x = np.array([[1.0, 2.0, -1.0], [0.5, -0.5, 2.0]])
    dy = np.array([[1.0, -1.0], [0.5, 2.0]])
    outs = []
    for storage in (None, round_bf16):
        st = Stage(specs, [Wm, b], policy="latest", lam=0.1, lr=0.3, momentum=0.9, n=1, storage=storage)
        y = st.forward(0, 0, x)
        st.backward(0, dy)
        g = [t.copy() for t in st.g]
        st.update(0)
        outs.append((y, g, [t.copy() for t in st.m], [t.copy() for t in st.weights[1]]))
    (y0, g0, m0, w0), (y1, g1, m1, w1) = outs
    assert np.array_equal(y1, round_bf16(y0)) and not np.array_equal(y1, y0)   # the output IS stored in bf16
    for a, c in zip(g0 + m0 + w0, g1 + m1 + w1):
        assert np.array_equal(a, c)                                # bias kept exact: same gradients, momentum, weights


@pytest.mark.parametrize("name", ["dense", "conv", "bottleneck", "transformer"])
def test_bf16_storage_stays_close_to_pure_fp64_on_smooth_nets(name):
    # every activation GELU (or none), no pooling: nothing hinges on a sign or a maximum, so the rounded run is the
    # pure run plus rounding noise: 2^-9 relative per stored tensor, a handful of stored tensors deep
    specs = _cases()[name]
    specs = tuple(s for s in specs if s.kind != "pool")
    if name == "conv":
        specs = (W.Conv2d(3, 4, 4, 6, "gelu"), W.Conv2d(4, 5, 4, 6, "gelu"))
    if name == "bottleneck":                                       # statistics over 128 / 32 values, not over 8
        specs = W.bottleneck_down_block(8, 4, 16, 8, 8) + W.bottleneck_block(16, 8, 4, 4)
    specs = tuple(type(s)(**{**s.__dict__, "act": "gelu"}) if getattr(s, "act", "none") == "relu" else s for s in specs)
    params = _params(specs, 3)
    pure = _run(specs, params, None, lr=0.01)
    rnd = _run(specs, params, round_bf16, lr=0.01)
    for k in pure:
        err = np.linalg.norm(rnd[k] - pure[k]) / np.linalg.norm(pure[k])
        assert err < 2e-2, (k, err)                              # the bf16 tolerance itself
        if k.startswith(("y", "dx")):
            assert np.array_equal(rnd[k], round_bf16(rnd[k])), k   # what leaves the stage is bf16
            assert err > 1e-5, (k, err)                            # and the hook did round something


def test_relu_side_is_the_side_of_the_stored_output():
    # relu'(z) = [z > 0] on the fp64 pre-activation is the same decision as [stored output > 0]: rounding to
    # bfloat16 never moves a positive value to zero (short of underflow) nor a non-positive one above it
    specs = (W.Dense(16, 64, "relu"), W.Dense(64, 8, "none"))
    params = _params(specs, 4)
    st = Stage(specs, params, policy="latest", lam=0.1, lr=0.1, momentum=0.0, n=1, storage=round_bf16)
    x = np.random.default_rng(5).standard_normal((32, 16))
    st.forward(0, 0, x)
    (x0, z0), (x1, z1) = st.inflight[0]["saved"][0]
    assert np.array_equal(z0 > 0, x1 > 0)                          # x1 = stored output of layer 0
    assert 0.2 < np.mean(z0 > 0) < 0.8


def test_pooling_maximum_is_taken_on_stored_values():
    # an identity convolution stores q(x); two window entries that differ in fp64 but share one bfloat16 value tie
    # in storage mode (first one wins), while the pure run sends the gradient to the larger one
    specs = (W.Conv2d(1, 1, 2, 2, "none"), W.MaxPool2(1, 2, 2))
    Wc = np.zeros((1, 3, 3, 1)); Wc[0, 1, 1, 0] = 1.0
    x = np.array([1.0 + 2.0 ** -10, 1.0 + 2.0 ** -9, 0.5, -1.0]).reshape(1, 2, 2, 1)
    dx = {}
    for key, storage in (("pure", None), ("bf16", round_bf16)):
        st = Stage(specs, [Wc, np.zeros(1)], policy="latest", lam=0.1, lr=0.1, momentum=0.0, n=1, storage=storage)
        y = st.forward(0, 0, x)
        dx[key] = st.backward(0, np.ones_like(y)).reshape(-1)
        assert y.reshape(-1)[0] == (1.0 if storage else 1.0 + 2.0 ** -9)
    assert np.array_equal(dx["pure"], [0.0, 1.0, 0.0, 0.0])
    assert np.array_equal(dx["bf16"], [1.0, 0.0, 0.0, 0.0])
