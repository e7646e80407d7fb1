"""The forward passes on streams of their own (stage_set_forward_streams) -- the micro-batches of a mini-batch side by
side, and beside the backward pass of an earlier mini-batch on the stage's stream: the same bits as with everything
on one stream, parity with the oracle, the joins that order the forward streams' results, and the refusals."""
import numpy as np
import pytest

from synth_inputs import workloads as W
from stage_parity import run_stage as _run_stage

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dense_stage_parity_with_second_forward_stream(dtype):
    # five micro-batches (the last even one has no partner), ragged widths in fp32 and matrix-core shapes in bf16
    dims = (72, 200, 48) if dtype == "f32" else (256, 512, 128)
    specs = (W.Dense(dims[0], dims[1], "gelu"), W.Dense(dims[1], dims[1], "relu"), W.Dense(dims[1], dims[2], "none"))
    print(dtype, _run_stage(specs, f"fwd2_mlp_{dtype}", dtype, mb=64, n=5, depth=3, minibatches=4, forward_stream=2))


def test_conv_pool_stage_parity_with_second_forward_stream():
    w = W.vgg_stage0(mb=4, n=4, size=16, c1=64, c2=64)
    print(_run_stage(w.stages[0], "fwd2_vgg", "bf16", mb=w.mb, n=w.n, depth=2, minibatches=3, needs_dx=False,
                     mean_loss_dy=True, lr=0.01, forward_stream=2))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_bottleneck_stage_parity_with_four_forward_streams(dtype):
    # batch normalisation per micro-batch on both streams at once (each with scratch of its own), strided block
    # with projection shortcut, identity block
    specs = W.bottleneck_down_block(16, 16, 32, 8, 8, "gelu") + W.bottleneck_block(32, 16, 4, 4, "gelu")
    print(dtype, _run_stage(specs, f"fwd2_bneck_{dtype}", dtype, mb=4, n=4, depth=3, minibatches=3, forward_stream=3))


def test_last_stage_own_stream_takes_a_turn_bf16():
    # one mini-batch in flight (pipeline depth 1): the backward pass needs the forwards just enqueued, so the stage's
    # own stream runs micro-batches 0 and 4, three forward streams the others; loss-free head: pooling + classifier
    specs = W.resnet_head_stage(c=96, mid=24, h=2, blocks=1, classes=10, act="gelu")
    print(_run_stage(specs, "fwd_last_stage", "bf16", mb=16, n=5, depth=1, minibatches=3, stage_index=3,
                     storage_floor=True, forward_stream=3))


def test_streaming_normalisation_on_both_streams_bf16():
    # 9000 rows per micro-batch: statistics, finalize and normalise kernels with partial sums in scratch memory
    specs = (W.Dense(8, 16, "none", tokens=3000), W.BatchNorm(16, 3000, "gelu"),
             W.Dense(16, 8, "none", tokens=3000), W.BatchNorm(8, 3000, "none"))
    print(_run_stage(specs, "fwd2_bn_rows", "bf16", mb=3, n=4, forward_stream=3))


_INPUTS = {}


def _inputs(st, w, s, steps):
    """Synthetic inputs and upstream gradients of the run, on the device and complete; made once per workload."""
    import torch
    key = (w.name, s, steps, st.tdtype)
    if key not in _INPUTS:
        _INPUTS.clear()
        rows, depth = w.n * w.mb, w.K - s
        xs = [torch.from_numpy(W.stage_input(w, s, j).reshape(rows, -1)).cuda().to(st.tdtype) for j in range(steps + depth)]
        dys = [torch.from_numpy(W.stage_upstream_grad(w, s, j, mean_loss=True).reshape(rows, -1)).cuda().to(st.tdtype)
               for j in range(steps)]
        torch.cuda.synchronize()
        _INPUTS[key] = (xs, dys)
    return _INPUTS[key]


def _drive(st, w, s, steps, join_before_read):
    """bench.py's order of calls: backward, update, then the forwards of a later mini-batch -- whose outputs are read
    only at the end, so that with forward streams they are still under way when the next backward pass is enqueued."""
    import torch
    rows = w.n * w.mb
    depth = w.K - s
    outs, ys = [], []
    xs, dys = _inputs(st, w, s, steps)

    def forward(j):
        y = torch.empty(rows, st.out_elems, dtype=st.tdtype, device="cuda")
        for ub in range(w.n):
            st.forward(j, ub, xs[j][ub * w.mb:(ub + 1) * w.mb], y[ub * w.mb:(ub + 1) * w.mb])
        ys.append(y)

    for j in range(depth):
        forward(j)
    for j in range(steps):
        dx, _ = st.backward(j, dys[j])                      # waits for the forwards of mini-batch j, not for the later ones
        outs.append(dx.float().cpu().numpy())
        outs.append(st.grad.cpu().numpy().copy())
        if depth > 1:
            st.blend_update(j, j + 1)                       # waits for every forward
        else:
            st.blend_update(j)                              # one mini-batch in flight: the next one is not there yet
        outs.append(st.export(j + 1).cpu().numpy())
        forward(j + depth)
    if join_before_read:
        st.forward_join()
    outs.extend(y.float().cpu().numpy() for y in ys)
    return outs


def test_two_streams_give_the_bits_of_one():
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple
    w = W.mlp_wide(width=512, mb=128, n=8)
    s = 1
    layers = [layer_tuple(l) for l in w.stages[s]]
    results = []
    for extra in (0, 1, 3):
        st = GpuStage(layers, W.init_params(w, s), dtype=w.dtype, mb=w.mb, n=w.n, stage_index=s, num_stages=w.K,
                      policy="convex", lam=w.lam, lr=w.lr, momentum=w.momentum, forward_stream=extra)
        results.append(_drive(st, w, s, steps=4, join_before_read=extra > 0))
        st.close()
    for other in results[1:]:
        assert len(results[0]) == len(other)
        for a, b in zip(results[0], other):
            assert np.array_equal(a, b)


def test_two_streams_give_the_bits_of_one_bottleneck_stage():
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple
    w = W.bottleneck_stage(c=256, mid=64, h=4, w=4, blocks=1, mb=16, n=4, down=True)
    s = 1
    layers = [layer_tuple(l) for l in w.stages[s]]
    results = []
    for extra in (0, 2, 3):
        st = GpuStage(layers, W.init_params(w, s), dtype=w.dtype, mb=w.mb, n=w.n, stage_index=s, num_stages=w.K,
                      policy="convex", lam=w.lam, lr=w.lr, momentum=w.momentum, forward_stream=extra)
        results.append(_drive(st, w, s, steps=3, join_before_read=extra > 0))
        st.close()
    for other in results[1:]:
        for a, b in zip(results[0], other):
            assert np.array_equal(a, b)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("which", ["mlp", "conv4_x", "head"])
def test_full_size_stages_in_the_order_of_calls_of_the_benchmark(which):
    # the stages bench.py times, at their full sizes and with its streams, in its order of calls (the forwards of a
    # later mini-batch still under way when the next backward pass is enqueued): every output, input gradient,
    # gradient arena and weight version bit for bit what the same calls give on the stage's stream alone
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple
    if which == "mlp":
        w, s, streams = W.mlp_wide(width=4096, mb=256, n=8), 1, 2
    elif which == "conv4_x":
        w, s, streams = W.resnet_middle_stages(mb=128, n=4), 2, 2
    else:
        w, s, streams = W.resnet_stages(mb=128, n=4), 3, 3
    layers = [layer_tuple(l) for l in w.stages[s]]
    results = []
    for extra in (0, streams):
        st = GpuStage(layers, W.init_params(w, s), dtype=w.dtype, mb=w.mb, n=w.n, stage_index=s, num_stages=w.K,
                      policy="convex", lam=w.lam, lr=w.lr, momentum=w.momentum, forward_stream=extra)
        results.append(_drive(st, w, s, steps=2, join_before_read=extra > 0))
        st.close()
    _INPUTS.clear()
    assert len(results[0]) == len(results[1])
    for a, b in zip(*results):
        assert np.array_equal(a, b)


def test_saved_inputs_of_odd_micro_batches_are_ordered_by_the_accessor():
    import torch
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple
    w = W.mlp_wide(width=256, mb=64, n=4)
    layers = [layer_tuple(l) for l in w.stages[1]]
    st = GpuStage(layers, W.init_params(w, 1), dtype=w.dtype, mb=w.mb, n=w.n, stage_index=1, num_stages=w.K,
                  policy="convex", lam=w.lam, lr=w.lr, momentum=w.momentum, forward_stream=True)
    x = torch.from_numpy(W.stage_input(w, 1, 0).reshape(w.n * w.mb, -1)).cuda().to(st.tdtype)
    torch.cuda.synchronize()
    for ub in range(w.n):
        st.forward(0, ub, x[ub * w.mb:(ub + 1) * w.mb])
    for ub in range(w.n):                                  # the stage's own copy of what each micro-batch came in with
        assert torch.equal(st.saved_input(0, ub, 0).reshape(w.mb, -1), x[ub * w.mb:(ub + 1) * w.mb])
    st.close()


def test_forward_stream_refusals():
    import torch
    from paper_2509_23241_amd import binding as B
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple
    mk = dict(dtype="bf16", mb=4, n=2, stage_index=0, num_stages=2, lam=0.1, lr=0.01, momentum=0.9)
    dense = [(64, 64, "relu")]
    side = [torch.cuda.Stream() for _ in range(4)]
    h = [q.cuda_stream for q in side]
    st = GpuStage(dense, None, policy="convex", **mk)
    for bad in ([0], [st.stream.cuda_stream] if st.stream.cuda_stream else [0], [h[0], h[0]], h):   # null, the stage's own, twice the same, too many
        with pytest.raises(B.StageLibError) as ei:
            B.stage_set_forward_streams(st.handle, bad)
        assert ei.value.code == B.TP_EINVAL
    B.stage_set_forward_streams(st.handle, h[:3])
    B.stage_set_forward_streams(st.handle, [])             # taken away again
    B.stage_forward_join(st.handle)
    st.close()
    attn = [layer_tuple(l) for l in W.transformer_block(64, 2, 128, 8)]
    for layers, policy in ((attn, "convex"), (dense, "timeprest")):
        st = GpuStage(layers, None, policy=policy, **mk)
        with pytest.raises(B.StageLibError) as ei:
            B.stage_set_forward_streams(st.handle, h[:1])
        assert ei.value.code == B.TP_EINVAL
        st.close()
