"""GPU parity at the full sizes that bench.py times, in its launch configuration (the forwards on two streams of
their own; what differs from bench.py is that the outputs are read after every mini-batch's forwards, so the next
backward pass starts behind them -- tests/test_gpu_forward_streams.py covers forwards still under way beside it): the interior
stage of the width-4096 GELU MLP (micro-batch 256 x 8, pipeline depth 3) and stage 0 of the
VGG-style net on 32x32x3 images (micro-batch 64 x 4, depth 4).  The fp64 oracle is small enough at
these sizes to run whole (a few seconds per mini-batch on the host), so every output element is
compared, not a sample: outputs, input gradients, weight and bias gradients and the updated
weights of every mini-batch, with real staleness under the I-TiMePReSt blend."""
import time

import numpy as np
import pytest

from synth_inputs import workloads as W
from stage_parity import run_stage as _run_stage

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
def test_mlp4096_interior_stage_full_size(progress):
    w = W.mlp_wide(width=4096, mb=256, n=8)
    t0 = time.time()
    worst = _run_stage(w.stages[1], "mlp4096_full", "bf16", mb=w.mb, n=w.n, policy="convex", depth=3, minibatches=3,
                       needs_dx=True, lr=w.lr, forward_stream=2, progress=progress)
    print(f"{time.time() - t0:.1f} s", worst)


@pytest.mark.timeout(900)
def test_vgg_stage0_full_size(progress):
    # the workload's own optimiser settings (lr 0.01, momentum 0.9); the synthetic upstream gradient is scaled like
    # that of a loss averaged over the mini-batch, the scale at which such a step is a training step
    w = W.vgg_stage0(mb=64, n=4)
    t0 = time.time()
    worst = _run_stage(w.stages[0], "vgg32_full", "bf16", mb=w.mb, n=w.n, policy="convex", depth=4, minibatches=5,
                       needs_dx=False, lr=w.lr, lam=w.lam, mean_loss_dy=True, forward_stream=2, progress=progress)
    print(f"{time.time() - t0:.1f} s", worst)


@pytest.mark.timeout(900)
def test_vgg_stage0_full_size_fixed_masks(progress):
    w = W.vgg_stage0(mb=64, n=4)
    t0 = time.time()
    worst = _run_stage(w.stages[0], "vgg32_full_fixed", "bf16", mb=w.mb, n=w.n, policy="convex", depth=4, minibatches=4,
                       needs_dx=False, lr=w.lr, lam=w.lam, mean_loss_dy=True, fixed_masks=True, progress=progress)
    print(f"{time.time() - t0:.1f} s", worst)


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("act,fixed", [("gelu", False), ("relu", True)])
def test_conv4_group_whole_full_geometry(act, fixed, progress):
    # the stage bench.py --workload bneck times, whole: the strided first bottleneck [8, 8, 512] -> [4, 4, 1024] with
    # its projection shortcut and the five identity bottlenecks 1024-256-256-1024, micro-batch 128 x 4, the workload's
    # lr 0.01; two mini-batches in flight, so the second backward runs on blended weights (delta 1).  Every tensor,
    # stored activations included, in two forms: ReLUs with fixed masks at the normal tolerance; GELU in place of the
    # ReLUs at the larger of the normal tolerance and the distance between the oracle's own two modes on that tensor
    # (storing 52 layers' activations in bf16 moves the exact gradients by more than 2e-2 by itself: the GPU has to
    # agree with the bf16-storing oracle at least as well as that oracle agrees with the exact one)
    w = W.bottleneck_stage(blocks=5, down=True, act=act)
    t0 = time.time()
    worst = _run_stage(w.stages[1], f"conv4x_whole_{act}", "bf16", mb=w.mb, n=w.n, policy="convex", depth=2, minibatches=2,
                       needs_dx=True, lr=w.lr, lam=w.lam, mean_loss_dy=True, fixed_masks=fixed, stage_index=2,
                       storage_floor=(act == "gelu"), forward_stream=2, progress=progress)
    print(f"{time.time() - t0:.1f} s", {k: v for k, v in worst.items() if "[" not in k})


@pytest.mark.timeout(900)
def test_conv4_group_first_blocks_full_geometry_centred_relu(progress):
    # the strided first bottleneck and one identity bottleneck at the real geometry with the workload's own ReLUs on
    # centred pre-activations: the mask decisions that differ between the two sides are counted, each must lie within
    # the rounding noise of zero, and their share bounds the gradient tolerance
    w = W.bottleneck_stage(blocks=1, down=True)
    t0 = time.time()
    worst = _run_stage(w.stages[1], "conv4x_first2_relu", "bf16", mb=w.mb, n=w.n, policy="convex", depth=3, minibatches=3,
                       needs_dx=True, lr=w.lr, lam=w.lam, mean_loss_dy=True, stage_index=1, progress=progress)
    print(f"{time.time() - t0:.1f} s", {k: v for k, v in worst.items() if "[" not in k})


@pytest.mark.timeout(900)
def test_conv3_group_first_block_full_geometry(progress):
    # the first block of the conv3_x group at its real geometry: [16, 16, 256] -> [8, 8, 512] with 128 middle
    # channels (32768 rows per micro-batch in front of the stride: the streaming normalisation kernels), one
    # identity block behind it
    w = W.bottleneck_stage(c=512, mid=128, h=8, w=8, blocks=1, down=True)
    t0 = time.time()
    worst = _run_stage(w.stages[1], "conv3_down_full", "bf16", mb=w.mb, n=w.n, policy="convex", depth=3, minibatches=2,
                       needs_dx=True, lr=2e-4, progress=progress)
    print(f"{time.time() - t0:.1f} s", worst)


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("act,fixed", [("gelu", False), ("relu", True)])
def test_stem_stage_full_geometry(act, fixed, progress):
    # stage 0 of the ResNet-style net as bench.py --workload bneck --stage 0 runs it: 64x64x3 images, 7x7 stride-2 stem
    # to 64 channels (matrix-core kernels on the padded input), batch normalisation over 131072 positions per
    # micro-batch, pooling to 16x16, then the first bottleneck of conv2_x with its projection shortcut and one
    # identity bottleneck (the second one repeats it), micro-batch 128 x 4, no input gradient.  The gradients of
    # the stem's normalisation are sums of terms that nearly cancel; every tensor is held to the larger of the
    # tolerance and what bf16 storage does to it by the oracle's own account
    w = W.resnet_stages()
    specs = W.resnet_stem_stage(64, 64, 64, 256, 1, act)
    t0 = time.time()
    n = w.n if act == "gelu" else 2      # the second form on half the mini-batch: the oracle's time goes with it
    worst = _run_stage(specs, f"stem_full_{act}", "bf16", mb=w.mb, n=n, policy="convex", depth=2, minibatches=2,
                       needs_dx=False, lr=w.lr, lam=w.lam, mean_loss_dy=True, fixed_masks=fixed, storage_floor=True,
                       forward_stream=2, progress=progress)
    print(f"{time.time() - t0:.1f} s", {k: v for k, v in worst.items() if "[" not in k})


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("act", ["gelu", "relu"])
def test_head_stage_full_geometry(act, progress):
    # stage 3 as bench.py --workload bneck --stage 3 runs it, whole: conv5_x ([4, 4, 1024] -> [2, 2, 2048], 512 middle
    # channels: strided bottleneck with projection shortcut and two identity bottlenecks, 3x3 convolutions on 2x2
    # maps), global average pooling, classifier 2048 -> 200; micro-batch 128 x 4.  With GELU every tensor is held to
    # the larger of the tolerance and the oracle's own bf16-storage distance; with the net's ReLUs (centred
    # pre-activations) the differing mask decisions are counted and bound the gradient tolerance
    w = W.resnet_stages()
    specs = W.resnet_head_stage(2048, 512, 2, 2, 200, act)
    t0 = time.time()
    worst = _run_stage(specs, f"head_full_{act}", "bf16", mb=w.mb, n=w.n, policy="convex", depth=2, minibatches=2,
                       needs_dx=True, lr=w.lr, lam=w.lam, mean_loss_dy=True, stage_index=2, storage_floor=(act == "gelu"),
                       forward_stream=2, progress=progress)
    print(f"{time.time() - t0:.1f} s", {k: v for k, v in worst.items() if "[" not in k})


@pytest.mark.timeout(1500)
def test_transformer_block_full_geometry_sampled_sequences():
    """One of the four identical blocks of the transformer stage at its real geometry (d_model 2048, 16 heads
    of 128, FFN 8192, 1024 tokens, micro-batch 8 x 4: GEMMs with 8192 / 32768 rows, attention over 1024 keys),
    two mini-batches in flight: backward 0 (delta 0), the fused update + blend over all 50 M parameters, backward 1 on
    the blended weights (delta 1).  The whole oracle would take minutes per mini-batch in fp64, but sequences do not
    interact: outputs and input gradients of three sampled sequences -- the first of the mini-batch, one in the
    middle, the last (rows up to 32767 of the stacked GEMMs) -- and ALL parameter gradients, momenta, updated and
    blended weights when only those sequences carry an upstream gradient, are compared, tensor by tensor, with the
    oracle run on those sequences alone."""
    import torch
    from oracle.stage import Stage
    from paper_2509_23241_amd.runner import GpuStage, layer_tuple
    from parity_utils import TOL, oracle_flat_to_arena, rel_err, to_np

    w = W.transformer_stage(layers=1)
    specs, mb, n, tokens, dm = w.stages[1], w.mb, w.n, 1024, 2048
    t0 = time.time()
    params = W.init_params(w, 1)
    rng = np.random.default_rng(3)
    params = [p if p.ndim > 1 else W.round_f32(p + 0.1 * rng.standard_normal(p.shape)) for p in params]
    st = GpuStage([layer_tuple(l) for l in specs], params, dtype="bf16", mb=mb, n=n, stage_index=2, num_stages=4,
                  policy="convex", lam=0.1, lr=w.lr, momentum=w.momentum, needs_dx=True)
    rows = n * mb
    picks = [0, 2 * mb + 1, rows - 1]                             # micro-batches 0, 2 and 3; first and last row blocks
    ost = Stage(specs, params, policy="convex", lam=0.1, lr=w.lr, momentum=w.momentum, n=len(picks), storage=W.round_bf16)
    tol = TOL["bf16"]
    worst = {}

    def note(k, e):
        print(f"{k} {e:.2e}", flush=True)
        worst[k] = max(worst.get(k, 0.0), e)
        assert e <= tol, (k, e)

    ys = {}
    for j in range(2):                                            # two mini-batches forward on version 0
        x = W.stage_input(w, 1, j)                                # [32, 1024, 2048], bf16 values
        xt = torch.from_numpy(x.reshape(rows, -1)).cuda().to(st.tdtype)
        y = torch.empty(rows, st.out_elems, dtype=st.tdtype, device="cuda")
        for ub in range(n):
            st.forward(j, ub, xt[ub * mb:(ub + 1) * mb], y[ub * mb:(ub + 1) * mb])
        for i, b in enumerate(picks):
            note(f"y{j}[{b}]", rel_err(to_np(y[b]), ost.forward(j, i, x[b:b + 1]).reshape(-1)))
        print(f"mini-batch {j} forwarded, {time.time() - t0:.0f} s", flush=True)
    for j in range(2):
        # upstream gradient on the sampled sequences only, scaled like that of a loss averaged over the mini-batch
        dy = np.zeros((rows, tokens, dm))
        dy[picks] = W.round_bf16(np.random.default_rng(4 + j).standard_normal((len(picks), tokens, dm)) / (np.sqrt(dm) * rows))
        dx, delta = st.backward(j, torch.from_numpy(dy.reshape(rows, -1)).cuda().to(st.tdtype))
        assert delta == j
        ref_dx = ost.backward(j, dy[picks])
        assert ost.trace[-1][4] == j
        for i, b in enumerate(picks):
            note(f"dx{j}[{b}]", rel_err(to_np(dx[b]), ref_dx[i].reshape(-1)))
        other = [b for b in range(rows) if b not in picks]
        assert float(dx[other].abs().max()) == 0.0                # no upstream gradient, no input gradient
        if j == 1:                                                # the weights this backward ran on: built by the fused update
            for pi, (got, ref) in enumerate(zip(st.unpack(to_np(st.wbwd)), ost.last_W_b)):
                if ref.ndim > 1:                                  # matrices live in the bf16 copy; vectors are blended in fp32 in the kernels
                    note(f"W_b[{pi}]", rel_err(got, ref))
        for pi, (got, ref) in enumerate(zip(st.unpack(to_np(st.grad)), ost.g)):
            note(f"g{j}[{pi}]", rel_err(got, ref))
        ost.update(j)
        assert st.blend_update(j, j + 1 if j == 0 else 2 ** 64 - 1) == j + 1
        for pi, (got, ref, mg, mr) in enumerate(zip(st.unpack(to_np(st.export(j + 1))), ost.weights[j + 1],
                                                    st.unpack(to_np(st.momentum)), ost.m)):
            note(f"W{j + 1}[{pi}]", rel_err(got, ref))
            note(f"m{j + 1}[{pi}]", rel_err(mg, mr))
        print(f"mini-batch {j} backward + update, {time.time() - t0:.0f} s", flush=True)
    st.close()
    print(f"{time.time() - t0:.0f} s", {k: f"{v:.1e}" for k, v in worst.items() if "[" not in k})
