"""GPU parity at the full sizes that bench.py times, in its launch configuration: the interior
stage of the width-4096 GELU MLP (micro-batch 256 x 8, pipeline depth 3) and stage 0 of the
VGG-style net on 32x32x3 images (micro-batch 64 x 4, depth 4).  The fp64 oracle is small enough at
these sizes to run whole (a few seconds per mini-batch on the host), so every output element is
compared, not a sample: outputs, input gradients, weight and bias gradients and the updated
weights of every mini-batch, with real staleness under the I-TiMePReSt blend."""
import time

import numpy as np
import pytest

from synth_inputs import workloads as W
from test_gpu_conv_stage import _run_stage

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
def test_mlp4096_interior_stage_full_size():
    w = W.mlp_wide(width=4096, mb=256, n=8)
    t0 = time.time()
    worst = _run_stage(w.stages[1], "mlp4096_full", "bf16", mb=w.mb, n=w.n, policy="convex", depth=3, minibatches=3,
                       needs_dx=True, lr=w.lr)
    print(f"{time.time() - t0:.1f} s", worst)


@pytest.mark.timeout(900)
def test_vgg_stage0_full_size():
    # The synthetic upstream gradient is no loss gradient: summed over 262,144 output pixels it is
    # about 80 x the weights' own scale, so at the workload's lr 0.01 one update would replace the
    # weights by the gradient and the following mini-batches would compare amplified bf16 noise.
    # lr 2e-4 makes one update move the weights by a percent or two, as a training step does.
    w = W.vgg_stage0(mb=64, n=4)
    t0 = time.time()
    worst = _run_stage(w.stages[0], "vgg32_full", "bf16", mb=w.mb, n=w.n, policy="convex", depth=4, minibatches=5,
                       needs_dx=False, lr=2e-4)
    print(f"{time.time() - t0:.1f} s", worst)


@pytest.mark.timeout(900)
def test_bottleneck_blocks_full_geometry():
    # two of the identity bottlenecks of the conv4_x group at their real geometry (1024 -> 256 -> 1024
    # channels on 4x4 feature maps, micro-batch 128 x 4): small enough for the whole oracle
    w = W.bottleneck_stage(blocks=2)
    t0 = time.time()
    worst = _run_stage(w.stages[1], "bneck_full", "bf16", mb=w.mb, n=w.n, policy="convex", depth=3, minibatches=3,
                       needs_dx=True, lr=2e-4)
    print(f"{time.time() - t0:.1f} s", worst)


@pytest.mark.timeout(900)
def test_bottleneck_down_block_full_geometry():
    # the first block of the conv4_x group at its real geometry: [8, 8, 512] -> [4, 4, 1024], 3x3 with stride 2 on
    # 256 channels, projection shortcut 512 -> 1024; followed by one identity block
    w = W.bottleneck_stage(blocks=1, down=True)
    t0 = time.time()
    worst = _run_stage(w.stages[1], "bneck_down_full", "bf16", mb=w.mb, n=w.n, policy="convex", depth=3, minibatches=3,
                       needs_dx=True, lr=2e-4)
    print(f"{time.time() - t0:.1f} s", worst)


@pytest.mark.timeout(900)
def test_conv3_group_first_block_full_geometry():
    # the first block of the conv3_x group at its real geometry: [16, 16, 256] -> [8, 8, 512] with 128 middle
    # channels (32768 rows per micro-batch in front of the stride: the streaming normalisation kernels), one
    # identity block behind it
    w = W.bottleneck_stage(c=512, mid=128, h=8, w=8, blocks=1, down=True)
    t0 = time.time()
    worst = _run_stage(w.stages[1], "conv3_down_full", "bf16", mb=w.mb, n=w.n, policy="convex", depth=3, minibatches=2,
                       needs_dx=True, lr=2e-4)
    print(f"{time.time() - t0:.1f} s", worst)


@pytest.mark.timeout(1200)
def test_transformer_block_full_geometry_sampled_sequences():
    """One of the four identical blocks of the transformer stage at its real geometry (d_model 2048, 16 heads
    of 128, FFN 8192, 1024 tokens, micro-batch 8 x 4: GEMMs with 8192 rows, attention over 1024 keys).  The
    whole oracle would take minutes per mini-batch in fp64, but sequences do not interact: the outputs and
    input gradients of two sampled sequences, and the parameter gradients when only those two sequences carry
    an upstream gradient, are compared with the oracle run on those two sequences alone."""
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
    x = W.stage_input(w, 1, 0)                                   # [32, 1024, 2048], bf16 values
    print(f"inputs and {sum(p.size for p in params) / 1e6:.1f} M parameters generated in {time.time() - t0:.0f} s", flush=True)
    st = GpuStage([layer_tuple(l) for l in specs], params, dtype="bf16", mb=mb, n=n, stage_index=1, num_stages=4,
                  policy="convex", lam=0.1, lr=w.lr, momentum=w.momentum, needs_dx=True)
    rows = n * mb
    xt = torch.from_numpy(x.reshape(rows, -1)).cuda().to(st.tdtype)
    y = torch.empty(rows, st.out_elems, dtype=st.tdtype, device="cuda")
    for ub in range(n):
        st.forward(0, ub, xt[ub * mb:(ub + 1) * mb], y[ub * mb:(ub + 1) * mb])
    picks = [3, 2 * mb + 1]                                       # one sequence of micro-batch 0, one of micro-batch 2
    ost = Stage(specs, params, policy="convex", lam=0.1, lr=w.lr, momentum=w.momentum, n=2, storage=W.round_bf16)
    ref_y = [ost.forward(0, i, x[b:b + 1]) for i, b in enumerate(picks)]
    tol = TOL["bf16"]
    for b, ry in zip(picks, ref_y):
        e = rel_err(to_np(y[b]), ry.reshape(-1))
        print(f"y[{b}] {e:.2e}", flush=True)
        assert e <= tol
    dy = np.zeros((rows, tokens, dm))
    dy[picks] = W.round_bf16(np.random.default_rng(4).standard_normal((2, tokens, dm)) / np.sqrt(dm))
    dx, delta = st.backward(0, torch.from_numpy(dy.reshape(rows, -1)).cuda().to(st.tdtype))
    assert delta == 0
    ref_dx = ost.backward(0, dy[picks])
    for i, b in enumerate(picks):
        e = rel_err(to_np(dx[b]), ref_dx[i].reshape(-1))
        print(f"dx[{b}] {e:.2e}", flush=True)
        assert e <= tol
    other = [b for b in range(rows) if b not in picks]
    assert float(dx[other].abs().max()) == 0.0                    # no upstream gradient, no input gradient
    for pi, (got, ref) in enumerate(zip(st.unpack(to_np(st.grad)), ost.g)):
        e = rel_err(got, ref)
        print(f"g[{pi}] {e:.2e}", flush=True)
        assert e <= tol, pi
    st.close()
    print(f"{time.time() - t0:.0f} s")
