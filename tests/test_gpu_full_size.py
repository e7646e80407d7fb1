"""GPU parity at the full sizes that bench.py times, in its launch configuration: the interior
stage of the width-4096 GELU MLP (micro-batch 256 x 8, pipeline depth 3) and stage 0 of the
VGG-style net on 32x32x3 images (micro-batch 64 x 4, depth 4).  The fp64 oracle is small enough at
these sizes to run whole (a few seconds per mini-batch on the host), so every output element is
compared, not a sample: outputs, input gradients, weight and bias gradients and the updated
weights of every mini-batch, with real staleness under the I-TiMePReSt blend."""
import time

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
