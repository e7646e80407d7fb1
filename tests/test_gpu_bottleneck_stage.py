"""GPU parity of bottleneck-shaped stages (1x1 convolutions as per-position dense layers, batch
normalisation per micro-batch, 3x3 convolution, residual add followed by ReLU) against the fp64 oracle."""
import pytest

from synth_inputs import workloads as W
from test_gpu_conv_stage import _run_stage

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_batchnorm_between_dense_layers(dtype):
    # 5 positions x 24 channels (ragged), GELU so that bf16 stays away from kinks, three micro-batches
    specs = (W.Dense(24, 40, "none", tokens=5), W.BatchNorm(40, 5, "gelu"), W.Dense(40, 16, "none", tokens=5),
             W.BatchNorm(16, 5, "none"))
    print(dtype, _run_stage(specs, f"bn_{dtype}", dtype, mb=4, n=3))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_bottleneck_blocks(dtype):
    specs = W.bottleneck_block(16, 8, 4, 4) + W.bottleneck_block(16, 8, 4, 4)
    print(dtype, _run_stage(specs, f"bneck_small_{dtype}", dtype, mb=4, n=2, depth=3, minibatches=4))


def test_bottleneck_first_stage_no_input_gradient():
    print(_run_stage(W.bottleneck_block(16, 8, 2, 4), "bneck_first", "f32", mb=3, n=2, needs_dx=False))


@pytest.mark.parametrize("act", ["gelu", "relu"])
def test_bottleneck_matrix_core_shapes_bf16(act):
    # 256 -> 128 -> 256 channels at 4x4: bf16 GEMMs and the gathered 3x3 convolution on the matrix cores.
    # With GELU in place of the ReLUs every tensor meets the normal bf16 tolerance; with ReLU the gradients
    # are held to the looser one (mask decisions behind a batch normalisation, see _run_stage).
    specs = W.bottleneck_block(256, 128, 4, 4, act) + W.bottleneck_block(256, 128, 4, 4, act)
    print(act, _run_stage(specs, f"bneck_mfma_{act}", "bf16", mb=8, n=2, depth=2, minibatches=3))
