"""GPU parity of bottleneck-shaped stages (1x1 convolutions as per-position dense layers, batch
normalisation per micro-batch, 3x3 convolution, residual add followed by ReLU) against the fp64 oracle."""
import pytest

from synth_inputs import workloads as W
from stage_parity import run_stage as _run_stage

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


@pytest.mark.parametrize("act,fixed", [("gelu", False), ("relu", True), ("relu", False)])
def test_bottleneck_matrix_core_shapes_bf16(act, fixed):
    # 256 -> 128 -> 256 channels at 4x4: bf16 GEMMs and the gathered 3x3 convolution on the matrix cores.
    # With GELU in place of the ReLUs, and with ReLUs whose masks are fixed by the normalisation shifts (four
    # standard deviations from zero), every tensor meets the normal bf16 tolerance; with ReLUs on centred
    # pre-activations the differing mask decisions are counted, must be near zero, and widen the gradient tolerance
    specs = W.bottleneck_block(256, 128, 4, 4, act) + W.bottleneck_block(256, 128, 4, 4, act)
    print(act, fixed, _run_stage(specs, f"bneck_mfma_{act}", "bf16", mb=8, n=2, depth=2, minibatches=3, fixed_masks=fixed))


# ---- first block of a group: 3x3 with stride 2, projection shortcut (subsample + 1x1 + batch norm) -------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_down_block_then_identity_block(dtype):
    # 16 channels on 8x8 -> 32 channels on 4x4 (generic kernels); 64 values per channel and micro-batch behind the
    # stride, so that the batch statistics do not amplify bf16 noise
    specs = W.bottleneck_down_block(16, 16, 32, 8, 8, "gelu") + W.bottleneck_block(32, 16, 4, 4, "gelu")
    print(dtype, _run_stage(specs, f"bneck_down_small_{dtype}", dtype, mb=4, n=2, depth=3, minibatches=3))


def test_down_block_first_stage_relu_fp32():
    print(_run_stage(W.bottleneck_down_block(8, 4, 8, 4, 6), "bneck_down_first", "f32", mb=3, n=2, needs_dx=False))


def test_strided_convolution_alone_fp32_and_bf16():
    # 3x3 stride 2 on a non-square image, followed by a dense layer on the smaller grid
    specs = (W.Conv2d(8, 16, 6, 4, "gelu", stride=2), W.Dense(16, 8, "none", tokens=6))
    print(_run_stage(specs, "conv_s2_f32", "f32", mb=3, n=2))
    print(_run_stage(specs, "conv_s2_bf16", "bf16", mb=3, n=2))


@pytest.mark.parametrize("act,fixed", [("gelu", False), ("relu", True), ("relu", False)])
def test_down_block_matrix_core_shapes_bf16(act, fixed):
    # 128 channels on 8x8 -> 256 on 4x4 with 64 / 128 in the middle: the strided 3x3 runs on the gathered matrix-core
    # kernels (fprop rows: output pixels; dgrad rows: input pixels, taps of the wrong parity read zeros; wgrad
    # contraction over the output pixels)
    for mid in (64, 128):
        specs = W.bottleneck_down_block(128, mid, 256, 8, 8, act) + W.bottleneck_block(256, mid, 4, 4, act)
        print(act, fixed, mid, _run_stage(specs, f"bneck_down_mfma_{act}_{mid}", "bf16", mb=8, n=2, depth=2, minibatches=3,
                                          fixed_masks=fixed))


@pytest.mark.parametrize("mb,positions", [(6, 300), (3, 3000), (2, 9000)])
def test_batchnorm_row_counts_across_kernel_families_bf16(mb, positions):
    # rows per micro-batch 1800 (register-resident kernels, two loads per lane, ragged), 9000 (forward in registers,
    # backward streaming) and 18000 (both streaming); GELU keeps bf16 away from kinks
    specs = (W.Dense(8, 16, "none", tokens=positions), W.BatchNorm(16, positions, "gelu"),
             W.Dense(16, 8, "none", tokens=positions), W.BatchNorm(8, positions, "none"))
    print(mb * positions, _run_stage(specs, f"bn_rows_{mb * positions}", "bf16", mb=mb, n=3))


def test_dense_weight_gradient_split_over_rows_bf16():
    # 2048 rows (64 x 2 samples x 16 positions) against weight matrices of 128 x 256 and 64 x 128: too few output
    # tiles to fill the chip, so the gradient is formed over several row ranges and summed in a fixed order
    specs = (W.Dense(256, 128, "gelu", tokens=16), W.Dense(128, 64, "none", tokens=16))
    print(_run_stage(specs, "wgrad_split", "bf16", mb=64, n=2))
