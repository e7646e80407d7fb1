"""GPU parity of convolution / pooling stages against the fp64 oracle: a single stage driven with
synthetic inputs and upstream gradients through forward, backward (with real staleness under the
I-TiMePReSt blend) and update, in both precisions, at shapes that cover image borders, channel
counts that do and do not fit the matrix-core kernels, and the VGG-style first stage."""
import numpy as np
import pytest

from stage_parity import run_stage as _run_stage
from synth_inputs import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_conv_pool_stage(dtype):
    # ragged channel counts and a non-square image: the generic kernels, every border case
    specs = (W.Conv2d(3, 5, 6, 4, "gelu"), W.Conv2d(5, 7, 6, 4, "gelu"), W.MaxPool2(7, 6, 4), W.Conv2d(7, 6, 3, 2, "gelu"))
    print(dtype, _run_stage(specs, f"convsmall_{dtype}", dtype, mb=3, n=2))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pool_first_and_last(dtype):
    specs = (W.MaxPool2(4, 4, 4), W.Conv2d(4, 8, 2, 2, "gelu"), W.MaxPool2(8, 2, 2))
    print(dtype, _run_stage(specs, f"poolends_{dtype}", dtype, mb=2, n=2))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_conv_channels_multiple_of_64(dtype):
    # channel counts the matrix-core kernels take (64, 128), small images, 3 stale versions in play
    specs = (W.Conv2d(64, 64, 8, 8, "gelu"), W.MaxPool2(64, 8, 8), W.Conv2d(64, 128, 4, 4, "gelu"),
             W.Conv2d(128, 128, 4, 4, "gelu"))
    print(dtype, _run_stage(specs, f"conv64_{dtype}", dtype, mb=4, n=2, depth=3, minibatches=4))


@pytest.mark.parametrize("pure_oracle", [False, True])
def test_conv_matrix_core_tile_variants(pure_oracle):
    # non-square power-of-two image, channel counts that are multiples of 64 but not of 128 (the
    # narrower tiles), 768 pixels per mini-batch = six row tiles, no pooling: normal tolerance throughout,
    # against the oracle with bf16-stored tensors and against the plain fp64 oracle
    specs = (W.Conv2d(128, 192, 4, 16, "gelu"), W.Conv2d(192, 64, 4, 16, "gelu"), W.Conv2d(64, 128, 4, 16, "none"))
    print(_run_stage(specs, "convtiles_bf16", "bf16", mb=6, n=2, depth=2, minibatches=3, pure_oracle=pure_oracle))


def test_first_layer_few_channels_bf16():
    # a first layer with 5 input channels (padded to 8 inside the stage), 128 output channels = two
    # channel blocks, input gradient requested: the few-channel forward and weight-gradient kernels next
    # to the generic input-gradient kernel
    specs = (W.Conv2d(5, 128, 16, 16, "gelu"), W.Conv2d(128, 64, 16, 16, "none"))
    print(_run_stage(specs, "conv5ch_bf16", "bf16", mb=2, n=2, depth=2, minibatches=3, needs_dx=True))


def test_vgg_first_stage_reduced_bf16():
    # the VGG-style stage 0 (conv3-64, conv3-64, pool, conv3-128, conv3-128, pool) on 16x16 images,
    # micro-batch 4 x 2; GELU instead of ReLU keeps the bf16 comparison away from the ReLU kink
    w = W.vgg_stage0(mb=4, n=2, size=16)
    specs = tuple(type(l)(**{**l.__dict__, "act": "gelu"}) if l.kind == "conv" else l for l in w.stages[0])
    print(_run_stage(specs, "vgg16px_bf16", "bf16", mb=4, n=2, depth=4, minibatches=4, needs_dx=False))


def test_vgg_first_stage_relu_fp32():
    w = W.vgg_stage0(mb=2, n=2, size=8, c1=16, c2=32, dtype="f32")
    print(_run_stage(w.stages[0], "vgg8px_f32", "f32", mb=2, n=2, depth=4, minibatches=4, needs_dx=False))


# ---- ReLU in bf16 with masks that do not hinge on rounding: normal tolerance on every tensor ----------------------

def test_conv_relu_fixed_masks_patch_kernels_bf16():
    # 16x16 images (256 pixels: the patch kernels), few-channel first layer, 64 / 128 channels, ReLU everywhere with
    # every pre-activation four standard deviations away from zero: the input-gradient kernels take their ReLU mask
    # from the saved outputs and must meet the normal tolerance
    specs = (W.Conv2d(3, 64, 16, 16, "relu"), W.Conv2d(64, 64, 16, 16, "relu"), W.Conv2d(64, 128, 16, 16, "relu"),
             W.Conv2d(128, 64, 16, 16, "none"))
    print(_run_stage(specs, "conv_relu_fixed_patch", "bf16", mb=4, n=2, depth=3, minibatches=4, needs_dx=False,
                     fixed_masks=True))


def test_conv_relu_fixed_masks_gather_kernels_bf16():
    # 4x4 images (the gathered kernels), a ReLU in front of a subsampling (its mask is applied by the elementwise
    # kernel) and in front of convolutions (by the input-gradient epilogue), input gradient requested
    specs = (W.Conv2d(64, 128, 8, 8, "relu"), W.Subsample2(128, 8, 8), W.Conv2d(128, 128, 4, 4, "relu"),
             W.Conv2d(128, 64, 4, 4, "relu"), W.Conv2d(64, 64, 4, 4, "none"))
    print(_run_stage(specs, "conv_relu_fixed_gather", "bf16", mb=4, n=2, depth=2, minibatches=3, fixed_masks=True))


def test_vgg_first_stage_reduced_relu_fixed_masks_bf16():
    # the VGG-style stage 0 with its ReLUs and pools on 16x16 images; ReLU masks fixed, pooling windows decided by
    # the data (differing windows are counted and must be near-ties)
    w = W.vgg_stage0(mb=4, n=2, size=16)
    print(_run_stage(w.stages[0], "vgg16px_relu_fixed", "bf16", mb=4, n=2, depth=4, minibatches=4, needs_dx=False,
                     fixed_masks=True))


def test_dense_relu_fixed_masks_bf16():
    # dense ReLU layers at matrix-core shapes: dgrad with the mask read off the saved output
    specs = (W.Dense(256, 512, "relu"), W.Dense(512, 256, "relu"), W.Dense(256, 128, "relu"), W.Dense(128, 64, "none"))
    print(_run_stage(specs, "dense_relu_fixed", "bf16", mb=64, n=2, depth=3, minibatches=4, fixed_masks=True))


def test_deep_dense_stack_more_sums_than_one_launch_takes_bf16():
    # 60 dense GELU layers of width 64 on 1024 rows: every layer's weight gradient is formed over two row ranges, so
    # with the bias column sums the backward pass ends with 120 sums of partials -- more than the 96 one launch takes,
    # so they go out in two.  Weights N(0, 1 / fan_in): every layer contracts, so the rounding noise of bf16 storage is
    # damped on its way through the stack instead of amplified (at unit scale 60 GELU layers turn it into 10-40 % of
    # the exact gradients); what is left of it floors the tolerance (see run_stage).
    from synth_inputs import normal, round_f32
    specs = tuple(W.Dense(64, 64, "gelu") for _ in range(60))
    params = []
    for i in range(60):
        params.append(round_f32(normal(f"deep_dense60/W{i}", (64, 64), std=float(np.sqrt(1.0 / 64)))))
        params.append(round_f32(normal(f"deep_dense60/b{i}", (64,), std=0.05)))
    worst = _run_stage(specs, "deep_dense60", "bf16", mb=256, n=4, policy="convex", minibatches=2, depth=2, needs_dx=True,
                       mean_loss_dy=True, lr=0.01, params=params, storage_floor=True)
    print({k: v for k, v in worst.items() if "[" not in k})
