"""GPU parity of the layers a ResNet-style net has around its bottleneck groups -- convolutions with kernels other
than 3x3 (the 7x7 stride-2 stem), global average pooling, the classifier -- and of the first and last stage of the
4-stage split built from them, against the fp64 oracle."""
import pytest

from synth_inputs import workloads as W
from stage_parity import run_stage as _run_stage

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("k,stride", [(7, 2), (7, 1), (5, 2), (5, 1), (1, 2), (1, 1)])
def test_convolution_kernel_sizes_fp32_and_bf16(k, stride):
    # a non-square image smaller than the 7x7 kernel is wide: every tap meets the border somewhere; the input
    # gradient (needs_dx) runs the transposed product with taps of the wrong parity skipped at stride 2
    h, w = 6, 8
    specs = (W.Conv2d(3, 16, h, w, "gelu", k=k, stride=stride, pad=(k - 1) // 2),
             W.Dense(16, 8, "none", tokens=(h // stride) * (w // stride)))
    print(_run_stage(specs, f"conv_k{k}_s{stride}_f32", "f32", mb=3, n=2))
    print(_run_stage(specs, f"conv_k{k}_s{stride}_bf16", "bf16", mb=3, n=2))


def test_convolution_7x7_many_channels_bf16():
    # 7x7 on 24 -> 72 channels (ragged against the 64-wide tiles of the generic kernel), contraction 49 * 24 = 1176
    specs = (W.Conv2d(24, 72, 8, 8, "gelu", k=7, stride=2, pad=3), W.Conv2d(72, 16, 4, 4, "none", k=5, stride=1, pad=2))
    print(_run_stage(specs, "conv_k7_wide_bf16", "bf16", mb=4, n=3))


@pytest.mark.parametrize("h,w,cin,cout", [(32, 32, 3, 64), (64, 32, 3, 128), (32, 64, 5, 64), (16, 128, 1, 64)])
def test_stem_convolution_on_the_matrix_cores_bf16(h, w, cin, cout):
    # 7x7 stride 2 as the first layer of a stage on few input channels: the matrix-core kernels on the 8-slot padded
    # copy of the input (forward, weight gradient); tiles of 256 / 128 output pixels are 16, 8, 4 or 2 output rows
    specs = (W.Conv2d(cin, cout, h, w, "gelu", k=7, stride=2, pad=3), W.Dense(cout, 16, "none", tokens=(h // 2) * (w // 2)))
    print(_run_stage(specs, f"stem_mfma_{h}x{w}_{cin}_{cout}", "bf16", mb=2, n=3, needs_dx=False))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_average_pooling_then_classifier(dtype):
    specs = (W.Dense(8, 24, "gelu", tokens=6), W.AvgPool(24, 6), W.Dense(24, 10, "none"))
    print(dtype, _run_stage(specs, f"avg_head_{dtype}", dtype, mb=5, n=3))


def test_average_pooling_as_last_and_first_layer_fp32():
    print(_run_stage((W.Dense(8, 12, "relu", tokens=4), W.AvgPool(12, 4)), "avg_last", "f32", mb=3, n=2))
    print(_run_stage((W.AvgPool(12, 4), W.Dense(12, 6, "none")), "avg_first", "f32", mb=3, n=2))
    print(_run_stage((W.AvgPool(12, 4), W.Dense(12, 6, "none")), "avg_first_nodx", "f32", mb=3, n=2, needs_dx=False))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_stem_stage(dtype):
    # 16x16x3 images: 7x7 stride 2 -> 8x8x24, BN, pooling -> 4x4, a projection bottleneck 24 -> 96 and one identity
    # bottleneck (generic kernels); first stage of the pipeline, so no input gradient.  The gradients of the stem's
    # normalisation are sums that nearly cancel (what follows it is pooling, then dense layers whose outputs are
    # normalised: their input gradients add up to almost nothing over a micro-batch), so storing the terms in bf16
    # moves them by 2-6 % of their size by the oracle's own account: the bf16 run is held to the larger of the
    # tolerance and that distance
    specs = W.resnet_stem_stage(size=16, c=24, mid=24, cout=96, blocks=1, act="gelu")
    print(dtype, _run_stage(specs, f"stem_small_{dtype}", dtype, mb=16, n=2, depth=4, minibatches=3, needs_dx=False,
                            mean_loss_dy=True, lr=0.01, storage_floor=dtype == "bf16"))


def test_small_stem_stage_relu_fp32():
    specs = W.resnet_stem_stage(size=16, c=8, mid=8, cout=32, blocks=1, act="relu")
    print(_run_stage(specs, "stem_small_relu", "f32", mb=8, n=2, depth=4, minibatches=3, needs_dx=False))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_head_stage(dtype):
    # [4, 4, 48] -> stride-2 bottleneck with projection -> [2, 2, 96], one identity bottleneck, average pooling,
    # classifier (generic kernels); 16 samples x 4 positions per channel behind the stride.  In bf16 every tensor is
    # held to the larger of the tolerance and what bf16 storage does to it by the oracle's own account
    specs = W.resnet_head_stage(c=96, mid=24, h=2, blocks=1, classes=10, act="gelu")
    print(dtype, _run_stage(specs, f"head_small_{dtype}", dtype, mb=16, n=2, depth=2, minibatches=3, stage_index=2,
                            storage_floor=dtype == "bf16"))


@pytest.mark.parametrize("act,fixed", [("gelu", False), ("relu", True)])
def test_stem_stage_matrix_core_shapes_bf16(act, fixed):
    # 32x32x3 images, 64 channels behind the stem: the conv2_x group's 1x1 and 3x3 convolutions (64 -> 64 -> 256 on
    # 8x8 maps) and the stem run on the matrix cores
    specs = W.resnet_stem_stage(size=32, c=64, mid=64, cout=256, blocks=1, act=act)
    print(act, _run_stage(specs, f"stem_mfma_{act}", "bf16", mb=8, n=2, depth=4, minibatches=3, needs_dx=False,
                          fixed_masks=fixed, mean_loss_dy=True, lr=0.01, storage_floor=True))


@pytest.mark.parametrize("act,fixed", [("gelu", False), ("relu", False)])
def test_head_stage_matrix_core_shapes_bf16(act, fixed):
    # [4, 4, 128] -> [2, 2, 256] with 64 middle channels: the 3x3 convolutions run on the gathered matrix-core kernels
    # on 2x2 maps (every tap but the centre meets the border), the classifier's 200 columns are not a multiple of 64.
    # ReLUs on centred pre-activations, their differing decisions counted: shifts that fix the masks would leave the
    # classifier, which no normalisation follows, with inputs that are a constant plus a small remainder
    specs = W.resnet_head_stage(c=256, mid=64, h=2, blocks=1, classes=200, act=act)
    print(act, _run_stage(specs, f"head_mfma_{act}", "bf16", mb=32, n=2, depth=2, minibatches=3, stage_index=2,
                          fixed_masks=fixed))
