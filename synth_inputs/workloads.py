"""Shapes and seeded tensors of the synthetic workloads.

Each workload is a chain of layers cut into K pipeline stages, plus the batch
geometry (n micro-batches of `mb` samples per mini-batch) and the optimiser
constants.  Nothing here computes anything of the method: the functions only
describe shapes and draw seeded tensors (inputs, labels, initial parameters,
upstream gradients for a stage timed on its own).

The image workloads stand in for CIFAR-100 / Tiny-ImageNet-200 shaped data:
pixels are N(0,1) draws and labels are uniform; no record of either dataset is
used or reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Tuple

import numpy as np

from . import GLOBAL_SEED, labels as _labels, normal as _normal, round_bf16, round_f32


@dataclass(frozen=True)
class Dense:
    """Fully connected layer; with tokens > 1 it is applied to every one of `tokens` positions of a sample
    (activations [tokens, features] per sample)."""
    in_features: int
    out_features: int
    act: str  # "relu" | "gelu" | "none"
    kind: str = "dense"
    tokens: int = 1

    def param_shapes(self):
        return [(self.out_features, self.in_features), (self.out_features,)]

    def in_shape(self):
        return (self.in_features,) if self.tokens == 1 else (self.tokens, self.in_features)

    def out_shape(self):
        return (self.out_features,) if self.tokens == 1 else (self.tokens, self.out_features)

    def out_dim(self):
        return self.tokens * self.out_features


@dataclass(frozen=True)
class LayerNorm:
    """Layer normalisation over the feature axis of [tokens, d] samples; parameters scale and shift."""
    d: int
    tokens: int
    kind: str = "ln"
    act: str = "none"

    def param_shapes(self):
        return [(self.d,), (self.d,)]

    def in_shape(self):
        return (self.tokens, self.d)

    def out_shape(self):
        return (self.tokens, self.d)

    def out_dim(self):
        return self.tokens * self.d


@dataclass(frozen=True)
class BatchNorm:
    """Batch normalisation (training mode) over all samples and positions of a micro-batch, per channel, on
    [tokens, c] samples (tokens = H*W of an NHWC image), followed by an activation; parameters scale and shift."""
    c: int
    tokens: int
    act: str = "none"
    kind: str = "bn"

    def param_shapes(self):
        return [(self.c,), (self.c,)]

    def in_shape(self):
        return (self.tokens, self.c)

    def out_shape(self):
        return (self.tokens, self.c)

    def out_dim(self):
        return self.tokens * self.c


@dataclass(frozen=True)
class Attention:
    """Causal multi-head self-attention on [tokens, 3*d] (queries | keys | values) -> [tokens, d]; no parameters."""
    d: int
    heads: int
    tokens: int
    kind: str = "attn"
    act: str = "none"

    def param_shapes(self):
        return []

    def in_shape(self):
        return (self.tokens, 3 * self.d)

    def out_shape(self):
        return (self.tokens, self.d)

    def out_dim(self):
        return self.tokens * self.d


@dataclass(frozen=True)
class Residual:
    """mark = "begin": remember the current activation; mark = "add": add the remembered one, then apply the
    activation (if any). No parameters."""
    d: int
    tokens: int
    mark: str
    kind: str = "res"
    act: str = "none"

    def param_shapes(self):
        return []

    def in_shape(self):
        return (self.tokens, self.d)

    def out_shape(self):
        return (self.tokens, self.d)

    def out_dim(self):
        return self.tokens * self.d


@dataclass(frozen=True)
class ResidualSwap:
    """Between a Residual "begin" and its "add": sets the current activation (the main branch's result,
    [tokens, d]) aside as the one the add will add, and hands the tensor remembered at the begin
    ([out_tokens, out_d]) to the next layer, so that the layers up to the add form a projection shortcut."""
    d: int
    tokens: int
    out_d: int
    out_tokens: int
    kind: str = "swap"
    act: str = "none"

    def param_shapes(self):
        return []

    def in_shape(self):
        return (self.tokens, self.d)

    def out_shape(self):
        return (self.out_tokens, self.out_d)

    def out_dim(self):
        return self.out_tokens * self.out_d


@dataclass(frozen=True)
class Subsample2:
    """Every second pixel of every second row of an NHWC image (what a stride-2 1x1 convolution reads); no parameters."""
    c: int
    h: int
    w: int
    act: str = "none"
    kind: str = "sub"

    def param_shapes(self):
        return []

    def in_shape(self):
        return (self.h, self.w, self.c)

    def out_shape(self):
        return (self.h // 2, self.w // 2, self.c)

    def out_dim(self):
        return (self.h // 2) * (self.w // 2) * self.c


@dataclass(frozen=True)
class Conv2d:
    """k x k convolution (k odd) on NHWC activations, weights [Cout][kh][kw][Cin], plus bias and activation."""
    cin: int
    cout: int
    h: int           # input height
    w: int           # input width
    act: str
    k: int = 3
    stride: int = 1
    pad: int = 1
    kind: str = "conv"

    def param_shapes(self):
        return [(self.cout, self.k, self.k, self.cin), (self.cout,)]

    @property
    def ho(self):
        return (self.h + 2 * self.pad - self.k) // self.stride + 1

    @property
    def wo(self):
        return (self.w + 2 * self.pad - self.k) // self.stride + 1

    def in_shape(self):
        return (self.h, self.w, self.cin)

    def out_shape(self):
        return (self.ho, self.wo, self.cout)

    def out_dim(self):
        return self.ho * self.wo * self.cout


@dataclass(frozen=True)
class MaxPool2:
    """2x2 max pooling with stride 2 on NHWC activations; no parameters."""
    c: int
    h: int
    w: int
    act: str = "none"
    kind: str = "pool"

    def param_shapes(self):
        return []

    def in_shape(self):
        return (self.h, self.w, self.c)

    def out_shape(self):
        return (self.h // 2, self.w // 2, self.c)

    def out_dim(self):
        return (self.h // 2) * (self.w // 2) * self.c


@dataclass(frozen=True)
class AvgPool:
    """Global average pooling: [positions, c] -> [c]; no parameters."""
    c: int
    tokens: int      # positions (H * W) that are averaged
    act: str = "none"
    kind: str = "avg"

    def param_shapes(self):
        return []

    def in_shape(self):
        return (self.tokens, self.c)

    def out_shape(self):
        return (self.c,)

    def out_dim(self):
        return self.c


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                     # "f32" or "bf16" (bf16 storage, fp32 master weights)
    stages: Tuple[tuple, ...]
    mb: int                        # samples per micro-batch
    n: int                         # micro-batches per mini-batch
    classes: int
    lr: float = 0.01
    momentum: float = 0.9
    lam: float = 0.1               # lambda of the significance function
    seed: int = GLOBAL_SEED

    @property
    def K(self) -> int:
        return len(self.stages)

    @property
    def in_dim(self) -> int:
        return self.stage_in_dim(0)

    def stage_in_dim(self, s: int) -> int:
        return int(np.prod(self.stages[s][0].in_shape()))

    def stage_out_dim(self, s: int) -> int:
        return self.stages[s][-1].out_dim()

    def param_count(self, s: int) -> int:
        return sum(int(np.prod(sh)) for l in self.stages[s] for sh in l.param_shapes())

    def cast(self, x: np.ndarray) -> np.ndarray:
        """Round to the workload's activation storage type; values stay fp64."""
        return round_bf16(x) if self.dtype == "bf16" else round_f32(x)


def mlp_small() -> Workload:
    """2-stage pipeline of an fp32 MLP 256-512-512-10 (ReLU), stage 0 = first two layers."""
    return Workload(
        name="mlp256_f32_k2", dtype="f32",
        stages=((Dense(256, 512, "relu"), Dense(512, 512, "relu")),
                (Dense(512, 10, "none"),)),
        mb=32, n=4, classes=10)


def mlp_wide(width: int = 4096, mb: int = 256, n: int = 8, classes: int = 1000,
             dtype: str = "bf16") -> Workload:
    """4-stage pipeline of an 8-layer GELU MLP, two layers per stage.

    Layers 1-7 are width->width with GELU, layer 8 is width->classes (logits).
    Reduced copies (smaller width / batch) keep the same structure for parity
    runs the CPU oracle can finish in seconds.
    """
    hidden = Dense(width, width, "gelu")
    stages = ((hidden, hidden), (hidden, hidden), (hidden, hidden),
              (hidden, Dense(width, classes, "none")))
    return Workload(name=f"mlp{width}_{dtype}_k4", dtype=dtype, stages=stages,
                    mb=mb, n=n, classes=classes)


def vgg_stage0(mb: int = 64, n: int = 4, size: int = 32, c1: int = 64, c2: int = 128, classes: int = 100,
               dtype: str = "bf16") -> Workload:
    """First stage of a VGG-16-style net on size x size x 3 images: conv3-c1, conv3-c1, pool, conv3-c2,
    conv3-c2, pool (3x3 convolutions, stride 1, pad 1, bias, ReLU), as stage 0 of a 4-stage pipeline.
    Only this stage is described; the other three are not built, so the workload is used stage-wise."""
    s0 = (Conv2d(3, c1, size, size, "relu"), Conv2d(c1, c1, size, size, "relu"), MaxPool2(c1, size, size),
          Conv2d(c1, c2, size // 2, size // 2, "relu"), Conv2d(c2, c2, size // 2, size // 2, "relu"),
          MaxPool2(c2, size // 2, size // 2))
    return Workload(name=f"vgg{size}_{c1}_{c2}_{dtype}_s0", dtype=dtype, stages=(s0, (), (), ()), mb=mb, n=n,
                    classes=classes)


def bottleneck_block(c: int, mid: int, h: int, w: int, act: str = "relu") -> tuple:
    """Identity bottleneck of a ResNet-50-style net on [h, w, c] images: 1x1 conv c->mid, BN, ReLU, 3x3 conv
    mid->mid, BN, ReLU, 1x1 conv mid->c, BN, add the block input, ReLU.  1x1 convolutions are per-position
    dense layers; NHWC images and [positions, channels] samples are the same memory.  `act` replaces the ReLUs
    (parity runs in bf16 use a smooth activation where they want the tight tolerance)."""
    t = h * w
    return (Residual(c, t, "begin"), Dense(c, mid, "none", tokens=t), BatchNorm(mid, t, act),
            Conv2d(mid, mid, h, w, "none"), BatchNorm(mid, t, act), Dense(mid, c, "none", tokens=t),
            BatchNorm(c, t, "none"), Residual(c, t, "add", act=act))


def bottleneck_down_block(cin: int, mid: int, cout: int, h: int, w: int, act: str = "relu") -> tuple:
    """First bottleneck of a group: [h, w, cin] -> [h/2, w/2, cout].  Main branch 1x1 conv cin->mid, BN, ReLU, 3x3
    conv mid->mid with stride 2, BN, ReLU, 1x1 conv mid->cout, BN; shortcut 1x1 conv cin->cout with stride 2
    (= subsampling, then a per-position dense layer), BN; sum, ReLU."""
    t, to = h * w, (h // 2) * (w // 2)
    return (Residual(cin, t, "begin"), Dense(cin, mid, "none", tokens=t), BatchNorm(mid, t, act),
            Conv2d(mid, mid, h, w, "none", stride=2), BatchNorm(mid, to, act), Dense(mid, cout, "none", tokens=to),
            BatchNorm(cout, to, "none"), ResidualSwap(cout, to, cin, t), Subsample2(cin, h, w),
            Dense(cin, cout, "none", tokens=to), BatchNorm(cout, to, "none"), Residual(cout, to, "add", act=act))


def bottleneck_stage(c: int = 1024, mid: int = 256, h: int = 4, w: int = 4, blocks: int = 5, mb: int = 128, n: int = 4,
                     dtype: str = "bf16", down: bool = False, act: str = "relu") -> Workload:
    """A bottleneck group of a ResNet-50-style net as an interior stage; the defaults are conv4_x on 64x64
    inputs (4x4 feature maps, 1024 channels).  down=True puts the group's first block in front -- from
    [2h, 2w, c/2] with stride 2 and a projection shortcut -- followed by `blocks` identity bottlenecks."""
    layers = tuple(l for _ in range(blocks) for l in bottleneck_block(c, mid, h, w, act))
    if down:
        layers = bottleneck_down_block(c // 2, mid, c, 2 * h, 2 * w, act) + layers
    tag = f"d{blocks}" if down else f"{blocks}"
    return Workload(name=f"bneck{c}x{tag}_{dtype}_s1", dtype=dtype, stages=((), layers, (), ()), mb=mb, n=n, classes=2)


def resnet_middle_stages(mb: int = 128, n: int = 4, dtype: str = "bf16") -> Workload:
    """The two middle stages of a 4-stage split of a ResNet-50-style net on 64x64 inputs: stage 1 = the conv3_x
    group ([16, 16, 256] -> [8, 8, 512], four bottlenecks with 128 middle channels), stage 2 = the conv4_x group
    ([8, 8, 512] -> [4, 4, 1024], six bottlenecks with 256 middle channels).  Stages 0 and 3 are not described."""
    conv3 = bottleneck_stage(c=512, mid=128, h=8, w=8, blocks=3, mb=mb, n=n, dtype=dtype, down=True).stages[1]
    conv4 = bottleneck_stage(c=1024, mid=256, h=4, w=4, blocks=5, mb=mb, n=n, dtype=dtype, down=True).stages[1]
    return Workload(name=f"resnet_mid_{dtype}", dtype=dtype, stages=((), conv3, conv4, ()), mb=mb, n=n, classes=2)


def bottleneck_proj_block(cin: int, mid: int, cout: int, h: int, w: int, act: str = "relu") -> tuple:
    """First bottleneck of a group that keeps the image size (conv2_x): [h, w, cin] -> [h, w, cout].  Main branch 1x1
    conv cin->mid, BN, ReLU, 3x3 conv mid->mid, BN, ReLU, 1x1 conv mid->cout, BN; shortcut 1x1 conv cin->cout, BN; sum,
    ReLU."""
    t = h * w
    return (Residual(cin, t, "begin"), Dense(cin, mid, "none", tokens=t), BatchNorm(mid, t, act),
            Conv2d(mid, mid, h, w, "none"), BatchNorm(mid, t, act), Dense(mid, cout, "none", tokens=t),
            BatchNorm(cout, t, "none"), ResidualSwap(cout, t, cin, t),
            Dense(cin, cout, "none", tokens=t), BatchNorm(cout, t, "none"), Residual(cout, t, "add", act=act))


def resnet_stem_stage(size: int = 64, c: int = 64, mid: int = 64, cout: int = 256, blocks: int = 2, act: str = "relu") -> tuple:
    """Stage 0 of the 4-stage split: 7x7 stride-2 convolution 3->c, BN, ReLU, 2x2 max pooling (size -> size/4), then
    the conv2_x group: a projection bottleneck c->cout and `blocks` identity bottlenecks, `mid` middle channels."""
    h = size // 4
    stem = (Conv2d(3, c, size, size, "none", k=7, stride=2, pad=3), BatchNorm(c, (size // 2) ** 2, act),
            MaxPool2(c, size // 2, size // 2))
    return stem + bottleneck_proj_block(c, mid, cout, h, h, act) + tuple(
        l for _ in range(blocks) for l in bottleneck_block(cout, mid, h, h, act))


def resnet_head_stage(c: int = 2048, mid: int = 512, h: int = 2, blocks: int = 2, classes: int = 200, act: str = "relu") -> tuple:
    """Stage 3 of the 4-stage split: the conv5_x group ([2h, 2h, c/2] -> [h, h, c]: a stride-2 bottleneck with
    projection shortcut and `blocks` identity bottlenecks), global average pooling, and the classifier c -> classes."""
    return (bottleneck_down_block(c // 2, mid, c, 2 * h, 2 * h, act) +
            tuple(l for _ in range(blocks) for l in bottleneck_block(c, mid, h, h, act)) +
            (AvgPool(c, h * h), Dense(c, classes, "none")))


def resnet_stages(mb: int = 128, n: int = 4, dtype: str = "bf16", scale: int = 1, size: int = 64, classes: int = 200,
                  act: str = "relu", identity: tuple = (2, 3, 5, 2)) -> Workload:
    """All four stages of a ResNet-50-style bottleneck net on size x size x 3 images: {stem, conv2_x}, {conv3_x},
    {conv4_x}, {conv5_x, average pooling, classifier}.  scale divides every channel count and `identity` gives the
    identity bottlenecks behind the first (projection) bottleneck of each group -- reduced copies the CPU oracle
    finishes in seconds keep the structure: strides, projection shortcuts, 3 + 4 + 6 + 3 bottlenecks by default."""
    c = 64 // scale
    q = size // 4
    s0 = resnet_stem_stage(size, c, c, 4 * c, identity[0], act)
    s1 = bottleneck_down_block(4 * c, 2 * c, 8 * c, q, q, act) + tuple(
        l for _ in range(identity[1]) for l in bottleneck_block(8 * c, 2 * c, q // 2, q // 2, act))
    s2 = bottleneck_down_block(8 * c, 4 * c, 16 * c, q // 2, q // 2, act) + tuple(
        l for _ in range(identity[2]) for l in bottleneck_block(16 * c, 4 * c, q // 4, q // 4, act))
    s3 = resnet_head_stage(32 * c, 8 * c, q // 8, identity[3], classes, act)
    tag = "" if tuple(identity) == (2, 3, 5, 2) else "_i" + "".join(str(i) for i in identity)
    return Workload(name=f"resnet{size}_c{c}{tag}_{dtype}_k4", dtype=dtype, stages=(s0, s1, s2, s3), mb=mb, n=n,
                    classes=classes)


def transformer_block(d: int, heads: int, ffn: int, tokens: int) -> tuple:
    """Pre-norm decoder block: x + proj(attn(qkv(LN(x)))), then x + ffn2(gelu(ffn1(LN(x))))."""
    return (Residual(d, tokens, "begin"), LayerNorm(d, tokens), Dense(d, 3 * d, "none", tokens=tokens),
            Attention(d, heads, tokens), Dense(d, d, "none", tokens=tokens), Residual(d, tokens, "add"),
            Residual(d, tokens, "begin"), LayerNorm(d, tokens), Dense(d, ffn, "gelu", tokens=tokens),
            Dense(ffn, d, "none", tokens=tokens), Residual(d, tokens, "add"))


def transformer_stage(d: int = 2048, heads: int = 16, ffn: int = 8192, tokens: int = 1024, layers: int = 4, mb: int = 8,
                      n: int = 4, dtype: str = "bf16") -> Workload:
    """An interior stage of a decoder-only transformer: `layers` blocks on [tokens, d] hidden states, as stage 1
    of a 4-stage pipeline.  Only this stage is described."""
    blocks = tuple(l for _ in range(layers) for l in transformer_block(d, heads, ffn, tokens))
    return Workload(name=f"tfm{d}x{layers}_{dtype}_s1", dtype=dtype, stages=((), blocks, (), ()), mb=mb, n=n, classes=2)


def with_lambda(w: Workload, lam: float) -> Workload:
    return replace(w, lam=lam)


# ---------------------------------------------------------------------------
# seeded tensors
# ---------------------------------------------------------------------------

def init_params(w: Workload, s: int) -> List[np.ndarray]:
    """Initial parameters of stage s as a flat list [W0, b0, W1, b1, ...].

    Weights are Kaiming-normal on fan-in with gain sqrt(2): N(0, 2/fan_in);
    biases start at zero.  Values are rounded to fp32 (the master precision on
    the GPU) and returned as fp64 arrays holding those fp32 values.
    """
    out = []
    for li, layer in enumerate(w.stages[s]):
        if not layer.param_shapes():
            continue
        wshape, bshape = layer.param_shapes()
        if layer.kind in ("ln", "bn"):                       # scale 1, shift 0
            out.append(np.ones(wshape, dtype=np.float64))
            out.append(np.zeros(bshape, dtype=np.float64))
            continue
        fan_in = int(np.prod(wshape[1:]))
        W = _normal(f"{w.name}/s{s}/l{li}/W", wshape, std=float(np.sqrt(2.0 / fan_in)), seed=w.seed)
        out.append(round_f32(W))
        out.append(np.zeros(bshape, dtype=np.float64))
    return out


def minibatch_input(w: Workload, j: int) -> np.ndarray:
    """Network input of mini-batch j: [n*mb, in_dim], N(0,1), cast to storage type."""
    x = _normal(f"{w.name}/x/{j}", (w.n * w.mb, w.in_dim), seed=w.seed)
    return w.cast(x)


def minibatch_labels(w: Workload, j: int) -> np.ndarray:
    return _labels(f"{w.name}/y/{j}", w.n * w.mb, w.classes, seed=w.seed)


def stage_input(w: Workload, s: int, j: int) -> np.ndarray:
    """Synthetic input of an interior stage timed on its own: N(0,1)."""
    x = _normal(f"{w.name}/s{s}/x/{j}", (w.n * w.mb,) + tuple(w.stages[s][0].in_shape()), seed=w.seed)
    return w.cast(x)


def stage_upstream_grad(w: Workload, s: int, j: int, mean_loss: bool = False) -> np.ndarray:
    """Synthetic gradient w.r.t. the output of stage s: N(0,1)/sqrt(out_dim), a sample's gradient has norm ~ 1.
    mean_loss: the same draw scaled like the gradient of a loss AVERAGED over the mini-batch's n*mb samples
    (a sample's gradient has norm ~ 1/(n*mb), as (softmax - onehot)/(n*mb) has at the last stage)."""
    d = w.stage_out_dim(s)
    std = 1.0 / np.sqrt(d)
    if mean_loss:
        std /= w.n * w.mb
    g = _normal(f"{w.name}/s{s}/dy/{j}", (w.n * w.mb,) + tuple(w.stages[s][-1].out_shape()), std=float(std), seed=w.seed)
    return w.cast(g)
