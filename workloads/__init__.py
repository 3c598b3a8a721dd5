"""Seeded synthetic inputs for the FF-INT8 layer-local train step.

This module holds only shapes and random-number recipes: none of the method's
arithmetic (no quantisation, no contraction, no loss).  It is the one piece of
code that both the CPU oracle's tests and the HIP path's tests/bench import,
so that the two sides are fed the same bytes.

The paper trains on MNIST (784-vectors) and CIFAR-10 (32x32x3 images)
(Table II).  Neither dataset is used here: the generators below stand in for
them with tensors of the same shapes and uniform[0,1) "pixel" statistics, and
build the positive / negative sets the way Section III describes (a one-hot
label written over the first ten input features: the true class for a positive
sample, a wrong class for a negative one).
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple

import numpy as np

NUM_CLASSES = 10


@dataclasses.dataclass(frozen=True)
class Layer:
    """One FF layer.  kind 'dense': in_features -> out_features.
    kind 'conv': NHWC, H x W x C_in -> H_out x W_out x C_out, square kernel.
    kind 'dwconv': depthwise convolution, one ks x ks filter per channel (C_in == C_out)."""
    kind: str
    in_features: int = 0
    out_features: int = 0
    H: int = 0
    W: int = 0
    C_in: int = 0
    C_out: int = 0
    ksize: int = 0
    stride: int = 1
    pad: int = 0
    relu: int = 1
    l2norm_out: int = 0
    # basic residual blocks: see the docstring of `res_stack`
    input_back: int = 0        # the layer input is the output of layer i-1-input_back
    role: str = "ff"           # 'ff' | 'proj' (1x1 projection branch of a down-sampling block)
    skip: str = "none"         # 'none' | 'identity' | 'projection'

    @property
    def H_out(self) -> int:
        return (self.H + 2 * self.pad - self.ksize) // self.stride + 1

    @property
    def W_out(self) -> int:
        return (self.W + 2 * self.pad - self.ksize) // self.stride + 1

    @property
    def K(self) -> int:
        """Reduction length of the forward contraction."""
        if self.kind == "dense":
            return self.in_features
        if self.kind == "dwconv":
            return self.ksize * self.ksize
        return self.ksize * self.ksize * self.C_in

    @property
    def N(self) -> int:
        return self.out_features if self.kind == "dense" else self.C_out

    @property
    def rows_per_sample(self) -> int:
        return 1 if self.kind == "dense" else self.H_out * self.W_out

    @property
    def terms_per_sample(self) -> int:
        """Number of activities summed into one sample's goodness."""
        return self.rows_per_sample * self.N

    @property
    def in_elems_per_sample(self) -> int:
        return self.in_features if self.kind == "dense" else self.H * self.W * self.C_in

    @property
    def weight_shape(self) -> Tuple[int, ...]:
        if self.kind == "dense":
            return (self.out_features, self.in_features)
        if self.kind == "dwconv":
            return (self.C_out, self.ksize, self.ksize)
        return (self.C_out, self.ksize, self.ksize, self.C_in)

    @property
    def fan_in(self) -> int:
        return self.K


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    layers: Tuple[Layer, ...]
    batch: int                 # samples per pass (positive == negative)
    input_dist: str            # 'uniform_onehot' | 'normal'
    theta: float = 2.0         # Section V-A
    lam: float = 0.0           # look-ahead coefficient used for the bench / parity run
    lr: float = 0.01
    weight_seed: int = 0
    data_seed: int = 1
    sr_seed: int = 2           # stochastic-rounding seed


def mlp(widths: List[int], l2norm: bool) -> Tuple[Layer, ...]:
    out = []
    for i in range(len(widths) - 1):
        last = i == len(widths) - 2
        out.append(Layer("dense", in_features=widths[i], out_features=widths[i + 1],
                         l2norm_out=int(l2norm and not last)))
    return tuple(out)


def conv_stack(channels: List[int], h: int, w: int) -> Tuple[Layer, ...]:
    return tuple(Layer("conv", H=h, W=w, C_in=channels[i], C_out=channels[i + 1],
                       ksize=3, stride=1, pad=1) for i in range(len(channels) - 1))


def res_stack(stem_out: int, stages: List[Tuple[int, int, int]], h: int, w: int, c_in: int = 3) -> Tuple[Layer, ...]:
    """Stem conv3x3 + basic residual blocks.  stages: (channels, first stride, blocks).
    A block is conv1 (3x3, stride s) and conv2 (3x3), the second one producing the block output
    relu(conv2 + skip); skip is the block input (identity) or, when the shape changes, a 1x1 stride-s
    projection of it, which is listed first: [proj, conv1 (input_back=1), conv2 (skip='projection')]."""
    layers = [Layer("conv", H=h, W=w, C_in=c_in, C_out=stem_out, ksize=3, stride=1, pad=1)]
    c = stem_out
    for (c_out, stride, blocks) in stages:
        for b in range(blocks):
            s = stride if b == 0 else 1
            ho, wo = (h + 2 - 3) // s + 1, (w + 2 - 3) // s + 1
            change = s != 1 or c != c_out
            if change:
                layers.append(Layer("conv", H=h, W=w, C_in=c, C_out=c_out, ksize=1, stride=s, pad=0, relu=0, role="proj"))
            layers.append(Layer("conv", H=h, W=w, C_in=c, C_out=c_out, ksize=3, stride=s, pad=1,
                                input_back=1 if change else 0))
            layers.append(Layer("conv", H=ho, W=wo, C_in=c_out, C_out=c_out, ksize=3, stride=1, pad=1,
                                skip="projection" if change else "identity"))
            c, h, w = c_out, ho, wo
    return tuple(layers)


def bottleneck_stack(stem_out: int, blocks: List[Tuple[int, int, int]], h: int, w: int, c_in: int = 3) -> Tuple[Layer, ...]:
    """Stem conv3x3 + inverted bottlenecks without skip connections.  blocks: (expansion, C_out, stride):
    conv1x1 C -> t*C, depthwise 3x3 (stride s), conv1x1 t*C -> C_out."""
    layers = [Layer("conv", H=h, W=w, C_in=c_in, C_out=stem_out, ksize=3, stride=1, pad=1)]
    c = stem_out
    for (t, c_out, s) in blocks:
        layers.append(Layer("conv", H=h, W=w, C_in=c, C_out=t * c, ksize=1, stride=1, pad=0))
        layers.append(Layer("dwconv", H=h, W=w, C_in=t * c, C_out=t * c, ksize=3, stride=s, pad=1))
        h, w = (h + 2 - 3) // s + 1, (w + 2 - 3) // s + 1
        layers.append(Layer("conv", H=h, W=w, C_in=t * c, C_out=c_out, ksize=1, stride=1, pad=0))
        c = c_out
    return tuple(layers)


def workload(name: str) -> Workload:
    """The benchmark configurations (shapes only; all data is synthetic)."""
    if name == "cfg1":   # small MLP, latency-bound
        return Workload("cfg1", mlp([784, 500, 500], False), 64, "uniform_onehot", lam=0.0)
    if name == "cfg2":   # MLP with look-ahead and L2-normalised hand-off
        return Workload("cfg2", mlp([784, 2000, 2000, 2000, 2000], True), 1024, "uniform_onehot", lam=0.05)
    if name == "cfg3":   # small CNN, conv3x3 3->64->128->256 at 32x32
        return Workload("cfg3", conv_stack([3, 64, 128, 256], 32, 32), 256, "uniform_onehot", lam=0.0)
    if name == "cfg4_plain":
        # The 3x3 convolutions of a ResNet-18-shaped stack on 32x32x3 images (stem + 4 stages of 64/128/256/512
        # channels, two basic blocks each, stride 2 at the start of stages 2-4), run as a plain sequence: the
        # residual additions and the three 1x1 projection branches are left out (not built).
        layers, c_in, hw = [], 3, 32
        plan = [(64, 1)] + [(64, 1)] * 4 + [(128, 2)] + [(128, 1)] * 3 + [(256, 2)] + [(256, 1)] * 3 + [(512, 2)] + [(512, 1)] * 3
        for c_out, stride in plan:
            layers.append(Layer("conv", H=hw, W=hw, C_in=c_in, C_out=c_out, ksize=3, stride=stride, pad=1))
            c_in, hw = c_out, (hw + 2 - 3) // stride + 1
        return Workload("cfg4_plain", tuple(layers), 256, "uniform_onehot", lam=0.05)
    if name == "cfg4":
        # ResNet-18-shaped: stem + 4 stages x 2 basic blocks (64/128/256/512 channels, 32 -> 16 -> 8 -> 4 pixels):
        # 17 conv3x3 + 3 conv1x1 projections, every convolution an FF layer (the projections share their block's loss)
        return Workload("cfg4", res_stack(64, [(64, 1, 2), (128, 2, 2), (256, 2, 2), (512, 2, 2)], 32, 32), 256,
                        "uniform_onehot", lam=0.05)
    if name == "tiny_res":   # stem 3->16 at 8x16, an identity block, a down-sampling block with projection
        return Workload("tiny_res", res_stack(16, [(16, 1, 1), (32, 2, 1)], 8, 16), 6, "uniform_onehot", lam=0.05)
    if name == "mbv2_like":
        # 1x1-heavy stack with depthwise 3x3 convolutions, shaped like the first stages of a MobileNet-V2 on
        # 32x32x3 images (Table II lists such networks): stem 32, then (t, c, s) = (1,16,1), (6,24,1), (6,24,1), (6,32,2), (6,32,1)
        return Workload("mbv2_like", bottleneck_stack(32, [(1, 16, 1), (6, 24, 1), (6, 24, 1), (6, 32, 2), (6, 32, 1)], 32, 32),
                        256, "uniform_onehot", lam=0.05)
    if name == "tiny_dw":   # stem 3->16 at 8x12, two bottlenecks (the second with stride 2)
        return Workload("tiny_dw", bottleneck_stack(16, [(2, 16, 1), (3, 20, 2)], 8, 12), 5, "uniform_onehot", lam=0.05)
    if name == "tiny_cnn_head":   # two 3x3 convolutions at 8x12, flatten, two dense layers (L2-normalised hand-off)
        convs = conv_stack([3, 16, 16], 8, 12)
        return Workload("tiny_cnn_head", convs + (Layer("dense", in_features=8 * 12 * 16, out_features=40, l2norm_out=1),
                                                   Layer("dense", in_features=40, out_features=24)), 6, "uniform_onehot", lam=0.05)
    if name == "cfg5":   # large-GEMM stress
        return Workload("cfg5", mlp([4096, 4096, 4096], False), 8192, "normal", lam=0.05)
    if name == "tiny":   # ragged shapes spanning tile tails, for quick parity tests
        return Workload("tiny", mlp([100, 72, 52], False), 24, "uniform_onehot", lam=0.25)
    if name == "tiny_l2":
        return Workload("tiny_l2", mlp([100, 72, 52, 36], True), 24, "uniform_onehot", lam=0.25)
    if name == "tiny_conv":     # C_in = 3 and 8: both layers take the explicit patch-matrix route
        return Workload("tiny_conv", conv_stack([3, 8, 16], 6, 11), 6, "uniform_onehot", lam=0.25)
    if name == "tiny_conv16":   # second and third layer run as implicit GEMM; 8x8 maps: 64 rows per sample
        return Workload("tiny_conv16", conv_stack([3, 16, 32, 16], 8, 12), 5, "uniform_onehot", lam=0.25)
    if name == "tiny_conv_s2":  # stride 2 and 1x1 layers, as a ResNet-shaped stack needs them
        layers = (Layer("conv", H=9, W=12, C_in=3, C_out=16, ksize=3, stride=1, pad=1),
                  Layer("conv", H=9, W=12, C_in=16, C_out=32, ksize=3, stride=2, pad=1),
                  Layer("conv", H=5, W=6, C_in=32, C_out=48, ksize=1, stride=2, pad=0),
                  Layer("conv", H=3, W=3, C_in=48, C_out=16, ksize=1, stride=1, pad=0))
        return Workload("tiny_conv_s2", layers, 7, "uniform_onehot", lam=0.25)
    raise KeyError(name)


def scaled(w: Workload, batch: int) -> Workload:
    """Same network, smaller batch (used for the bounded CPU-baseline sample)."""
    return dataclasses.replace(w, batch=batch, name=f"{w.name}@B{batch}")


def kaiming_uniform(shape: Tuple[int, ...], fan_in: int, rng: np.random.Generator) -> np.ndarray:
    """U(-sqrt(6/fan_in), +sqrt(6/fan_in)) in fp32."""
    bound = np.sqrt(6.0 / fan_in)
    return rng.uniform(-bound, bound, size=shape).astype(np.float32)


def make_weights(w: Workload) -> List[np.ndarray]:
    rng = np.random.default_rng(w.weight_seed)
    return [kaiming_uniform(l.weight_shape, l.fan_in, rng) for l in w.layers]


def _overlay(x: np.ndarray, labels: np.ndarray, first: Layer) -> None:
    """Write the one-hot label over the first ten features (dense) or the first ten
    pixels of channel 0 (conv, NHWC: h=0, w=0..9)."""
    B = x.shape[0]
    onehot = np.zeros((B, NUM_CLASSES), dtype=np.float32)
    onehot[np.arange(B), labels] = 1.0
    if first.kind == "dense":
        x[:, :NUM_CLASSES] = onehot
    else:
        x[:, 0, :NUM_CLASSES, 0] = onehot


def make_inputs(w: Workload, batch: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (x_pos, x_neg), fp32, shape [B, in_features] or [B, H, W, C_in]."""
    B = w.batch if batch is None else batch
    first = w.layers[0]
    shape = (B, first.in_features) if first.kind == "dense" else (B, first.H, first.W, first.C_in)
    rng = np.random.default_rng(w.data_seed)
    if w.input_dist == "normal":
        x_pos = rng.standard_normal(size=shape, dtype=np.float32)
        x_neg = rng.standard_normal(size=shape, dtype=np.float32)
        return x_pos, x_neg
    base = rng.random(size=shape, dtype=np.float32)
    labels = rng.integers(0, NUM_CLASSES, size=B)
    wrong = (labels + rng.integers(1, NUM_CLASSES, size=B)) % NUM_CLASSES
    x_pos = base.copy()
    x_neg = base.copy()
    _overlay(x_pos, labels, first)
    _overlay(x_neg, wrong, first)
    return x_pos, x_neg
