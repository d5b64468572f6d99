"""Seeded synthetic inputs for the eleven benchmark layer shapes (and ad-hoc shapes for tests).

This module holds data and random-number recipes only -- none of the layer's arithmetic -- so the
GPU tests, the benchmark and the CPU checker can all draw identical bits from it.  The output
sizes below are written out as data (they are the sizes the benchmark configurations chain
through: 28->24, 12->8, 84->20->9->7, 227->55, ...), not computed here.

Stand-ins: the shapes are those of digit-like 28x28x1, small-image 32x32x3, large-image
227x227x3 and stacked-frame 84x84x4 workloads; the values are the distributions the benchmark
configurations prescribe (no dataset is used).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

BASE_SEED = 1810_02272 * 10


@dataclass(frozen=True)
class Layer:
    name: str
    config: int          # index into the benchmark configuration list
    n: int
    c: int
    hw: int              # square input
    k: int               # num_output
    kernel: int
    stride: int
    pad: int
    group: int
    out_hw: int          # square output (data, see module docstring)
    x_dist: str          # "uniform01" or "normal"
    w_dist: str          # "xavier" or "gauss0.01"
    dy_std: float

    @property
    def x_shape(self):
        return (self.n, self.c, self.hw, self.hw)

    @property
    def w_shape(self):
        return (self.k, self.c // self.group, self.kernel, self.kernel)

    @property
    def y_shape(self):
        return (self.n, self.k, self.out_hw, self.out_hw)

    @property
    def flop_per_pass(self) -> int:
        """Multiply-adds x2 of one pass (forward; each backward pass has the same count)."""
        return 2 * self.n * self.k * (self.c // self.group) * self.kernel * self.kernel * self.out_hw * self.out_hw

    def params_dict(self) -> dict:
        return dict(n=self.n, c=self.c, h=self.hw, w=self.hw, num_output=self.k, kernel_h=self.kernel,
                    kernel_w=self.kernel, stride_h=self.stride, stride_w=self.stride, pad_h=self.pad, pad_w=self.pad,
                    dilation_h=1, dilation_w=1, group=self.group, bias_term=1)


# dy ~ N(0, 1e-2) is read as variance 1e-2, i.e. standard deviation 0.1.
LAYERS = [
    Layer("1.a", 0, 64, 1, 28, 20, 5, 1, 0, 1, 24, "uniform01", "xavier", 1.0),
    Layer("2.a", 1, 64, 20, 12, 50, 5, 1, 0, 1, 8, "uniform01", "xavier", 1.0),
    Layer("3.a", 2, 32, 4, 84, 32, 8, 4, 0, 1, 20, "uniform01", "gauss0.01", 0.1),
    Layer("3.b", 2, 32, 32, 20, 64, 4, 2, 0, 1, 9, "uniform01", "gauss0.01", 0.1),
    Layer("3.c", 2, 32, 64, 9, 64, 3, 1, 0, 1, 7, "uniform01", "gauss0.01", 0.1),
    Layer("4.a", 3, 100, 3, 32, 32, 5, 1, 2, 1, 32, "normal", "gauss0.01", 1.0),
    Layer("4.b", 3, 100, 32, 16, 32, 5, 1, 2, 1, 16, "normal", "gauss0.01", 1.0),
    Layer("4.c", 3, 100, 32, 8, 64, 5, 1, 2, 1, 8, "normal", "gauss0.01", 1.0),
    Layer("5.a", 4, 128, 3, 227, 96, 11, 4, 0, 1, 55, "normal", "gauss0.01", 0.1),
    Layer("5.b", 4, 128, 96, 27, 256, 5, 1, 2, 2, 27, "normal", "gauss0.01", 0.1),
    Layer("5.c", 4, 128, 256, 13, 384, 3, 1, 1, 1, 13, "normal", "gauss0.01", 0.1),
]
# Depthwise layers of a mobile-style network (one channel per group, 3x3, strides 1 and 2) at the
# resolutions such a network runs them; not part of the five benchmark configurations -- they
# exercise the thin-group (direct) kernels at a realistic size.
DW_LAYERS = [
    Layer("dw.a", 5, 64, 32, 112, 32, 3, 1, 1, 32, 112, "normal", "xavier", 1.0),
    Layer("dw.b", 5, 64, 64, 112, 64, 3, 2, 1, 64, 56, "normal", "xavier", 1.0),
    Layer("dw.c", 5, 64, 128, 56, 128, 3, 1, 1, 128, 56, "normal", "xavier", 1.0),
    Layer("dw.d", 5, 64, 256, 28, 256, 3, 1, 1, 256, 28, "normal", "xavier", 1.0),
    Layer("dw.e", 5, 64, 512, 14, 512, 3, 1, 1, 512, 14, "normal", "xavier", 1.0),
]
BY_NAME = {l.name: l for l in LAYERS + DW_LAYERS}


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def draw(shape, dist: str, seed: int, scale: float = 1.0) -> torch.Tensor:
    """fp32 CPU tensor from a named distribution with its own seed."""
    g = _gen(seed)
    if dist == "uniform01":
        return torch.rand(shape, generator=g, dtype=torch.float32)
    if dist == "normal":
        return torch.randn(shape, generator=g, dtype=torch.float32) * scale
    if dist == "uniform_pm":  # U[-scale, scale)
        return (torch.rand(shape, generator=g, dtype=torch.float32) * 2.0 - 1.0) * scale
    raise ValueError(dist)


def layer_inputs(layer: Layer, bias: str = "zero", n: int | None = None):
    """(x, w, b, dy) as fp32 CPU tensors.  bias: "zero" (benchmark) or "random" (parity, U[-0.1,0.1)).

    ``n`` draws only the first n images (x and dy are generated image-major, so a prefix of the
    full batch is bit-identical to the same images of the full draw).
    """
    idx = (LAYERS + DW_LAYERS).index(layer)
    seed = BASE_SEED + 1000 * idx
    nn = layer.n if n is None else n
    xs, ys = (nn,) + layer.x_shape[1:], (nn,) + layer.y_shape[1:]
    x = draw(xs, layer.x_dist, seed + 0)
    fan_in = (layer.c // layer.group) * layer.kernel * layer.kernel
    if layer.w_dist == "xavier":  # U[-a, a], a = sqrt(3 / fan_in)
        w = draw(layer.w_shape, "uniform_pm", seed + 1, math.sqrt(3.0 / fan_in))
    else:
        w = draw(layer.w_shape, "normal", seed + 1, 0.01)
    b = torch.zeros(layer.k, dtype=torch.float32) if bias == "zero" else draw((layer.k,), "uniform_pm", seed + 2, 0.1)
    dy = draw(ys, "normal", seed + 3, layer.dy_std)
    return x, w, b, dy


def random_inputs(x_shape, w_shape, y_shape, seed: int, bias: bool = True):
    """Inputs for an arbitrary shape (property tests): x, dy ~ N(0,1), w ~ N(0, 0.1), b ~ U[-1,1)."""
    x = draw(x_shape, "normal", seed)
    w = draw(w_shape, "normal", seed + 1, 0.1)
    b = draw((w_shape[0],), "uniform_pm", seed + 2, 1.0) if bias else None
    dy = draw(y_shape, "normal", seed + 3)
    return x, w, b, dy


# ---- InnerProduct layers that follow the convolution stacks above ----
# The fully connected layers of the network shape behind configuration 4 (256x6x6 = 9216 inputs ->
# 4096 -> 4096 -> 1000, ReLU after the first two) at its batch of 128, and of the small digit
# network behind configurations 0/1 (50x4x4 = 800 -> 500 with ReLU -> 10) at its batch of 64.
@dataclass(frozen=True)
class IpLayer:
    name: str
    m: int           # batch rows
    k: int           # inputs per row
    num_output: int
    relu: int

    @property
    def flop_per_pass(self) -> int:
        return 2 * self.m * self.k * self.num_output

    def params_dict(self, bias_term: int = 1) -> dict:
        return dict(m=self.m, k=self.k, num_output=self.num_output, bias_term=bias_term, relu=self.relu)


IP_LAYERS = [
    IpLayer("ip5.6", 128, 9216, 4096, 1),
    IpLayer("ip5.7", 128, 4096, 4096, 1),
    IpLayer("ip5.8", 128, 4096, 1000, 0),
    IpLayer("ip1.1", 64, 800, 500, 1),
    IpLayer("ip1.2", 64, 500, 10, 0),
]
IP_BY_NAME = {l.name: l for l in IP_LAYERS}


def ip_inputs(layer: IpLayer, bias: str = "zero"):
    """(x, w, b, dy) fp32 CPU tensors: x ~ N(0,1), w ~ N(0, 0.01^2), dy ~ N(0, 0.1^2) as for the
    convolution layers of configuration 4; bias zero (benchmark) or U[-0.1, 0.1) (parity)."""
    seed = BASE_SEED + 100000 + 1000 * IP_LAYERS.index(layer)
    x = draw((layer.m, layer.k), "normal", seed + 0)
    w = draw((layer.num_output, layer.k), "normal", seed + 1, 0.01)
    b = (torch.zeros(layer.num_output, dtype=torch.float32) if bias == "zero"
         else draw((layer.num_output,), "uniform_pm", seed + 2, 0.1))
    dy = draw((layer.m, layer.num_output), "normal", seed + 3, 0.1)
    return x, w, b, dy


def ip_random_inputs(m: int, k: int, num_output: int, seed: int, bias: bool = True):
    """Inputs for an arbitrary InnerProduct shape (property tests)."""
    x = draw((m, k), "normal", seed)
    w = draw((num_output, k), "normal", seed + 1, 0.1)
    b = draw((num_output,), "uniform_pm", seed + 2, 1.0) if bias else None
    dy = draw((m, num_output), "normal", seed + 3)
    return x, w, b, dy


# ---- policy-gradient batches (paper Appendix A / B) ----
def pg_batch(episodes: int, min_len: int, max_len: int, actions: int, seed: int):
    """A batch of finished episodes stored back to back, shaped like the pole-balancing task the
    paper describes (Appendix A step 5): a reward of 1 for every step but the last of an episode,
    0 for the step that ended it; lengths uniform in [min_len, max_len].  Returns fp32/int32 CPU
    tensors: offsets [episodes+1], reward [steps], aprob [steps] in (0,1), random [steps] in
    [0,1), logits [steps][actions] ~ N(0, 2^2), action [steps] uniform over the actions."""
    g = _gen(seed)
    lengths = torch.randint(min_len, max_len + 1, (episodes,), generator=g, dtype=torch.int64)
    offsets = torch.zeros(episodes + 1, dtype=torch.int64)
    offsets[1:] = torch.cumsum(lengths, 0)
    steps = int(offsets[-1])
    reward = torch.ones(steps, dtype=torch.float32)
    ends = offsets[1:][lengths > 0] - 1
    reward[ends] = 0.0
    aprob = torch.rand(steps, generator=g, dtype=torch.float32) * 0.98 + 0.01
    random = torch.rand(steps, generator=g, dtype=torch.float32)
    logits = torch.randn((steps, actions), generator=g, dtype=torch.float32) * 2.0
    action = torch.randint(0, actions, (steps,), generator=g, dtype=torch.int32)
    return offsets.to(torch.int32), reward, aprob, random, logits, action


# benchmark batch: 65536 episodes of 8..500 steps (about 16.6 M steps), 6 actions for the Softmax model
PG_BENCH = (65536, 8, 500, 6)
PG_SEED = BASE_SEED + 200000
