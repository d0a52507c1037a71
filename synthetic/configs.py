"""The workload shapes.  Layer shapes are the public AlexNet / VGG-16
classifier and conv4 dimensions; tensors are synthetic (dense normals), standing
in for the ImageNet-trained networks the paper measured."""
from dataclasses import dataclass, field
from typing import Tuple

import numpy as np

from .gen import normal_f32, to_bf16_bits


@dataclass(frozen=True)
class FcChain:
    name: str
    batch: int
    widths: Tuple[int, ...]          # n_0 .. n_L
    k: int                           # number of cuts, 2^k shards
    dtype: str                       # "f32" or "bf16"
    w_std: float
    seed: int
    relu: bool = True                # ReLU after every layer but the last

    @property
    def n_layers(self):
        return len(self.widths) - 1

    def act(self, layer):            # layer in 1..L
        return 1 if (self.relu and layer < self.n_layers) else 0

    def flops(self):                 # fwd + bwd, 3 GEMMs per layer
        return sum(6 * self.batch * self.widths[i] * self.widths[i + 1]
                   for i in range(self.n_layers))

    def _draw(self, stream, shape, std):
        v = normal_f32(self.seed, stream, shape, std)
        return to_bf16_bits(v) if self.dtype == "bf16" else v

    def x0(self):
        return self._draw(0, (self.batch, self.widths[0]), 1.0)

    def weight(self, layer):         # layer in 1..L, shape n_{l-1} x n_l
        return self._draw(100 + layer, (self.widths[layer - 1], self.widths[layer]), self.w_std)

    def grad_out(self):              # dC/dx_L
        return self._draw(1, (self.batch, self.widths[-1]), 1.0)


@dataclass(frozen=True)
class ConvLayer:
    name: str
    N: int
    C: int
    K: int
    H: int
    W: int
    R: int
    S: int
    pad: int
    k: int
    w_std: float
    seed: int
    dtype: str = "bf16"

    @property
    def P(self):
        return self.H + 2 * self.pad - self.R + 1

    @property
    def Q(self):
        return self.W + 2 * self.pad - self.S + 1

    def flops(self):
        return 6 * self.N * self.P * self.Q * self.K * self.C * self.R * self.S

    def _draw(self, stream, shape, std):
        v = normal_f32(self.seed, stream, shape, std)
        return to_bf16_bits(v) if self.dtype == "bf16" else v

    def x(self):                     # logical NCHW
        return self._draw(0, (self.N, self.C, self.H, self.W), 1.0)

    def weight(self):                # logical K C R S
        return self._draw(101, (self.K, self.C, self.R, self.S), self.w_std)

    def grad_out(self):              # logical N K P Q
        return self._draw(1, (self.N, self.K, self.P, self.Q), 1.0)


CONFIGS = {
    "tiny_mlp": FcChain("tiny_mlp", 32, (256, 512, 256, 10), 2, "f32", 0.02, 1001),
    "alexnet_fc": FcChain("alexnet_fc", 256, (9216, 4096, 4096, 1000), 3, "bf16", 0.01, 1002),
    "vgg16_fc": FcChain("vgg16_fc", 256, (25088, 4096, 4096, 1000), 3, "bf16", 0.005, 1003),
    "vgg16_conv4": ConvLayer("vgg16_conv4", 64, 512, 512, 28, 28, 3, 3, 1, 3, 0.02, 1004),
    "wide_mlp": FcChain("wide_mlp", 512, (8192,) * 9, 4, "bf16", 0.01, 1005),
}
