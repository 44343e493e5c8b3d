"""The benchmark workloads as tables of layers (1-5: the headline set; 6: the language-model shape).

Shapes follow the paper's fine-tuning workloads (ResNet-18 / MobileNetV2 tails
of its ImageNet table, segmentation-sized maps, transformer linear layers);
ranks, spectra, noise level and step counts are the benchmark's own choices.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple


@dataclass(frozen=True)
class Layer:
    name: str
    dims: Tuple[int, ...]            # (B,C,H,W) or (B,N,D)
    ranks: Tuple[int, ...]
    dtype: str                       # "f32" | "bf16"  (dtype of A and grad_out)
    kind: str                        # "conv2d" | "linear"
    cout: int                        # C' or D_out
    k: int = 1                       # square kernel size (conv2d)
    stride: int = 1
    pad: int = 0
    dil: int = 1
    groups: int = 1
    alpha: float = 1.5               # core decay exponent (0 = plain Gaussian core)
    noise: float = 1e-3              # noise std after scaling the signal to unit RMS

    @property
    def out_hw(self) -> Tuple[int, int]:
        _, _, H, W = self.dims
        f = lambda n: (n + 2 * self.pad - self.dil * (self.k - 1) - 1) // self.stride + 1
        return f(H), f(W)

    @property
    def grad_out_shape(self) -> Tuple[int, ...]:
        if self.kind == "conv2d":
            Ho, Wo = self.out_hw
            return (self.dims[0], self.cout, Ho, Wo)
        return (self.dims[0], self.dims[1], self.cout)

    @property
    def dw_shape(self) -> Tuple[int, ...]:
        if self.kind == "conv2d":
            return (self.cout, self.dims[1] // self.groups, self.k, self.k)
        return (self.cout, self.dims[2])

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def act_bytes(self) -> int:
        n = 1
        for d in self.dims:
            n *= d
        return n * self.itemsize


@dataclass(frozen=True)
class Config:
    index: int
    name: str
    layers: Tuple[Layer, ...]
    steps: int                       # training steps with drift (1 = single step)
    theta: float = 0.02              # drift angle per step, radians


def _conv(name, dims, ranks, cout, k, alpha, noise=1e-3, groups=1):
    return Layer(name, dims, ranks, "f32", "conv2d", cout, k=k, stride=1, pad=(k - 1) // 2,
                 groups=groups, alpha=alpha, noise=noise)


CONFIGS: Dict[int, Config] = {
    1: Config(1, "exact-tucker-small", (
        _conv("c1", (8, 32, 16, 16), (4, 8, 6, 6), 32, 3, alpha=0.0, noise=1e-6),), steps=1),
    2: Config(2, "resnet18-tail-b64", (
        _conv("l4.0.in", (64, 256, 14, 14), (16, 32, 7, 7), 256, 3, alpha=1.5),
        _conv("l4.0.c2", (64, 512, 7, 7), (16, 48, 5, 5), 512, 3, alpha=1.5),
        _conv("l4.1.c1", (64, 512, 7, 7), (16, 48, 5, 5), 512, 3, alpha=1.5),
        _conv("l4.1.c2", (64, 512, 7, 7), (16, 48, 5, 5), 512, 3, alpha=1.5)), steps=50),
    3: Config(3, "mobilenetv2-tail-b128", (
        _conv("expand", (128, 160, 7, 7), (24, 40, 6, 6), 960, 1, alpha=1.5),
        _conv("dw", (128, 960, 7, 7), (24, 40, 6, 6), 960, 3, alpha=1.5, groups=960),
        _conv("project", (128, 960, 7, 7), (24, 40, 6, 6), 320, 1, alpha=1.5),
        _conv("head", (128, 320, 7, 7), (24, 40, 6, 6), 1280, 1, alpha=1.5)), steps=1),
    4: Config(4, "highres-conv", (
        _conv("hr56", (32, 128, 56, 56), (16, 32, 24, 24), 128, 3, alpha=1.0),
        _conv("hr64", (8, 256, 64, 64), (8, 48, 32, 32), 256, 3, alpha=1.0)), steps=20),
    5: Config(5, "vit-b-linear-bf16", (
        Layer("fc1", (64, 197, 768), (32, 64, 96), "bf16", "linear", 3072, alpha=1.2),
        Layer("fc2", (64, 197, 3072), (32, 64, 192), "bf16", "linear", 768, alpha=1.2)), steps=1),
    # The paper's language-model experiment in shape (its TinyLlama table: batch 8, up to 512 tokens, rank 20
    # on every mode, the batch mode capped by its size): the linear layers of one decoder block of a
    # 2048-wide model with a 5632-wide feed-forward, tiny ranks against a huge unfolding.
    6: Config(6, "llm-block-linear-bf16", (
        Layer("attn.q", (8, 512, 2048), (8, 20, 20), "bf16", "linear", 2048, alpha=1.2),
        Layer("attn.o", (8, 512, 2048), (8, 20, 20), "bf16", "linear", 2048, alpha=1.2),
        Layer("mlp.up", (8, 512, 2048), (8, 20, 20), "bf16", "linear", 5632, alpha=1.2),
        Layer("mlp.down", (8, 512, 5632), (8, 20, 20), "bf16", "linear", 2048, alpha=1.2)), steps=1),
}


def layers_of(cfg: int) -> Tuple[Layer, ...]:
    return CONFIGS[cfg].layers
