"""Seeded synthetic workloads shared by the tests, the smoke check and the benchmark.

This module holds NONE of the method's arithmetic: it only names layer shapes
and draws integer levels, scales and offsets from a seeded generator.  Both the
CPU oracle and the GPU library are fed the arrays produced here.

The five workload families mirror the layer shapes of the networks the paper
evaluates (CIFAR10 ResNet-20, ImageNet ResNet-18, plus ResNet-50 bottlenecks
and a fully-connected layer); the datasets and trained weights themselves are
not available and not needed: integer parity is exact on any levels and kernel
time does not depend on the level values.  The first and last network layers
are left out because the paper does not quantise them (App. B.3).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional

import numpy as np

BASE_SEED = 20200317


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int
    pad: int

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def int_macs(self) -> int:
        """Nominal integer multiply-accumulates (padded taps included)."""
        return self.N * self.OH * self.OW * self.K * self.C * self.R * self.S


@dataclass(frozen=True)
class Case:
    config: int
    layer_index: int
    layer: Layer
    k_w: int
    k_a: int
    act_dist: str = "uniform"        # "uniform" | "halfnormal"
    scale_mode: str = "layer_const"  # "layer_const" (0.1, no offset) | "layer_uniform" | "channel"

    @property
    def seed(self) -> int:
        pair = 4 * (self.k_w - 1) + (self.k_a - 1)
        if self.k_w > 4 or self.k_a > 4:            # five-bit pairs: numbered after the sixteen pairs of {1..4}^2
            pair = 16 + 5 * (self.k_w - 1) + (self.k_a - 1)
        return BASE_SEED + 100000 * self.config + 100 * self.layer_index + pair

    @property
    def binary_ops(self) -> int:
        """2 binary ops (AND + bitcount-add) per bit-plane pair per integer MAC:
        s*n*c_o*M*K ANDs and as many bitcount bits (Sec. 4.3 complexities)."""
        return 2 * self.layer.int_macs * self.k_w * self.k_a

    def with_batch(self, N: int) -> "Case":
        return replace(self, layer=replace(self.layer, N=N))

    @property
    def tag(self) -> str:
        L = self.layer
        return (f"cfg{self.config}.{self.layer_index}:{L.name}:N{L.N}C{L.C}H{L.H}W{L.W}K{L.K}"
                f"R{L.R}S{L.S}s{L.stride}p{L.pad}:w{self.k_w}a{self.k_a}")


ALL_BITS = [(kw, ka) for kw in range(1, 5) for ka in range(1, 5)]
# Pairs with a five-bit operand: the rest of the paper's search space {1, ..., 5} (Sec. 5).
FIVE_BITS = [(5, ka) for ka in range(1, 6)] + [(kw, 5) for kw in range(1, 5)]
PAPER_BITS = ALL_BITS + FIVE_BITS


def _conv3(name, N, C, HW, K, stride=1):
    return Layer(name, N, C, HW, HW, K, 3, 3, stride, 1)


def _conv1(name, N, C, HW, K):
    return Layer(name, N, C, HW, HW, K, 1, 1, 1, 0)


def cifar_resnet20_layers(N: int = 128) -> List[Layer]:
    L = [_conv3(f"s1.{i}", N, 16, 32, 16) for i in range(6)]
    L.append(_conv3("s2.down", N, 16, 32, 32, 2))
    L += [_conv3(f"s2.{i}", N, 32, 16, 32) for i in range(5)]
    L.append(_conv3("s3.down", N, 32, 16, 64, 2))
    L += [_conv3(f"s3.{i}", N, 64, 8, 64) for i in range(5)]
    return L


def resnet18_layers(N: int = 64) -> List[Layer]:
    return [
        _conv3("c64@56", N, 64, 56, 64),
        _conv3("c128@28", N, 128, 28, 128),
        _conv3("c256@14", N, 256, 14, 256),
        _conv3("c512@7", N, 512, 7, 512),
        _conv3("c64->128@56s2", N, 64, 56, 128, 2),
        _conv3("c128->256@28s2", N, 128, 28, 256, 2),
        _conv3("c256->512@14s2", N, 256, 14, 512, 2),
    ]


def resnet50_layers(N: int = 64) -> List[Layer]:
    return [
        _conv1("b1x1.256->64@56", N, 256, 56, 64),
        _conv3("b3x3.64->64@56", N, 64, 56, 64),
        _conv1("b1x1.64->256@56", N, 64, 56, 256),
        _conv1("b1x1.1024->256@14", N, 1024, 14, 256),
        _conv1("b1x1.256->1024@14", N, 256, 14, 1024),
    ]


def config_cases(config: int, N: Optional[int] = None) -> List[Case]:
    """Cases of workload family `config` (1..6); N overrides the batch size."""
    cases: List[Case] = []
    if config == 1:
        cases.append(Case(1, 0, _conv3("tiny", N or 1, 16, 8, 16), 2, 2))
    elif config == 2:
        rng = np.random.default_rng(BASE_SEED + 100000 * 2)
        for i, L in enumerate(cifar_resnet20_layers(N or 128)):
            kw, ka = (int(v) for v in rng.integers(1, 5, 2))
            cases.append(Case(2, i, L, kw, ka, "uniform", "layer_uniform"))
    elif config == 3:
        for i, L in enumerate(resnet18_layers(N or 64)):
            for kw, ka in ALL_BITS:
                cases.append(Case(3, i, L, kw, ka, "halfnormal", "layer_const"))
    elif config == 4:
        for i, L in enumerate(resnet50_layers(N or 64)):
            for kw, ka in [(2, 4), (3, 3), (4, 2)]:
                cases.append(Case(4, i, L, kw, ka, "uniform", "layer_const"))
    elif config == 5:
        L = _conv1("fc2048->1000", N or 1024, 2048, 1, 1000)
        for kw, ka in [(4, 4), (1, 1)]:
            cases.append(Case(5, 0, L, kw, ka, "uniform", "channel"))
    elif config == 6:
        # the ResNet-18-shaped layers of config 3 at the pairs with a five-bit operand
        for i, L in enumerate(resnet18_layers(N or 64)):
            for kw, ka in FIVE_BITS:
                cases.append(Case(6, i, L, kw, ka, "halfnormal", "layer_const"))
    else:
        raise ValueError("config must be 1..6")
    return cases


def draw_levels(rng, shape, bits: int, dist: str = "uniform") -> np.ndarray:
    """uint8 levels in [0, 2^bits - 1].  "halfnormal": |z|, z~N(0,1), clipped to
    alpha = 3 and mapped to the nearest level with round-half-up, the shape a
    ReLU'd, clipped and uniformly quantised activation has."""
    top = (1 << bits) - 1
    if dist == "uniform":
        return rng.integers(0, top + 1, size=shape, dtype=np.uint8)
    if dist == "halfnormal":
        alpha = 3.0
        x = np.minimum(np.abs(rng.standard_normal(size=shape, dtype=np.float32)), alpha) / alpha
        return np.floor(top * x + 0.5).astype(np.uint8)
    raise ValueError(dist)


def make_inputs(case: Case) -> dict:
    """Arrays for one case: a (NHWC uint8), q (KRSC uint8), scale, offset, per_channel."""
    L = case.layer
    rng = np.random.default_rng(case.seed)
    q = draw_levels(rng, (L.K, L.R, L.S, L.C), case.k_w, "uniform")
    a = draw_levels(rng, (L.N, L.H, L.W, L.C), case.k_a, case.act_dist)
    if case.scale_mode == "layer_const":
        scale = np.array([0.1], dtype=np.float32)
        offset = None
        per_channel = False
    elif case.scale_mode == "layer_uniform":
        scale = rng.uniform(0.01, 0.2, size=1).astype(np.float32)
        offset = None
        per_channel = False
    elif case.scale_mode == "channel":
        scale = rng.uniform(0.01, 0.2, size=L.K).astype(np.float32)
        offset = rng.normal(0.0, 0.1, size=L.K).astype(np.float32)
        per_channel = True
    else:
        raise ValueError(case.scale_mode)
    return {"a": a, "q": q, "scale": scale, "offset": offset, "per_channel": per_channel}


def random_case(seed: int, N, C, H, W, K, R, S, stride, pad, k_w, k_a,
                per_channel=False, with_offset=False) -> dict:
    """Free-form seeded case for edge-shape tests (uniform levels)."""
    rng = np.random.default_rng(seed)
    q = draw_levels(rng, (K, R, S, C), k_w)
    a = draw_levels(rng, (N, H, W, C), k_a)
    n = K if per_channel else 1
    scale = rng.uniform(0.01, 0.2, size=n).astype(np.float32)
    offset = rng.normal(0.0, 0.1, size=n).astype(np.float32) if with_offset else None
    return {"a": a, "q": q, "scale": scale, "offset": offset, "per_channel": per_channel}


def _chain(layers: List[Layer], seed: int, max_bits: int = 5) -> dict:
    """A list of layers as ONE stack: layer i's re-quantised output is layer i+1's input (Eq. 1b-1c
    between the layers), signed weights (Eq. 1a), per-channel scale/offset as a merged batch
    normalisation would give them.  Returns the first layer's activation levels and, per layer, the
    weight levels, bitwidths, the next layer's activation bitwidth, alpha and the affine map.
    Scales follow a closed-form estimate of the accumulator's spread (independent uniform weight
    levels, activations around 45 % of their top level) so that the re-quantised levels use their
    whole range; no arithmetic of the method is involved."""
    rng = np.random.default_rng(seed)
    bits = [(int(rng.integers(1, max_bits + 1)), int(rng.integers(1, max_bits + 1))) for _ in layers]
    L0 = layers[0]
    out = {"a0": draw_levels(rng, (L0.N, L0.H, L0.W, L0.C), bits[0][1], "halfnormal"), "layers": []}
    for i, L in enumerate(layers):
        k_w, k_a = bits[i]
        k_next = bits[i + 1][1] if i + 1 < len(layers) else int(rng.integers(1, max_bits + 1))
        alpha = 6.0
        top_w, top_a = (1 << k_w) - 1, (1 << k_a) - 1
        sigma_w = np.sqrt((top_w * top_w + 2.0 * top_w) / 3.0)
        spread = np.sqrt(L.C * L.R * L.S) * sigma_w * 0.45 * top_a
        scale = (alpha / (2.0 * spread) * rng.uniform(0.7, 1.3, L.K)).astype(np.float32)
        offset = rng.normal(1.0, 0.5, L.K).astype(np.float32)
        out["layers"].append({"layer": L, "k_w": k_w, "k_a": k_a, "k_next": k_next, "alpha": alpha,
                              "q": draw_levels(rng, (L.K, L.R, L.S, L.C), k_w), "scale": scale, "offset": offset})
    return out


def resnet20_chain(N: int = 128, seed: int = BASE_SEED + 700000) -> dict:
    """The 18 ResNet-20-shaped layers of config 2 (CIFAR sizes) chained, bitwidths drawn from {1..5}."""
    return _chain(cifar_resnet20_layers(N), seed)


def resnet18_chain(N: int = 64, seed: int = BASE_SEED + 800000) -> dict:
    """The 3x3 convolutions of an ImageNet ResNet-18 body in network order (four per stage, the
    first of stages 2-4 with stride 2; shortcuts and the unquantised first/last layers left out),
    bitwidths drawn from {1..4} as in the headline workload."""
    L = resnet18_layers(N)          # s1: 64@56, 128@28, 256@14, 512@7; s2: 64->128, 128->256, 256->512
    order = [L[0]] * 4 + [L[4]] + [L[1]] * 3 + [L[5]] + [L[2]] * 3 + [L[6]] + [L[3]] * 3
    return _chain(order, seed, max_bits=4)
