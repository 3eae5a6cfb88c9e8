"""Seeded synthetic inputs for the 4-bit linear-layer path.

This module only draws random tensors with the shapes and value distributions
of the paper's two deployed workloads (the Llama-2-7B backbone of the VLA
policy, Sec. 5.4 "Robot Manipulation", and the ResNet encoder of the driving
policy, Sec. 5.4 "Autonomous Driving").  It holds none of the method's
arithmetic: no quantiser, no packing, no matmul.  The only numeric helper is
the float32 -> bfloat16 storage conversion of the activations, which is an
input format, not a step of the method.

Both the CPU oracle's tests and the GPU path's tests draw from here so that
the two sides see bit-identical inputs.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

# ---------------------------------------------------------------------------
# shapes
# ---------------------------------------------------------------------------

# (name, N, K) of the four linears of one Llama-2-7B decoder layer, with the
# Q/K/V and gate/up projections fused along N.
LLAMA7B_LINEARS: Tuple[Tuple[str, int, int], ...] = (
    ("qkv", 12288, 4096),
    ("out", 4096, 4096),
    ("gate_up", 22016, 4096),
    ("down", 4096, 11008),
)
LLAMA7B_LAYERS = 32
LLAMA7B_GROUP = 128


@dataclass(frozen=True)
class ConvShape:
    """One convolution of the ResNet-34 body as an implicit GEMM."""
    name: str
    B: int
    H: int       # input height
    W: int       # input width
    Cin: int
    Cout: int
    KH: int
    KW: int
    stride: int
    pad: int

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad - self.KH) // self.stride + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad - self.KW) // self.stride + 1

    @property
    def M(self) -> int:
        return self.B * self.OH * self.OW

    @property
    def N(self) -> int:
        return self.Cout

    @property
    def K(self) -> int:
        return self.KH * self.KW * self.Cin

    @property
    def ops(self) -> int:
        return 2 * self.M * self.N * self.K


def resnet34_convs(batch: int = 32, image: int = 224) -> List[ConvShape]:
    """All convolutions after the stem of a ResNet-34 for a square input.

    Stage widths 64/128/256/512 with 3/4/6/3 basic blocks (two 3x3 convs
    each); the first block of stages 2-4 has stride 2 and a 1x1 stride-2
    projection on the shortcut.  The stem (7x7/2 conv + 3x3/2 max-pool)
    only fixes the spatial size entering stage 1: image/4.
    Returns 32 3x3 convs + 3 1x1 convs = 35 calls, in network order.
    """
    widths = (64, 128, 256, 512)
    blocks = (3, 4, 6, 3)
    hw = image // 4
    cin = widths[0]
    out: List[ConvShape] = []
    for si, (c, nb) in enumerate(zip(widths, blocks)):
        for bi in range(nb):
            stride = 2 if (si > 0 and bi == 0) else 1
            tag = f"s{si + 1}.b{bi}"
            out.append(ConvShape(f"{tag}.conv1", batch, hw, hw, cin, c, 3, 3, stride, 1))
            if stride == 2:
                out.append(ConvShape(f"{tag}.down", batch, hw, hw, cin, c, 1, 1, 2, 0))
                hw //= 2
            out.append(ConvShape(f"{tag}.conv2", batch, hw, hw, c, c, 3, 3, 1, 1))
            cin = c
    return out


# ---------------------------------------------------------------------------
# storage-format helpers (bf16 is how the activations are handed over)
# ---------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------------------
# generators
# ---------------------------------------------------------------------------

def seed_for(config: int, item: int, stream: int) -> int:
    """Seed = 1000*config + 10*(shape or layer index) + stream id."""
    return 1000 * int(config) + 10 * int(item) + int(stream)


def _normal_f32(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def llm_weight(N: int, K: int, seed: int, std: float = 0.02,
               outlier_frac: float = 0.0, outlier_gain: float = 20.0) -> np.ndarray:
    """fp32 [N, K] ~ N(0, std^2); ceil(outlier_frac*K) input channels
    (columns, chosen by a seeded permutation) are multiplied by outlier_gain,
    standing in for the salient channels of an activation-aware quantiser."""
    rng = np.random.default_rng(seed)
    w = _normal_f32(rng, (N, K), std)
    if outlier_frac > 0.0:
        n_out = int(math.ceil(outlier_frac * K))
        cols = rng.permutation(K)[:n_out]
        w[:, cols] *= np.float32(outlier_gain)
    return w


def llm_activation_bf16(M: int, K: int, seed: int, outlier_frac: float = 0.0,
                        outlier_gain: float = 10.0) -> np.ndarray:
    """bf16 bit patterns [M, K] of N(0,1) draws; ceil(outlier_frac*K) columns
    (seeded, independent of the weight outliers) multiplied by outlier_gain
    before the bf16 rounding."""
    rng = np.random.default_rng(seed)
    x = _normal_f32(rng, (M, K), 1.0)
    if outlier_frac > 0.0:
        n_out = int(math.ceil(outlier_frac * K))
        cols = rng.permutation(K)[:n_out]
        x[:, cols] *= np.float32(outlier_gain)
    return f32_to_bf16_bits(x)


def lora_factors(N: int, K: int, r: int, seed: int, std_a: float = 0.02, std_b: float = 0.02):
    """bf16 bit patterns of the two low-rank factors of an adapter on an [N, K]
    linear: A [r, K] and B [N, r], both N(0, std^2) (a trained adapter: neither
    factor is zero)."""
    rng = np.random.default_rng(seed)
    a = _normal_f32(rng, (r, K), std_a)
    b = _normal_f32(rng, (N, r), std_b)
    return f32_to_bf16_bits(a), f32_to_bf16_bits(b)


def conv_weight(shape: ConvShape, seed: int) -> np.ndarray:
    """He-normal fp32 [Cout, KH, KW, Cin], std = sqrt(2 / fan_in)."""
    rng = np.random.default_rng(seed)
    std = math.sqrt(2.0 / shape.K)
    return _normal_f32(rng, (shape.Cout, shape.KH, shape.KW, shape.Cin), std)


def conv_activation(shape: ConvShape, seed: int) -> np.ndarray:
    """fp32 NHWC [B, H, W, Cin] = ReLU(N(0,1))."""
    rng = np.random.default_rng(seed)
    a = _normal_f32(rng, (shape.B, shape.H, shape.W, shape.Cin), 1.0)
    np.maximum(a, np.float32(0.0), out=a)
    return a


def conv_bias(shape: ConvShape, seed: int) -> np.ndarray:
    """fp32 [Cout] ~ N(0, 0.1^2), standing in for a folded batch-norm shift."""
    rng = np.random.default_rng(seed)
    return _normal_f32(rng, (shape.Cout,), 0.1)


def random_codes(shape, lo: int, hi: int, seed: int) -> np.ndarray:
    """Uniform integer codes in [lo, hi] (inclusive), int8."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int8)
