"""Seeded synthetic inputs shaped like the layers the Tiled Bit Networks paper evaluates.

This module holds no arithmetic of the method itself: it only draws real weights
``W_real ~ N(0, 0.02)`` and activations ``X ~ N(0, 1)`` with
``numpy.random.default_rng(seed)``, rounds activations to bfloat16 where a
workload asks for it, and lists the layer shapes.  Both the GPU tests and the
CPU oracle tests take their inputs from here so that they see identical data.

The paper's datasets and trained weights are not available; these tensors stand
in for them (CNN, ViT / transformer, MLP and time-series layer shapes, Sections
"Experiments" and "Implementation" of the paper).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 240712075 * 10


@dataclass(frozen=True)
class LinearWorkload:
    name: str
    cfg: int            # index of the benchmark configuration this belongs to
    layer: int          # layer number inside the configuration (seeds differ per layer)
    M: int              # batch rows
    cin: int
    cout: int
    k: int              # tile repeats (compression factor)
    n_alpha: int        # 1 or k
    dtype: str          # "f32" or "bf16"

    @property
    def n(self) -> int:
        return self.cin * self.cout

    @property
    def p(self) -> int:
        return self.n // self.k


@dataclass(frozen=True)
class ConvWorkload:
    name: str
    cfg: int
    layer: int
    N: int
    C: int
    H: int
    W: int
    O: int
    kh: int
    kw: int
    stride: Tuple[int, int]
    pad: Tuple[int, int]
    k: int
    n_alpha: int
    dtype: str = "f32"

    @property
    def n(self) -> int:
        return self.O * self.C * self.kh * self.kw

    @property
    def p(self) -> int:
        return self.n // self.k


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to the float32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def weight_seed(cfg: int, layer: int) -> int:
    return BASE_SEED + cfg + 100 * layer


def input_seed(cfg: int, layer: int) -> int:
    return BASE_SEED + cfg + 100 * layer + 7


def draw_w_real(n: int, cfg: int, layer: int = 0, std: float = 0.02) -> np.ndarray:
    """Flat float32 real-valued weight tensor of n entries, N(0, std)."""
    rng = np.random.default_rng(weight_seed(cfg, layer))
    return (std * rng.standard_normal(n, dtype=np.float32)).astype(np.float32)


def draw_x(shape, cfg: int, layer: int = 0, dtype: str = "f32"):
    """Activations N(0,1).  Returns (values float32, bits) where ``bits`` is the uint16
    bfloat16 pattern array for dtype "bf16" (values are then the rounded numbers) and
    None for "f32"."""
    rng = np.random.default_rng(input_seed(cfg, layer))
    x = rng.standard_normal(shape, dtype=np.float32)
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x)
        return bf16_bits_to_f32(bits).reshape(shape), bits.reshape(shape)
    if dtype != "f32":
        raise ValueError("dtype must be 'f32' or 'bf16'")
    return x, None


# ---------------------------------------------------------------------------
# The benchmark configurations.
# ---------------------------------------------------------------------------
CFG1 = LinearWorkload("cfg1_linear_256x256_k4_b8", 1, 0, 8, 256, 256, 4, 1, "f32")

CFG2 = (
    LinearWorkload("cfg2_vit_fc1_384_1536_k4", 2, 0, 197 * 64, 384, 1536, 4, 1, "f32"),
    LinearWorkload("cfg2_vit_fc2_1536_384_k4", 2, 1, 197 * 64, 1536, 384, 4, 1, "f32"),
)

CFG3 = ConvWorkload("cfg3_conv3x3_256_14x14_k8_b128", 3, 0, 128, 256, 14, 14, 256, 3, 3, (1, 1), (1, 1), 8, 1)
# the same convolution with a tile that does not hold whole filters (85 1/3 filters per tile)
CFG3_MISALIGNED = ConvWorkload("cfg3m_conv3x3_256_14x14_k3_b128", 3, 1, 128, 256, 14, 14, 256, 3, 3,
                               (1, 1), (1, 1), 3, 3)

CFG4 = (
    LinearWorkload("cfg4_linear_4096_k8_b1", 4, 0, 1, 4096, 4096, 8, 8, "bf16"),
    LinearWorkload("cfg4_linear_4096_k8_b16", 4, 0, 16, 4096, 4096, 8, 8, "bf16"),
)

# the shape the headline metric is quoted on
METRIC = LinearWorkload("metric_linear_4096_k8_b8192", 4, 0, 8192, 4096, 4096, 8, 8, "bf16")

CFG5 = tuple(
    LinearWorkload(f"cfg5_ffn_4096_16384_k{k}_b8192", 5, 0, 8192, 4096, 16384, k, k, "bf16")
    for k in (2, 4, 8, 16)
)
# in=3000: rows start at bit offsets that are not multiples of 32 and K is not a multiple of 32.
# k=6 is row-aligned (512 rows per tile); k=9 and k=5 put tile and alpha boundaries mid-row.
CFG5_MISALIGNED = tuple(
    LinearWorkload(f"cfg5m_3000_3072_k{k}_b8192", 5, 1, 8192, 3000, 3072, k, k, "bf16")
    for k in (6, 9, 5)
)

# small extra shapes from the paper's microcontroller MLP and time-series encoders
EXTRA = (
    LinearWorkload("mcu_mlp_784_128_k4", 6, 0, 1, 784, 128, 4, 4, "f32"),
    LinearWorkload("ts_encoder_512_512_k4", 6, 1, 96, 512, 512, 4, 1, "f32"),
    LinearWorkload("ts_encoder_128_512_k2", 6, 2, 96, 128, 512, 2, 1, "f32"),
)

# Shapes beyond the named configurations that the benchmark's table also times (same recipe, further layers of
# configurations 3 and 5): convolutions of the CNN section's networks at other map sizes, and a transformer's FFN
# down-projection (long rows) at a few hundred to a few thousand tokens.
CONV_MORE = (
    ConvWorkload("conv3x3_64_56x56_k4_b32", 3, 2, 32, 64, 56, 56, 64, 3, 3, (1, 1), (1, 1), 4, 1),
    ConvWorkload("conv3x3_64_56x56_k4_b32_bf16", 3, 2, 32, 64, 56, 56, 64, 3, 3, (1, 1), (1, 1), 4, 1, "bf16"),
    ConvWorkload("conv3x3_128_28x28_k4_b64", 3, 3, 64, 128, 28, 28, 128, 3, 3, (1, 1), (1, 1), 4, 1),
    ConvWorkload("conv3x3_64_112x112_k4_b8", 3, 4, 8, 64, 112, 112, 64, 3, 3, (1, 1), (1, 1), 4, 1),
    ConvWorkload("conv3x3_3_32x32_to64_k2_b128", 3, 5, 128, 3, 32, 32, 64, 3, 3, (1, 1), (1, 1), 2, 1),
    ConvWorkload("conv1x1_256_14x14_to1024_k8_b64_bf16", 3, 6, 64, 256, 14, 14, 1024, 1, 1, (1, 1), (0, 0), 8, 1, "bf16"),
    # a 7x7, stride 2 first layer (the networks of the CNN section leave it untiled; here it is tiled to time that window)
    ConvWorkload("conv7x7s2_3_224x224_to64_k4_b32", 3, 7, 32, 3, 224, 224, 64, 7, 7, (2, 2), (3, 3), 4, 1),
)

FFN_DOWN = tuple(LinearWorkload(f"ffn_down_16384_4096_k8_b{m}", 5, 10, m, 16384, 4096, 8, 8, "bf16") for m in (256, 512, 1024, 2048))

