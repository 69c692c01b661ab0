"""Seeded synthetic convolution workloads.

Layer shapes and value distributions that stand in for the CNN layers the paper
evaluates (Section 5.1, "Set up": forward convolutions of ResNet-50 at mini-batch 28,
channel widths that are multiples of 16).  The paper runs on trained networks and real
images; convolution time does not depend on the values, so seeded random tensors of the
same shapes are used instead.

This module holds no convolution arithmetic: only shapes, seeds and random draws.  It is
the one module that both the CPU oracle's tests and the GPU path's tests import, so that
both sides see the very same input bits.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
import math

import numpy as np


@dataclass(frozen=True)
class ConvShape:
    """Problem sizes of one forward convolution (the loop bounds of the paper's Fig. 4)."""
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int = 1
    pad: int = 0
    name: str = ""

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def flops(self) -> int:
        """2*N*K*P*Q*C*R*S with the real channel count (the headline convention)."""
        return 2 * self.N * self.K * self.P * self.Q * self.C * self.R * self.S

    @property
    def flops_issued(self) -> int:
        """Same with C rounded up to the 16-wide channel block (work the matrix cores issue)."""
        c16 = -(-self.C // 16) * 16
        return 2 * self.N * self.K * self.P * self.Q * c16 * self.R * self.S

    def algorithmic_bytes(self, elem_size: int = 4) -> int:
        """Each of input, filter and output touched once (output is always fp32)."""
        c16 = -(-self.C // 16) * 16
        return (self.N * c16 * self.H * self.W * elem_size
                + self.K * c16 * self.R * self.S * elem_size
                + self.N * self.K * self.P * self.Q * 4)

    def as_dict(self) -> dict:
        d = asdict(self)
        d["P"], d["Q"] = self.P, self.Q
        return d


# --- the five benchmark configurations -------------------------------------------------
MINIBATCH = 28  # Section 5.1: mini-batch 28, one image per core

CFG1 = ConvShape(1, 64, 14, 14, 64, 3, 3, 1, 1, "cfg1_3x3_64_14")
CFG2 = ConvShape(MINIBATCH, 64, 56, 56, 64, 3, 3, 1, 1, "3x3_64_56")
CFG3A = ConvShape(MINIBATCH, 256, 56, 56, 64, 1, 1, 1, 0, "1x1_256to64_56")
CFG3B = ConvShape(MINIBATCH, 512, 28, 28, 1024, 1, 1, 2, 0, "1x1s2_512to1024_28")


def resnet50_layers(N: int = MINIBATCH) -> list[ConvShape]:
    """ResNet-50-shaped layer sweep: four 3x3 layers, eight 1x1 layers, and the 7x7 stem."""
    layers = []
    for c, hw in ((64, 56), (128, 28), (256, 14), (512, 7)):
        layers.append(ConvShape(N, c, hw, hw, c, 3, 3, 1, 1, f"3x3_{c}_{hw}"))
    for (a, b), hw in (((64, 256), 56), ((128, 512), 28), ((256, 1024), 14), ((512, 2048), 7)):
        layers.append(ConvShape(N, a, hw, hw, b, 1, 1, 1, 0, f"1x1_{a}to{b}_{hw}"))
        layers.append(ConvShape(N, b, hw, hw, a, 1, 1, 1, 0, f"1x1_{b}to{a}_{hw}"))
    layers.append(ConvShape(N, 3, 224, 224, 64, 7, 7, 2, 3, "stem_7x7s2_3to64_224"))
    return layers


def heldout_layers(N: int = MINIBATCH) -> list[ConvShape]:
    """Layer shapes of the kind the paper's other networks have (Section 5.1 lists AlexNet, OverFeat, GoogLeNet and
    others besides ResNet-50, without tabulating their layers): channel widths that are not powers of two, 5x5 and
    11x11 filters, a strided 3x3, odd image sizes.  Synthetic stand-ins chosen here, not taken from the paper.  The
    tile model's constants were never tuned on them: they are the out-of-sample check of its ranking."""
    return [
        ConvShape(N, 96, 27, 27, 96, 3, 3, 1, 1, "3x3_96_27"),
        ConvShape(N, 192, 13, 13, 192, 3, 3, 1, 1, "3x3_192_13"),
        ConvShape(N, 384, 13, 13, 384, 3, 3, 1, 1, "3x3_384_13"),
        ConvShape(N, 48, 27, 27, 128, 5, 5, 1, 2, "5x5_48to128_27"),
        ConvShape(N, 128, 56, 56, 128, 3, 3, 2, 1, "3x3s2_128_56"),
        ConvShape(N, 192, 28, 28, 64, 1, 1, 1, 0, "1x1_192to64_28"),
        ConvShape(N, 480, 14, 14, 192, 1, 1, 1, 0, "1x1_480to192_14"),
        ConvShape(N, 3, 227, 227, 64, 11, 11, 4, 0, "11x11s4_3to64_227"),
    ]


def validation_layers(N: int = MINIBATCH) -> list[ConvShape]:
    """A third layer set of the same kind as heldout_layers (GoogLeNet-like widths such as 160, 208, 320 and 832, a 5x5
    over 32 channels, a strided 3x3, a 7x7 stem with 96 output channels).  heldout_layers exposed one weakness of the
    tile model, which was then changed; this set was swept only after that change and nothing was ever adjusted on
    it."""
    return [
        ConvShape(N, 160, 28, 28, 160, 3, 3, 1, 1, "3x3_160_28"),
        ConvShape(N, 320, 14, 14, 320, 3, 3, 1, 1, "3x3_320_14"),
        ConvShape(N, 32, 14, 14, 96, 5, 5, 1, 2, "5x5_32to96_14"),
        ConvShape(N, 256, 28, 28, 256, 3, 3, 2, 1, "3x3s2_256_28"),
        ConvShape(N, 96, 14, 14, 208, 1, 1, 1, 0, "1x1_96to208_14"),
        ConvShape(N, 832, 7, 7, 256, 1, 1, 1, 0, "1x1_832to256_7"),
        ConvShape(N, 1280, 7, 7, 320, 1, 1, 1, 0, "1x1_1280to320_7"),
        ConvShape(N, 3, 224, 224, 96, 7, 7, 2, 3, "stem_7x7s2_3to96_224"),
    ]


def first_layers(N: int = MINIBATCH) -> list[ConvShape]:
    """First layers of image networks of the kinds Section 5.1 lists: three input channels, 3x3 filters with stride 1
    or 2 at 224 to 416 pixels, 11x11 with stride 4.  The paper leaves such layers out (channel counts that are not
    multiples of 16); here the tap-packed loops run them.  Synthetic stand-ins chosen here; nothing in the tile model was
    ever adjusted on them."""
    return [
        ConvShape(N, 3, 299, 299, 32, 3, 3, 2, 0, "3x3s2_3to32_299"),
        ConvShape(N, 3, 224, 224, 32, 3, 3, 2, 1, "3x3s2_3to32_224"),
        ConvShape(N, 3, 224, 224, 64, 3, 3, 1, 1, "3x3_3to64_224"),
        ConvShape(N, 3, 416, 416, 32, 3, 3, 1, 1, "3x3_3to32_416"),
        ConvShape(N, 3, 227, 227, 96, 11, 11, 4, 0, "11x11s4_3to96_227"),
    ]


def random_first_layer_shapes(count: int, seed: int) -> list[ConvShape]:
    """Seeded small shapes of the first-layer kind: 1 to 8 input channels (three most often), square filters of side 3, 5, 7 or 11,
    strides 1-4, pads from none to more than the filter needs, images just large enough up to 40 pixels."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        F = int(rng.choice([3, 5, 7, 11]))
        stride, pad = int(rng.integers(1, 5)), int(rng.integers(0, F // 2 + 2))
        H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
        if H + 2 * pad < F or W + 2 * pad < F:
            continue
        out.append(ConvShape(int(rng.integers(1, 4)), int(rng.choice([1, 2, 3, 3, 3, 4, 6, 8])), H, W, 16 * int(rng.integers(1, 9)), F, F,
                             stride, pad, f"first{len(out)}_seed{seed}"))
    return out


def sweep_seed(layer_index: int) -> int:
    return 100 + layer_index


# --- value distributions ---------------------------------------------------------------
def uniform_pm1(shape: ConvShape, seed: int) -> tuple[np.ndarray, np.ndarray]:
    """Input and filter iid uniform on [-1, 1) (the small single-layer configuration)."""
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1.0, 1.0, size=(shape.N, shape.C, shape.H, shape.W)).astype(np.float32)
    w = rng.uniform(-1.0, 1.0, size=(shape.K, shape.C, shape.R, shape.S)).astype(np.float32)
    return x, w


def relu_like(shape: ConvShape, seed: int) -> tuple[np.ndarray, np.ndarray]:
    """Input uniform on [0, 1) (post-ReLU-like); filter normal with std sqrt(2/(C*R*S))."""
    rng = np.random.default_rng(seed)
    x = rng.random(size=(shape.N, shape.C, shape.H, shape.W), dtype=np.float32)
    sigma = math.sqrt(2.0 / (shape.C * shape.R * shape.S))
    w = (rng.standard_normal(size=(shape.K, shape.C, shape.R, shape.S), dtype=np.float32)
         * np.float32(sigma))
    return x, w


def small_integers(shape: ConvShape, seed: int, lo: int = -2, hi: int = 2) -> tuple[np.ndarray, np.ndarray]:
    """Integer-valued tensors in [lo, hi]: every partial sum is exact in fp32 and in bf16
    products, so a correct implementation reproduces the exact result bit for bit."""
    rng = np.random.default_rng(seed)
    x = rng.integers(lo, hi + 1, size=(shape.N, shape.C, shape.H, shape.W)).astype(np.float32)
    w = rng.integers(lo, hi + 1, size=(shape.K, shape.C, shape.R, shape.S)).astype(np.float32)
    return x, w


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); returned widened to fp32.

    Input preparation for the bf16 configuration: both the oracle and the GPU path consume
    these already-rounded values."""
    bits = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    is_nan = (bits & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    out = np.where(is_nan, bits | np.uint32(0x00400000), rounded).astype(np.uint32)
    out = out & np.uint32(0xFFFF0000)
    return out.view(np.float32).reshape(a.shape)


def bf16_bits(a_rounded: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of values that are already exactly representable in bfloat16."""
    bits = np.ascontiguousarray(a_rounded, dtype=np.float32).view(np.uint32)
    return (bits >> np.uint32(16)).astype(np.uint16).reshape(a_rounded.shape)


# ---- inputs of the pairwise ranker (Section 4.2.2): random draws only, no arithmetic of the method ----

RANKER_STATS = 4
RANKER_WIDTHS = (2 * RANKER_STATS, 64, 32, 16, 8, 2)


def ranker_params(seed: int, scale: float = 1.0) -> np.ndarray:
    """A random parameter vector in the flat layout of the library (per layer: weights [inputs][units], bias):
    weights normal with standard deviation scale * sqrt(2 / inputs), biases normal with 0.1 * scale."""
    rng = np.random.default_rng(seed)
    parts = []
    for a, b in zip(RANKER_WIDTHS[:-1], RANKER_WIDTHS[1:]):
        parts.append(rng.normal(0.0, scale * math.sqrt(2.0 / a), a * b))
        parts.append(rng.normal(0.0, 0.1 * scale, b))
    return np.concatenate(parts).astype(np.float32)


def ranker_stats(n: int, seed: int, zero_fraction: float = 0.2, duplicates: int = 0) -> np.ndarray:
    """Statistics of n variants, float32 [n][4]: sizes log-uniform between 1e3 and 1e9 with a share of exact zeros
    (a level that holds no working set), the way working-set sizes in bytes are spread; the last `duplicates` rows
    repeat earlier ones (variants that differ in nothing the statistics see)."""
    rng = np.random.default_rng(seed)
    s = np.exp(rng.uniform(math.log(1e3), math.log(1e9), (n, RANKER_STATS)))
    s[rng.uniform(size=s.shape) < zero_fraction] = 0.0
    for d in range(min(duplicates, n // 2)):
        s[n - 1 - d] = s[d]
    return s.astype(np.float32)


def random_shapes(count: int, seed: int) -> list[ConvShape]:
    """Seeded small convolution shapes that wander over the whole parameter space the library accepts: channel
    counts that are not multiples of 16, non-square images and filters up to 7 x 7, strides 1-3, pads 0-3 (also
    larger than the filter needs, which gives outputs that see nothing but padding)."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        R, S = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        if rng.uniform() < 0.5:
            S = R
        stride, pad = int(rng.integers(1, 4)), int(rng.integers(0, 4))
        H, W = int(rng.integers(1, 21)), int(rng.integers(1, 21))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        N = int(rng.integers(1, 4))
        C = int(rng.choice([1, 3, 4, 5, 16, 17, 32, 40, 64, 70]))
        K = 16 * int(rng.integers(1, 9))
        out.append(ConvShape(N, C, H, W, K, R, S, stride, pad, f"random{len(out)}_seed{seed}"))
    return out
