"""Seeded synthetic inputs: CNN-shaped FP32 weight sets and per-layer byte counts.

This module only *generates inputs* (layer shapes, He-normal weights, random
byte-count draws, edge-case layer tables).  It holds none of the method's
arithmetic: no packing, no truncation, no norms, no precision rule.  Both the
CPU oracle's tests and the GPU path's tests/bench draw their inputs from here so
that the two sides see identical data without sharing any code of the method.

The weight sets stand in for the trained networks of the paper's evaluation
(Section IV: AlexNet, VGG and ResNet trained on ImageNet ILSVRC-2012).  Pack and
unpack cost is data independent (pure byte selection), so only the shapes matter
for throughput; values matter only for the norm statistics.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

# A layer shape is (out_channels, in_channels, k_h, k_w); a fully-connected
# layer is (out_features, in_features, 1, 1).
Shape = Tuple[int, int, int, int]


def _conv(o: int, i: int, k: int) -> Shape:
    return (o, i, k, k)


def _fc(o: int, i: int) -> Shape:
    return (o, i, 1, 1)


def tiny_shapes() -> List[Shape]:
    return [_conv(16, 3, 3), _conv(32, 16, 3), _fc(10, 512)]


def alexnet_shapes() -> List[Shape]:
    return [
        _conv(64, 3, 11), _conv(192, 64, 5), _conv(384, 192, 3),
        _conv(256, 384, 3), _conv(256, 256, 3),
        _fc(4096, 9216), _fc(4096, 4096), _fc(1000, 4096),
    ]


def resnet50_shapes() -> List[Shape]:
    shapes: List[Shape] = [_conv(64, 3, 7)]
    in_ch = 64
    for width, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            shapes.append(_conv(width, in_ch, 1))        # 1x1 reduce
            shapes.append(_conv(width, width, 3))        # 3x3
            shapes.append(_conv(4 * width, width, 1))    # 1x1 expand
            if b == 0:
                shapes.append(_conv(4 * width, in_ch, 1))  # projection shortcut
            in_ch = 4 * width
    shapes.append(_fc(1000, 2048))
    return shapes


def vgg16_shapes() -> List[Shape]:
    cfg = [(64, 3), (64, 64), (128, 64), (128, 128), (256, 128), (256, 256),
           (256, 256), (512, 256), (512, 512), (512, 512), (512, 512),
           (512, 512), (512, 512)]
    shapes = [_conv(o, i, 3) for o, i in cfg]
    shapes += [_fc(4096, 25088), _fc(4096, 4096), _fc(1000, 4096)]
    return shapes


# The three networks of the paper's own evaluation (its Table 1, 200-class
# heads).  The table gives filter sizes and channel counts only; the first
# fully-connected layer is taken to see the usual 6x6x256 (AlexNet) and 7x7x512
# (VGG) feature maps.
def paper_alexnet_shapes() -> List[Shape]:
    """Modified AlexNet: 5 conv + 4 FC (an extra FC-4096), FC-200 head."""
    return [
        _conv(64, 3, 11), _conv(192, 64, 5), _conv(384, 192, 3), _conv(384, 384, 3),
        _conv(256, 384, 3),
        _fc(4096, 9216), _fc(4096, 4096), _fc(4096, 4096), _fc(200, 4096),
    ]


def paper_vgga_shapes() -> List[Shape]:
    """VGG configuration A: 8 conv + 3 FC, FC-200 head (129,574,592 weights)."""
    cfg = [(64, 3), (128, 64), (256, 128), (256, 256), (512, 256), (512, 512),
           (512, 512), (512, 512)]
    return [_conv(o, i, 3) for o, i in cfg] + [_fc(4096, 25088), _fc(4096, 4096),
                                              _fc(200, 4096)]


def paper_resnet34_shapes() -> List[Shape]:
    """ResNet-34 as the paper counts it: 33 conv (stem + 16 two-conv building
    blocks) + FC-200."""
    shapes: List[Shape] = [_conv(64, 3, 7)]
    in_ch = 64
    for width, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for _ in range(blocks):
            shapes.append(_conv(width, in_ch, 3))
            shapes.append(_conv(width, width, 3))
            in_ch = width
    shapes.append(_fc(200, 512))
    return shapes


def paper_resnet34_group_offsets() -> np.ndarray:
    """Layer-index ranges of the precision groups for ResNet (Section IV-B: the
    paper adapts precision per building block): stem, 16 blocks of two
    convolutions, head.  Group g covers layers [out[g], out[g+1])."""
    return np.array([0, 1] + [1 + 2 * (b + 1) for b in range(16)] + [34], dtype=np.int32)


SHAPES = {
    "tiny": tiny_shapes,
    "alexnet": alexnet_shapes,
    "resnet50": resnet50_shapes,
    "vgg16": vgg16_shapes,
    "paper_alexnet": paper_alexnet_shapes,
    "paper_vgga": paper_vgga_shapes,
    "paper_resnet34": paper_resnet34_shapes,
}

# Seed per configuration (Tiny is seed 0); byte-count draws use seed + 1000.
SEEDS = {"tiny": 0, "alexnet": 1, "resnet50": 2, "vgg16": 3,
         "paper_alexnet": 11, "paper_vgga": 12, "paper_resnet34": 13}


def layer_sizes(shapes: Sequence[Shape]) -> np.ndarray:
    return np.array([o * i * kh * kw for (o, i, kh, kw) in shapes], dtype=np.int64)


def offsets_from_sizes(sizes: Sequence[int]) -> np.ndarray:
    """Element offsets, length L+1, offsets[0] = 0, offsets[L] = N."""
    off = np.zeros(len(sizes) + 1, dtype=np.int64)
    np.cumsum(np.asarray(sizes, dtype=np.int64), out=off[1:])
    return off


@dataclass
class WeightSet:
    name: str
    shapes: List[Shape]
    layer_offsets: np.ndarray          # int64[L+1], element units
    weights: np.ndarray                # float32[N], all layers contiguous
    seed: int
    meta: dict = field(default_factory=dict)

    @property
    def n_layers(self) -> int:
        return len(self.layer_offsets) - 1

    @property
    def n_weights(self) -> int:
        return int(self.layer_offsets[-1])


def he_normal_weights(shapes: Sequence[Shape], seed: int) -> np.ndarray:
    """He-normal draw, std = sqrt(2 / fan_in), fan_in = in_ch * k_h * k_w.

    One generator per weight set; layers are drawn in order.
    """
    rng = np.random.default_rng(seed)
    parts = []
    for (o, i, kh, kw) in shapes:
        n = o * i * kh * kw
        std = np.float32(np.sqrt(2.0 / (i * kh * kw)))
        parts.append(rng.standard_normal(n, dtype=np.float32) * std)
    if not parts:
        return np.zeros(0, dtype=np.float32)
    return np.ascontiguousarray(np.concatenate(parts))


def make_weight_set(name: str) -> WeightSet:
    shapes = SHAPES[name]()
    seed = SEEDS[name]
    off = offsets_from_sizes(layer_sizes(shapes))
    return WeightSet(name, shapes, off, he_normal_weights(shapes, seed), seed)


def draw_bytes(n_layers: int, choices: Sequence[int], seed: int) -> np.ndarray:
    """Uniform per-layer draw of a byte count from `choices`."""
    rng = np.random.default_rng(seed + 1000)
    ch = np.asarray(choices, dtype=np.uint8)
    return ch[rng.integers(0, len(ch), size=n_layers)].astype(np.uint8)


def config_bytes(name: str, variant: str = "default") -> np.ndarray:
    """Per-layer byte counts of the named configuration.

    tiny: {2,3,4} in layer order.  alexnet: uniform draw from {1,2,3,4}.
    resnet50: uniform draw from {2,3,4}.  vgg16: variant in
    {"all2", "all3", "mixed"} (default "all2"); "mixed" draws from {1,2,3,4}.
    """
    L = len(SHAPES[name]())
    seed = SEEDS[name]
    if name == "tiny":
        return np.array([2, 3, 4], dtype=np.uint8)
    if name in ("alexnet", "paper_alexnet", "paper_vgga", "paper_resnet34"):
        return draw_bytes(L, (1, 2, 3, 4), seed)
    if name == "resnet50":
        return draw_bytes(L, (2, 3, 4), seed)
    if name == "vgg16":
        if variant in ("default", "all2"):
            return np.full(L, 2, dtype=np.uint8)
        if variant == "all3":
            return np.full(L, 3, dtype=np.uint8)
        if variant == "all1":
            return np.full(L, 1, dtype=np.uint8)
        if variant == "all4":
            return np.full(L, 4, dtype=np.uint8)
        if variant == "mixed":
            return draw_bytes(L, (1, 2, 3, 4), seed)
    raise ValueError(f"unknown config/variant {name}/{variant}")


def trajectory_noise(weights: np.ndarray, step: int, seed: int = 5,
                     rel_sigma: float = 1e-3) -> np.ndarray:
    """Noise of one step of the synthetic weight trajectory.

    Returns N(0, (rel_sigma * |w|)^2) element-wise, to be added to `weights`
    by the caller (multiplicative random walk; one generator per step).
    """
    rng = np.random.default_rng([seed, step])
    z = rng.standard_normal(weights.shape[0], dtype=np.float32)
    return z * (np.float32(rel_sigma) * np.abs(weights))


# ----------------------------------------------------------------------------
# Edge-case tables (not CNN shaped): ragged sizes, empty layers, every output
# misalignment.  Values are arbitrary bit patterns, including NaN/Inf/denormal.
# ----------------------------------------------------------------------------

def random_bit_patterns(n: int, seed: int) -> np.ndarray:
    """float32 array whose bit patterns are uniform over all 2^32 words."""
    rng = np.random.default_rng(seed)
    u = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    return u.view(np.float32)


def special_values() -> np.ndarray:
    """Bit patterns worth checking one by one: zeros, infinities, NaNs with
    payload in kept / dropped bytes, denormals, extremes."""
    u = np.array([
        0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00000, 0xFFC00000,
        0x7F800001, 0x7F8000FF, 0x7F80FF00, 0x7FFFFFFF, 0xFFFFFFFF, 0x00000001,
        0x000000FF, 0x0000FF00, 0x007FFFFF, 0x807FFFFF, 0x00800000, 0x7F7FFFFF,
        0xFF7FFFFF, 0x3F800000, 0xBF800000, 0x3F7FFFFF, 0x40490FDB, 0x01020304,
        0xA1B2C3D4, 0x00FF00FF, 0xFF00FF00, 0x12345678, 0x87654321, 0x0F0F0F0F,
    ], dtype=np.uint32)
    return u.view(np.float32)


def ragged_case(sizes: Sequence[int], rbytes: Sequence[int], seed: int,
                he: bool = False):
    """Arbitrary layer sizes / byte counts with random bit-pattern weights
    (or finite normal values when he=True, for the norm statistics)."""
    sizes = np.asarray(sizes, dtype=np.int64)
    off = offsets_from_sizes(sizes)
    n = int(off[-1])
    if he:
        rng = np.random.default_rng(seed)
        w = (rng.standard_normal(n, dtype=np.float32) * np.float32(0.05))
    else:
        w = random_bit_patterns(n, seed)
    return off, np.asarray(rbytes, dtype=np.uint8), np.ascontiguousarray(w)


def alignment_sweep_case(seed: int = 11):
    """Layer sizes and byte counts chosen so that the packed start offset of
    the layers takes every value 0..15 modulo 16, with ragged sizes around
    tile boundaries, empty layers and the r pattern 1,3,1,3,... included."""
    ragged = [1, 2, 3, 5, 15, 17, 4095, 4097, 1023, 1025, 7, 16, 31, 33, 63,
              65, 127, 129, 255, 257, 511, 513, 2047, 2049, 8191, 8193, 12289,
              4096, 1024, 6, 10, 14, 18, 22, 26, 30, 34, 9, 11, 13, 1021, 3071,
              5000, 64, 256, 100, 1000, 37, 41, 43, 47, 53, 59, 61, 67, 71, 73,
              79, 83, 89, 97, 101, 4093, 2051]
    sizes: List[int] = [1, 0, 2, 3, 5, 15, 17, 0]
    rb: List[int] = [1, 3, 1, 3, 1, 3, 1, 3]
    pos = sum(s * r for s, r in zip(sizes, rb))
    k = 0
    # For every (byte count, start offset mod 16) pair: a 1-byte filler layer
    # moves the running stream offset to the wanted residue, then a ragged
    # layer with that byte count follows.
    for r in (1, 2, 3, 4):
        for want in range(16):
            fill = (want - pos) % 16
            sizes.append(fill)
            rb.append(1)
            pos += fill
            n = ragged[k % len(ragged)]
            k += 1
            sizes.append(n)
            rb.append(r)
            pos += n * r
    sizes += [0, 0, 5]
    rb += [2, 4, 3]
    return ragged_case(sizes, rb, seed)
