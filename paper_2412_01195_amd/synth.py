"""Seeded synthetic inputs for the 8-bit optimizer step (shapes and random data only).

This module holds none of the method's arithmetic: it lists tensor shapes that
follow the speaker-extractor architectures the paper trains (ResNet34 and
ResNet293 style backbones, embedding dimension 256 and a 5994-speaker
classification head, Sec. V "Training Settings" and "Datasets") and draws
weights / gradients from a counter-based generator (numpy Philox keyed by
(seed, config, tensor, step)).  The CPU oracle and the HIP path are both fed
from here by the tests and by the benchmark; neither of them imports this file.

Distribution conventions: "N(0, s)" means a normal law with standard deviation
s; "U(a, b)" a uniform law on [a, b).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

SPEAKERS = 5994        # classes of the training set (Sec. V, datasets)
EMBED = 256            # speaker-embedding dimension (Sec. V, training settings)
FBANK = 80             # input feature dimension (Sec. V, training settings)


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: Tuple[int, ...]
    fan_in: int

    @property
    def numel(self) -> int:
        return int(np.prod(self.shape))


def _conv(name, cout, cin, k):
    return TensorSpec(name, (cout, cin, k, k), cin * k * k)


def _bn(name, c):
    return [TensorSpec(name + ".gamma", (c,), 1), TensorSpec(name + ".beta", (c,), 1)]


def _tail(specs, width_last, freq_bins, expansion):
    """Embedding layer over (mean, std) statistics pooling and the speaker head."""
    feat = width_last * expansion * freq_bins * 2
    specs.append(TensorSpec("embed.weight", (EMBED, feat), feat))
    specs.append(TensorSpec("embed.bias", (EMBED,), 1))
    specs.append(TensorSpec("head.weight", (SPEAKERS, EMBED), EMBED))


def resnet34_specs() -> List[TensorSpec]:
    """Basic-block backbone, widths 32/64/128/256, 3/4/6/3 blocks per stage."""
    specs = [_conv("conv1", 32, 1, 3)] + _bn("bn1", 32)
    cin = 32
    for s, (w, nblk) in enumerate(zip((32, 64, 128, 256), (3, 4, 6, 3))):
        for b in range(nblk):
            p = f"layer{s + 1}.{b}"
            specs.append(_conv(p + ".conv1", w, cin, 3)); specs += _bn(p + ".bn1", w)
            specs.append(_conv(p + ".conv2", w, w, 3)); specs += _bn(p + ".bn2", w)
            if cin != w:
                specs.append(_conv(p + ".shortcut", w, cin, 1)); specs += _bn(p + ".bn_sc", w)
            cin = w
    _tail(specs, 256, FBANK // 8, 1)
    return specs


def resnet293_specs() -> List[TensorSpec]:
    """Bottleneck backbone (1x1, 3x3, 1x1 with expansion 4), 10/20/64/3 blocks."""
    specs = [_conv("conv1", 32, 1, 3)] + _bn("bn1", 32)
    cin = 32
    for s, (w, nblk) in enumerate(zip((32, 64, 128, 256), (10, 20, 64, 3))):
        for b in range(nblk):
            p = f"layer{s + 1}.{b}"
            specs.append(_conv(p + ".conv1", w, cin, 1)); specs += _bn(p + ".bn1", w)
            specs.append(_conv(p + ".conv2", w, w, 3)); specs += _bn(p + ".bn2", w)
            specs.append(_conv(p + ".conv3", 4 * w, w, 1)); specs += _bn(p + ".bn3", 4 * w)
            if b == 0:
                specs.append(_conv(p + ".shortcut", 4 * w, cin, 1)); specs += _bn(p + ".bn_sc", 4 * w)
            cin = 4 * w
    _tail(specs, 256, FBANK // 8, 4)
    return specs


def df_resnet_specs(blocks=(3, 8, 48, 3)) -> List[TensorSpec]:
    """Depth-first bottleneck backbone in its reversible form (Sec. III-C, table of
    DF-RevNet66): per stage with half-width c in (24, 48, 96, 192), `blocks[s]` pairs of
    residual functions F and G, each a 1x1 conv c->4c with BN, a depth-wise 3x3 conv on 4c
    channels and a 1x1 conv 4c->c; 3x3 down-sampling convs between stages; a 7680x256
    embedding layer and the speaker head.  blocks=(2, 2, 4, 2) gives the 4.8 M-parameter
    DF-RevNet66, the default the deepest variant."""
    specs = [_conv("conv1", 48, 1, 3)] + _bn("bn1", 48) + [_conv("conv2", 48, 48, 3)] + _bn("bn2", 48)
    widths = (24, 48, 96, 192)
    for s, (c, nblk) in enumerate(zip(widths, blocks)):
        for b in range(nblk):
            for fn in ("F", "G"):
                p = f"stage{s + 1}.{b}.{fn}"
                specs.append(_conv(p + ".expand", 4 * c, c, 1)); specs += _bn(p + ".bn", 4 * c)
                specs.append(TensorSpec(p + ".dconv", (4 * c, 1, 3, 3), 9))
                specs.append(_conv(p + ".project", c, 4 * c, 1))
        if s + 1 < len(widths):
            specs.append(_conv(f"down{s + 1}", 4 * c, 2 * c, 3)); specs += _bn(f"down{s + 1}.bn", 4 * c)
    specs.append(TensorSpec("embed.weight", (EMBED, 7680), 7680))
    specs.append(TensorSpec("embed.bias", (EMBED,), 1))
    specs.append(TensorSpec("head.weight", (SPEAKERS, EMBED), EMBED))
    return specs


def _rng(seed: int, *counter: int) -> np.random.Generator:
    key = np.zeros(2, dtype=np.uint64)
    key[0] = np.uint64(seed & 0xFFFFFFFFFFFFFFFF)
    h = 0x9E3779B97F4A7C15
    for c in counter:
        h = ((h ^ (int(c) + 0x632BE59BD9B4E019)) * 0xD1342543DE82EF95) & 0xFFFFFFFFFFFFFFFF
        h ^= h >> 29
    key[1] = np.uint64(h)
    return np.random.Generator(np.random.Philox(key=key))


def uniform_weights(seed: int, tensor: int, n: int, lo=-0.1, hi=0.1) -> np.ndarray:
    r = _rng(seed, 1, tensor)
    return (lo + (hi - lo) * r.random(n, dtype=np.float32)).astype(np.float32)


def normal_grad(seed: int, tensor: int, step: int, n: int, std: float) -> np.ndarray:
    r = _rng(seed, 2, tensor, step)
    return (r.standard_normal(n, dtype=np.float32) * np.float32(std)).astype(np.float32)


def heavy_tail_scale(seed: int, tensor: int) -> float:
    """Per-tensor gradient scale, log-uniform in [1e-6, 1e-1]."""
    return float(10.0 ** _rng(seed, 3, tensor).uniform(-6.0, -1.0))


def heavy_tail_grad(seed: int, tensor: int, step: int, n: int, scale: float, block: int) -> np.ndarray:
    """Student-t (3 degrees of freedom) gradient times `scale`; in every block of
    `block` entries max(1, round(0.01 * len)) distinct entries are multiplied by 100."""
    r = _rng(seed, 4, tensor, step)
    z = r.standard_normal(n, dtype=np.float32).astype(np.float64)
    chi = r.standard_normal((3, n), dtype=np.float32).astype(np.float64)
    t = z / np.sqrt((chi * chi).sum(axis=0) / 3.0 + 1e-300)
    g = t * scale
    nb = (n + block - 1) // block
    for b in range(nb):
        lo, hi = b * block, min(n, (b + 1) * block)
        k = max(1, int(round(0.01 * (hi - lo))))
        pick = r.choice(hi - lo, size=k, replace=False)
        g[lo + pick] *= 100.0
    return g.astype(np.float32)


def fan_in_std(spec: TensorSpec, base: float) -> float:
    return base / math.sqrt(spec.fan_in)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Inputs for the bfloat16-storage entry points: the upper 16 bits of each float32
    (plain truncation -- this only manufactures representable test inputs)."""
    x = np.ascontiguousarray(x, np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16)


def f16_bits(x: np.ndarray) -> np.ndarray:
    """Inputs for the binary16-storage entry points: numpy's float16 cast of each value, as bit
    patterns (this only manufactures representable test inputs)."""
    return np.ascontiguousarray(x, np.float32).astype(np.float16).view(np.uint16)
