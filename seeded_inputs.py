"""Seeded synthetic input generators shared by the CPU oracle and the HIP path.

This module holds none of the method's arithmetic: it only turns
(seed, tensor name, element index) into reproducible pseudo-random numbers
(raw 64-bit words, uniform int8 codes, standard normals, class labels).
Quantisation, Fixup scaling and everything else the paper defines is done
separately by each side on the arrays produced here.

Generator: a counter-based integer hash.  For element i of tensor `name`
under `seed`, the 64-bit word is  mix(seed*K1 + crc32(name)*K2 + i*K3 + stream)
with the splitmix64 finaliser as `mix`.  No state is carried between calls, so
any element can be regenerated on its own.
"""
from __future__ import annotations

import zlib

import numpy as np

_K1 = np.uint64(0x9E3779B97F4A7C15)
_K2 = np.uint64(0xC2B2AE3D27D4EB4F)
_K3 = np.uint64(0xD6E8FEB86659FD93)
_K4 = np.uint64(0xA0761D6478BD642F)


def _mix(z: np.ndarray) -> np.ndarray:
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= np.uint64(0xBF58476D1CE4E5B9)
    z ^= z >> np.uint64(27)
    z *= np.uint64(0x94D049BB133111EB)
    z ^= z >> np.uint64(31)
    return z


def tensor_id(name: str) -> int:
    return zlib.crc32(name.encode("utf-8")) & 0xFFFFFFFF


def words(seed: int, name: str, n: int, stream: int = 0) -> np.ndarray:
    """n raw 64-bit words for tensor `name` (uint64)."""
    with np.errstate(over="ignore"):
        base = (np.uint64(seed & 0xFFFFFFFFFFFFFFFF) * _K1
                + np.uint64(tensor_id(name)) * _K2
                + np.uint64(stream) * _K4)
        idx = np.arange(n, dtype=np.uint64) * _K3
        return _mix(_mix(idx + base) ^ base)


def uniform_int8(seed: int, name: str, shape, lo: int = -127, hi: int = 127) -> np.ndarray:
    """Integers uniform in [lo, hi] as int8 (word mod span + lo)."""
    n = int(np.prod(shape))
    span = np.uint64(hi - lo + 1)
    w = words(seed, name, n)
    return ((w % span).astype(np.int64) + lo).astype(np.int8).reshape(shape)


def uniform01(seed: int, name: str, n: int, stream: int = 0) -> np.ndarray:
    """Doubles in (0, 1]: (top 53 bits + 1) / 2^53."""
    w = words(seed, name, n, stream)
    return ((w >> np.uint64(11)).astype(np.float64) + 1.0) / 9007199254740992.0


def standard_normal(seed: int, name: str, shape) -> np.ndarray:
    """N(0,1) doubles by Box-Muller from two hashed uniforms per element."""
    n = int(np.prod(shape))
    u1 = uniform01(seed, name, n, stream=1)
    u2 = uniform01(seed, name, n, stream=2)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return z.reshape(shape)


def labels(seed: int, name: str, n: int, classes: int) -> np.ndarray:
    """Class labels in [0, classes) as int32."""
    return (words(seed, name, n) % np.uint64(classes)).astype(np.int32)


# Workload shapes (configuration only).  They take the shapes and class counts of
# the paper's workloads: CIFAR-10-like 32x32x3 / 10 classes, ImageNet-like
# 224x224x3 / 1000 classes.  `block`: basic = two 3x3 convs, bottleneck = 1x1-3x3-1x1
# with 4x expansion and the stride on the 3x3.  `stem`: "cifar" = 3x3/1 conv,
# "imagenet" = 7x7/2 conv + 3x3/2 max pool.
WORKLOADS = {
    "block16": dict(block="basic", depths=(1,), widths=(16,), stem="none", classes=0, in_hw=32, in_ch=16),
    "resnet20": dict(block="basic", depths=(3, 3, 3), widths=(16, 32, 64), stem="cifar", classes=10,
                     in_hw=32, in_ch=3),
    "resnet110": dict(block="basic", depths=(18, 18, 18), widths=(16, 32, 64), stem="cifar", classes=10,
                      in_hw=32, in_ch=3),
    "resnet18": dict(block="basic", depths=(2, 2, 2, 2), widths=(64, 128, 256, 512), stem="imagenet",
                     classes=1000, in_hw=224, in_ch=3),
    "resnet34": dict(block="basic", depths=(3, 4, 6, 3), widths=(64, 128, 256, 512), stem="imagenet",
                     classes=1000, in_hw=224, in_ch=3),
    "resnet50": dict(block="bottleneck", depths=(3, 4, 6, 3), widths=(64, 128, 256, 512), stem="imagenet",
                     classes=1000, in_hw=224, in_ch=3),
    # reduced shapes for fast tests (same topology rules, tiny sizes)
    "tiny_basic": dict(block="basic", depths=(1, 2), widths=(16, 32), stem="cifar", classes=10,
                       in_hw=16, in_ch=3),
    "tiny_bottleneck": dict(block="bottleneck", depths=(2, 1), widths=(16, 32), stem="imagenet", classes=12,
                            in_hw=32, in_ch=3),
}


def batch_images(seed: int, step: int, n: int, hw: int, ch: int = 3) -> np.ndarray:
    """fp32 NHWC images ~ N(0,1) for training step `step` (the step index is part of the counter)."""
    return standard_normal(seed, f"images.step{step}", (n, hw, hw, ch)).astype(np.float32)


def batch_labels(seed: int, step: int, n: int, classes: int) -> np.ndarray:
    return labels(seed, f"labels.step{step}", n, classes)
