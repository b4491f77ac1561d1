"""Initial parameters of a Fixup residual network as input data for FixupNet (host arithmetic, runs once).

Section 3.1: every convolution is drawn Kaiming-normal, N(0, 2/n) with n = C*R*S inputs per output unit, and the
convolutions inside a residual branch are scaled by the layer-wise coefficient of Eq.1, L^(-1/(2m-2)) (L residual
blocks in the network, m convolutions per branch); multipliers start at 1, biases at 0 (Section 3.2.3).  The
arrays returned here are real-valued fp32; the caller turns them into int8 codes with Q_w (Eq.8) through
eoq_quantize(EOQ_CQ), i.e. in the library's kernel.  The classifier stays in floating point (Section 5.1).
"""
from __future__ import annotations

import math

import numpy as np

import seeded_inputs as si


def branch_coefficient(n_blocks: int, convs_per_branch: int) -> float:
    """Eq.1."""
    return float(n_blocks) ** (-1.0 / (2 * convs_per_branch - 2))


def conv_weights_f32(seed: int, name: str, shape_krsc, scale: float) -> np.ndarray:
    """fp32 K x R x S x C filters: hashed standard normals times sqrt(2 / (C*R*S)) times `scale`."""
    K, R, S, Cc = shape_krsc
    z = si.standard_normal(seed, name + ".w", (K, R, S, Cc))
    return (z * (math.sqrt(2.0 / (Cc * R * S)) * scale)).astype(np.float32)


def classifier_f64(seed: int, classes: int, features: int):
    """(W [classes x features], b [classes]) in fp64: Kaiming-normal weights, zero bias."""
    z = si.standard_normal(seed, "fc.w", (classes, features))
    return z * math.sqrt(2.0 / features), np.zeros(classes, dtype=np.float64)
