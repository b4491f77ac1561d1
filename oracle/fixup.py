"""Oracle: Fixup initialisation rules (Section 3.1, Eq.1; Section 3.2.3, weight
and scale/bias paragraphs).  TEST INFRASTRUCTURE ONLY -- see the package docstring.
"""
from __future__ import annotations

import math

import numpy as np

from .quant import cq_code, q_code


def alpha(L: int, m: int) -> float:
    """Eq.1: layer-wise coefficient L^(-1/(2m-2)); L = residual blocks in the
    network, m = layers (convolutions) in the block's branch."""
    return float(L) ** (-1.0 / (2 * m - 2))


def kaiming_std(fan_in: int) -> float:
    """Kaiming normal: N(0, 2/n), n = number of inputs of one output unit (C*R*S)."""
    return math.sqrt(2.0 / fan_in)


def init_conv_real(z, fan_in: int, scale: float = 1.0) -> np.ndarray:
    """Real-valued initial weights from standard normals z, as fp32:
    Kaiming everywhere, times Eq.1's coefficient inside residual branches."""
    return (np.asarray(z, dtype=np.float64) * (kaiming_std(fan_in) * scale)).astype(np.float32)


def init_conv_codes(z, fan_in: int, scale: float = 1.0) -> np.ndarray:
    """Q_w (Eq.8) of the initial weights -> int8 codes."""
    return cq_code(init_conv_real(z, fan_in, scale)).astype(np.int8)


def init_gamma_code() -> int:
    """Multiplier starts at 1 -> Q(1, 8) = code 128 (unclamped, Eq.10)."""
    return int(q_code(1.0))


def init_bias_code() -> int:
    """Biases start at 0."""
    return int(q_code(0.0))
