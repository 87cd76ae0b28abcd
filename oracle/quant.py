"""Oracle side of the 4-bit projection weights (test infrastructure, never imported by the product path).

The paper's larger verifier is a weight-only 4-bit checkpoint of the AWQ family (Section IV-A).  Such a
checkpoint stores, per output row and group of 128 inputs, a scale and a zero point, and per weight a code
in 0..15; the weight it stands for is (code - zero) * scale.  The verifier's products take their operands
in bf16, so the weight that enters a product is that value rounded to bf16 (nearest, ties to even).
"""
import numpy as np

from .forward import round_bf16


def dequant_w4(codes, scales, zeros, group=128):
    """codes [N, K] (0..15), scales [N, K/group], zeros [N, K/group] -> float64 [N, K] of bf16 values."""
    codes = np.asarray(codes, dtype=np.float64)
    n, k = codes.shape
    s = np.repeat(np.asarray(scales, dtype=np.float64), group, axis=1)
    z = np.repeat(np.asarray(zeros, dtype=np.float64), group, axis=1)
    assert s.shape == (n, k) and z.shape == (n, k)
    return round_bf16((codes - z) * s)
