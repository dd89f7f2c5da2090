"""CPU ORACLE (test infrastructure, not part of the product path).

Dequantisation of 4-bit weight-only quantised matrices with groups of input channels, the format of the paper's
intermediate model ("a quantized 4-bit version of M_1", group size 128: three-model system design and
experimental setup): W[n][k] = scale[n][k // group] * (q[n][k] - zero[n][k // group]).  The oracle's forward
pass then runs on the dequantised matrix as on any other weight (fp64 accumulation), which is the definition
of a weight-only quantised layer.
"""
import numpy as np


def unpack_codes(codes):
    """uint8 [n, K/2], byte b holding k = 2b in the low nibble and k = 2b + 1 in the high one -> uint8 [n, K]."""
    codes = np.asarray(codes, dtype=np.uint8)
    n, half = codes.shape
    q = np.empty((n, 2 * half), dtype=np.uint8)
    q[:, 0::2] = codes & 0xF
    q[:, 1::2] = codes >> 4
    return q


def dequantize(codes, scale, zero, group=128):
    """codes uint8 [n, K/2]; scale float [n, K/group]; zero integer [n, K/group] -> float32 [n, K]
    (scale times a small integer is exact in fp32)."""
    q = unpack_codes(codes).astype(np.float64)
    s = np.repeat(np.asarray(scale, dtype=np.float64), group, axis=1)
    z = np.repeat(np.asarray(zero, dtype=np.float64), group, axis=1)
    return (s * (q - z)).astype(np.float32)
