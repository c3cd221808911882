"""CPU oracle for the two variants beside the 2:4 format -- TEST INFRASTRUCTURE ONLY.

  * quantisation-only deltas (paper Section 4.1 step 3 without the pruning of step 2; the
    compressed-matmul comparison of Section 4.1 sets this format against 2:4 + quantisation): every
    column carries a b-bit code,
        value[n][k] = (code[n][k] - zero[n][k // G]) * scale[n][k // G]     (fp32, exact);
  * the merged weight of one variant (Section 5.1 Eq. (2) read right to left):
        merged[n][k] = f16( float(W[n][k]) + delta[n][k] ).

The quantiser is the rule of the compressor oracle's step 3 applied to all G values of a group
instead of the G/2 kept ones.  Plain numpy, one group at a time.
"""
from __future__ import annotations

import numpy as np


def dequant_dense(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray, bits: int, group: int) -> np.ndarray:
    """codes u8 [N][K], scale / zero f16 [N][K/G] -> fp32 [N][K]."""
    N, K = codes.shape
    assert K % group == 0 and scale.shape == (N, K // group) and zero.shape == (N, K // group)
    assert int(codes.max(initial=0)) < (1 << bits)
    dense = np.zeros((N, K), np.float32)
    for gq in range(K // group):
        s = scale[:, gq].astype(np.float32)[:, None]
        z = zero[:, gq].astype(np.float32)[:, None]
        dense[:, gq * group:(gq + 1) * group] = (codes[:, gq * group:(gq + 1) * group].astype(np.float32) - z) * s
    return dense


def quantize_dense(delta: np.ndarray, bits: int, group: int):
    """delta f16 [N][K] -> (codes u8 [N][K], scale f16 [N][K/G], zero f16 [N][K/G]): per row and group
    of G columns lo = min(0, min v), hi = max(0, max v), s = f16((hi - lo) / (2^b - 1)) (s = 1, z = 0 if
    that is zero), z = clamp(rint((0 - lo) / s)), code = clamp(rint(v / s) + z); fp32, half to even."""
    N, K = delta.shape
    assert K % group == 0
    qmax = np.float32((1 << bits) - 1)
    codes = np.zeros((N, K), np.uint8)
    scale = np.zeros((N, K // group), np.float16)
    zero = np.zeros((N, K // group), np.float16)
    for gq in range(K // group):
        v = delta[:, gq * group:(gq + 1) * group].astype(np.float32)
        lo = np.minimum(np.float32(0), v.min(axis=1))
        hi = np.maximum(np.float32(0), v.max(axis=1))
        s16 = ((hi - lo) / qmax).astype(np.float16)
        dead = s16 == 0
        s16 = np.where(dead, np.float16(1), s16)
        s = s16.astype(np.float32)
        z = np.where(dead, np.float32(0), np.clip(np.rint((np.float32(0) - lo) / s), np.float32(0), qmax))
        codes[:, gq * group:(gq + 1) * group] = np.clip(np.rint(v / s[:, None]) + z[:, None], np.float32(0), qmax).astype(np.uint8)
        scale[:, gq] = s16
        zero[:, gq] = z.astype(np.float16)
    return codes, scale, zero


def merged_weight(W: np.ndarray, dense_delta: np.ndarray) -> np.ndarray:
    """f16 [N][K]: the variant's own weight, W + delta, rounded to fp16 once (the sum is formed in fp64,
    where it is exact, so the result is the correctly rounded one)."""
    return (W.astype(np.float64) + dense_delta.astype(np.float64)).astype(np.float16)
