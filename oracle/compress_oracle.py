"""CPU oracle for the data-free delta compressor -- TEST INFRASTRUCTURE ONLY.

The paper's compressor (Section 4.1) takes the delta between fine-tuned and base weights, prunes it
to the 2:4 pattern (step 2: in every group of four consecutive entries two are kept, each with a
2-bit position) and quantises the kept values to b-bit codes (step 3).  Its Algorithm 1 chooses mask
and codes with calibration data, which this build does not have; the compressor built here is the
data-free rule this build uses everywhere a compressed delta is needed:

  step 2  per group of four consecutive k keep the two entries of largest magnitude (ties: the lower
          position wins), listed in ascending position;
  step 3  per row and per `group` dense columns (= group/2 kept values) an asymmetric uniform grid that
          contains zero:  lo = min(0, min v), hi = max(0, max v),  s = f16((hi - lo) / (2^b - 1))
          (s = 1, z = 0 if that is zero),  z = clamp(rint((0 - lo) / s), 0, 2^b - 1),
          q = clamp(rint(v / s) + z, 0, 2^b - 1);  rint rounds half to even; arithmetic in fp32.

Output: the canonical tables (codes u8 [N][K/2], idx u8 [N][K/2], scale f16 [N][K/G], zero f16
[N][K/G]) whose meaning is value = (code - zero) * scale at column 4g + idx.  Written with plain numpy,
group by group, independently of the input generator's vectorised version; shares no code with the GPU
library.  Pins: tests/test_oracle_compress.py.
"""
from __future__ import annotations

import numpy as np


def prune_2of4(delta: np.ndarray):
    """delta f16 [N][K] -> (kept f16 [N][K/2], idx u8 [N][K/2])."""
    N, K = delta.shape
    assert K % 4 == 0
    kept = np.zeros((N, K // 2), np.float16)
    idx = np.zeros((N, K // 2), np.uint8)
    mag = np.abs(delta.astype(np.float32))
    for g in range(K // 4):
        m = mag[:, 4 * g:4 * g + 4]
        # rank by (magnitude descending, position ascending): a stable sort of -magnitude does that
        order = np.argsort(-m, axis=1, kind="stable")[:, :2]
        pos = np.sort(order, axis=1)
        for j in range(2):
            idx[:, 2 * g + j] = pos[:, j]
            kept[:, 2 * g + j] = delta[np.arange(N), 4 * g + pos[:, j]]
    return kept, idx


def quantize(kept: np.ndarray, bits: int, group: int):
    """kept f16 [N][K/2] -> (codes u8 [N][K/2], scale f16 [N][K/G], zero f16 [N][K/G])."""
    N, half = kept.shape
    per = group // 2
    assert half % per == 0
    qmax = np.float32((1 << bits) - 1)
    codes = np.zeros((N, half), np.uint8)
    scale = np.zeros((N, half // per), np.float16)
    zero = np.zeros((N, half // per), np.float16)
    for gq in range(half // per):
        v = kept[:, gq * per:(gq + 1) * per].astype(np.float32)
        lo = np.minimum(np.float32(0), v.min(axis=1))
        hi = np.maximum(np.float32(0), v.max(axis=1))
        s16 = ((hi - lo) / qmax).astype(np.float16)
        dead = s16 == 0
        s16 = np.where(dead, np.float16(1), s16)
        s = s16.astype(np.float32)
        z = np.clip(np.rint((np.float32(0) - lo) / s), np.float32(0), qmax)
        z = np.where(dead, np.float32(0), z)
        q = np.clip(np.rint(v / s[:, None]) + z[:, None], np.float32(0), qmax)
        codes[:, gq * per:(gq + 1) * per] = q.astype(np.uint8)
        scale[:, gq] = s16
        zero[:, gq] = z.astype(np.float16)
    return codes, scale, zero


def compress(delta: np.ndarray, bits: int, group: int):
    """delta f16 [N][K] -> canonical tables (codes, idx, scale, zero)."""
    kept, idx = prune_2of4(delta)
    codes, scale, zero = quantize(kept, bits, group)
    return codes, idx, scale, zero
