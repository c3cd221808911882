"""numpy twin of the C oracle (test infrastructure only).

Same definition (paper Section 5.1 Eq. (2); Section 5.2 SBMM statement; Section 4.1 steps 2-3 for
what the compressed delta stands for), written with array indexing and a library matmul instead of
loops, so that an indexing mistake in one writing shows up as a disagreement with the other.
"""
from __future__ import annotations

import numpy as np


def dequant(codes, idx, scale, zero, bits: int, group: int, dtype=np.float32) -> np.ndarray:
    N, half = codes.shape
    K = half * 2
    col = (np.arange(half) // 2) * 4                     # first column of each kept value's group of 4
    cols = col[None, :] + idx.astype(np.int64)           # [N][K/2] destination columns
    qg = col // group                                    # quantisation group of each kept value
    s = scale.astype(dtype)[:, qg]
    z = zero.astype(dtype)[:, qg]
    vals = (codes.astype(dtype) - z) * s
    dense = np.zeros((N, K), dtype)
    np.put_along_axis(dense, cols, vals, axis=1)
    return dense


def linear(x, W, dense_deltas, token_to_delta, dtype=np.float32) -> np.ndarray:
    """Per request: one matrix-vector product with that request's own effective weight."""
    T, K = x.shape
    N = W.shape[0] if W is not None else dense_deltas[0].shape[0]
    y = np.zeros((T, N), dtype)
    xf = x.astype(dtype)
    for t in range(T):
        m = -1 if token_to_delta is None else int(token_to_delta[t])
        w = np.zeros((N, K), dtype) if W is None else W.astype(dtype)
        if dense_deltas and 0 <= m < len(dense_deltas):
            w = w + dense_deltas[m].astype(dtype)
        y[t] = w @ xf[t]
    return y


def segment(token_to_delta, D: int):
    ids = np.asarray(token_to_delta, np.int64)
    key = np.where((ids >= 0) & (ids < D), ids, D)
    perm = np.argsort(key, kind="stable").astype(np.int32)
    counts = np.bincount(key, minlength=D + 1)[:D].astype(np.int32)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    return counts, offsets, perm
