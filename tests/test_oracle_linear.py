"""Pins for the oracle's linear layer: y[t] = x[t] . (W_base + Delta_{Idx[t]})^T.

Paper Section 5.1 Eq. (2) (the distributive split into a base product and a delta product) and
Section 5.2 (SBMM: request i is multiplied by the delta Idx_i names).  Nothing here calls the GPU
library.
"""
import numpy as np
import pytest
import torch

import dz_synth as S
import oracle


def _case(seed, T, N, K, D, bits, G, ids=None):
    W = S.make_base(N, K, S.stream(seed, "W")).numpy()
    x = S.make_x(T, K, S.stream(seed, "x")).numpy()
    tabs = [S.make_delta_tables(N, K, bits, G, S.stream(seed, "d", m), std=0.002) for m in range(D)]
    dense = [oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G)
             for t in tabs]
    if ids is None:
        ids = S.ids_uniform(T, D, S.stream(seed, "ids")).numpy()
    return W, x, tabs, dense, np.asarray(ids, np.int32)


def test_brute_force_8x8_tiles():
    """Separately written pure-Python triple loop straight from the definition, G = 8."""
    T = N = K = 8
    for bits in (2, 4):
        W, x, tabs, dense, ids = _case(bits, T, N, K, 3, bits, 8)
        ids[0] = -1                                  # one base-only request
        y = oracle.c.linear(x, W, dense, ids)
        y64 = oracle.c.linear(x, W, dense, ids, acc64=True)
        for t in range(T):
            m = int(ids[t])
            for n in range(N):
                acc = 0.0
                for k in range(K):
                    w = float(W[n, k])
                    if m >= 0:
                        tb = tabs[m]
                        g4 = k // 4
                        for j in range(2):
                            if int(tb.idx[n, 2 * g4 + j]) == k % 4:
                                w += (float(tb.codes[n, 2 * g4 + j]) - float(tb.zero[n, k // 8])) \
                                    * float(tb.scale[n, k // 8])
                    acc += float(x[t, k]) * w
                assert abs(y64[t, n] - acc) <= 1e-6 * max(1.0, abs(acc))
                assert abs(y[t, n] - acc) <= 1e-5 * max(1.0, abs(acc))


def test_zero_delta_reproduces_base_bit_for_bit():
    T, N, K, D, bits, G = 5, 24, 256, 2, 4, 64
    W, x, tabs, dense, ids = _case(1, T, N, K, D, bits, G)
    # a delta whose every code equals its zero-point dequantises to exactly 0
    z = tabs[0]
    qg = (np.arange(K // 2) // 2 * 4) // G
    codes0 = z.zero.numpy().astype(np.uint8)[:, qg]
    d0 = oracle.c.dequant(codes0, z.idx.numpy(), z.scale.numpy(), z.zero.numpy(), bits, G)
    assert not d0.any()
    y_base = oracle.c.linear(x, W, None, None)
    y_zero = oracle.c.linear(x, W, [d0, d0], ids)
    assert y_base.tobytes() == y_zero.tobytes()
    # ids outside [0, D) are base-only too
    y_none = oracle.c.linear(x, W, dense, np.full(T, -1, np.int32))
    assert y_base.tobytes() == y_none.tobytes()
    y_oob = oracle.c.linear(x, W, dense, np.full(T, D, np.int32))
    assert y_base.tobytes() == y_oob.tobytes()


def test_linearity_base_plus_delta():
    T, N, K, D, bits, G = 9, 40, 512, 3, 4, 128
    W, x, tabs, dense, ids = _case(2, T, N, K, D, bits, G)
    y = oracle.c.linear(x, W, dense, ids, acc64=True)
    yb = oracle.c.linear(x, W, None, None, acc64=True)
    yd = oracle.c.linear(x, None, dense, ids, acc64=True)
    assert np.abs(yd).max() > 0
    np.testing.assert_allclose(y, yb + yd, rtol=0, atol=2e-6)
    # fp32 accumulation: error bounded by K * 2^-24 * sum|terms|
    y32 = oracle.c.linear(x, W, dense, ids)
    xf = np.abs(x.astype(np.float64))
    bound = np.zeros_like(y, dtype=np.float64)
    for t in range(T):
        w = np.abs(W.astype(np.float64) + dense[ids[t]])
        bound[t] = K * 2.0 ** -24 * (w @ xf[t])
    assert (np.abs(y32.astype(np.float64) - y) <= bound + 1e-7).all()
    assert np.abs(y32 - y).max() < 2e-5


def test_each_request_uses_its_own_delta():
    """A swapped or ignored Idx would go unnoticed if deltas were alike: make them very different."""
    T, N, K, D, bits, G = 6, 16, 256, 3, 4, 64
    W, x, tabs, dense, _ = _case(3, T, N, K, D, bits, G)
    dense = [d * (10.0 ** m) for m, d in enumerate(dense)]
    ids = np.array([2, 0, 1, 1, 2, 0], np.int32)
    y = oracle.c.linear(x, None, dense, ids, acc64=True)
    for t in range(T):
        want = dense[ids[t]].astype(np.float64) @ x[t].astype(np.float64)
        np.testing.assert_allclose(y[t], want, rtol=1e-6, atol=1e-9)


def test_against_library_matmul_and_numpy_twin():
    T, N, K, D, bits, G = 16, 64, 1024, 4, 2, 128
    W, x, tabs, dense, ids = _case(4, T, N, K, D, bits, G)
    yb = oracle.c.linear(x, W, None, None)
    lib = x.astype(np.float32) @ W.astype(np.float32).T          # library sgemm
    np.testing.assert_allclose(yb, lib, rtol=0, atol=3e-5)
    exact = x.astype(np.float64) @ W.astype(np.float64).T
    assert np.abs(yb - exact).max() < 3e-5
    y_c = oracle.c.linear(x, W, dense, ids)
    y_np = oracle.np_.linear(x, W, dense, ids)
    np.testing.assert_allclose(y_c, y_np, rtol=0, atol=5e-5)
    y_np64 = oracle.np_.linear(x, W, dense, ids, dtype=np.float64)
    y_c64 = oracle.c.linear(x, W, dense, ids, acc64=True)
    np.testing.assert_allclose(y_c64, y_np64, rtol=0, atol=2e-6)


def test_transposed_operand_would_fail():
    """Non-square shapes: y is [T][N] with W [N][K]; a transposed W could not even be indexed the
    same way, and one-hot inputs pick out single weights."""
    T, N, K = 3, 8, 16
    W = (np.arange(N * K, dtype=np.float32).reshape(N, K) / 64).astype(np.float16)
    x = np.zeros((T, K), np.float16)
    x[0, 5] = 1; x[1, 0] = 2; x[2, 15] = -1
    y = oracle.c.linear(x, W, None, None)
    assert y.shape == (T, N)
    for n in range(N):
        assert y[0, n] == float(W[n, 5]) and y[1, n] == 2 * float(W[n, 0]) and y[2, n] == -float(W[n, 15])


@pytest.mark.parametrize("impl", ["c", "np"])
def test_fp16_subnormal_weights_are_widened_exactly(impl):
    """About 0.2 % of base weights drawn from N(0, 0.02) are fp16 subnormals (|w| < 2^-14).  A one-hot
    activation picks single weights out, so every subnormal bit pattern, both signs, must come back as
    exactly m * 2^-24 -- no tolerance: a wrong exponent in the widening of subnormals cannot hide."""
    pats = np.concatenate([np.arange(1, 1024, dtype=np.uint16), np.arange(1, 1024, dtype=np.uint16) | 0x8000])
    N, K = pats.size, 8
    W = np.zeros((N, K), np.uint16)
    W[:, 3] = pats
    W[:, 5] = 0x3C00                    # 1.0 in a column the activation does not select
    W = W.view(np.float16)
    x = np.zeros((2, K), np.float16)
    x[0, 3] = 1.0
    x[1, 3] = -2.0
    lin = oracle.c.linear if impl == "c" else oracle.np_.linear
    y = lin(x, W, None, None)
    m = (pats & 0x3FF).astype(np.float64) * np.where(pats & 0x8000, -1.0, 1.0)
    want = m * 2.0 ** -24               # exact in binary64 and in binary32
    assert y.dtype == np.float32
    assert (y[0].astype(np.float64) == want).all()
    assert (y[1].astype(np.float64) == -2.0 * want).all()
    # a subnormal activation against a normal weight, and subnormal times subnormal (exact in fp32: 20 bits)
    x2 = np.zeros((1, K), np.uint16)
    x2[0, 3] = 0x0203                   # 515 * 2^-24
    y2 = lin(x2.view(np.float16), W, None, None)
    assert (y2[0].astype(np.float64) == 515 * 2.0 ** -24 * want).all()
