"""Pins for the low-rank adapter oracle: y[t] = B_m (A_m x[t]), m = Idx[t] (paper Section 5.2 with a
low-rank matrix in place of a compressed delta; Section 3.2, Section 6.4).  Nothing here calls the GPU
library."""
import numpy as np

import dz_synth as S
import oracle


def _case(seed, T, N, K, D, r):
    x = S.make_x(T, K, S.stream(seed, "x")).numpy()
    A = [S.make_base(r, K, S.stream(seed, "A", m), 0.05).numpy() for m in range(D)]
    B = [S.make_base(N, r, S.stream(seed, "B", m), 0.05).numpy() for m in range(D)]
    ids = S.ids_uniform(T, D, S.stream(seed, "ids")).numpy()
    return x, A, B, ids


def test_brute_force_triple_loop():
    T, N, K, D, r = 4, 6, 8, 3, 2
    x, A, B, ids = _case(1, T, N, K, D, r)
    ids[1] = -1
    y = oracle.lora.lora_sbmm(x, A, B, ids)
    for t in range(T):
        m = int(ids[t])
        for n in range(N):
            acc = 0.0
            if m >= 0:
                for rho in range(r):
                    u = 0.0
                    for k in range(K):
                        u += float(A[m][rho, k]) * float(x[t, k])
                    acc += float(B[m][n, rho]) * u
            assert abs(y[t, n] - acc) <= 1e-12 * max(1.0, abs(acc))


def test_rank_one_closed_form():
    """A = a^T (1 x K), B = b (N x 1): y[t][n] = b[n] * (a . x[t]); a transposed operand or a swapped
    A/B could not produce this."""
    T, N, K = 5, 7, 16
    x, A, B, _ = _case(2, T, N, K, 1, 1)
    ids = np.zeros(T, np.int32)
    y = oracle.lora.lora_sbmm(x, A, B, ids)
    a, b = A[0][0].astype(np.float64), B[0][:, 0].astype(np.float64)
    want = np.outer(x.astype(np.float64) @ a, b)
    np.testing.assert_allclose(y, want, rtol=1e-13, atol=1e-15)
    # one-hot activation picks out a column of B A
    x1 = np.zeros((1, K), np.float16); x1[0, 3] = 2.0
    y1 = oracle.lora.lora_sbmm(x1, A, B, np.zeros(1, np.int32))
    np.testing.assert_allclose(y1[0], 2.0 * b * a[3], rtol=1e-13, atol=0)


def test_zero_adapter_and_base_only_requests():
    T, N, K, D, r = 6, 10, 32, 2, 4
    x, A, B, ids = _case(3, T, N, K, D, r)
    Bz = [np.zeros_like(b) for b in B]
    assert not oracle.lora.lora_sbmm(x, A, Bz, ids).any()
    assert not oracle.lora.lora_sbmm(x, A, B, np.full(T, -1, np.int32)).any()
    assert not oracle.lora.lora_sbmm(x, A, B, np.full(T, D, np.int32)).any()


def test_equals_the_dense_delta_oracle_on_B_times_A():
    """An adapter stands for the dense update B A: the pinned linear-layer oracle (C, plain loops) fed
    with that dense matrix must give the same rows, request by request."""
    T, N, K, D, r = 9, 24, 64, 3, 8
    x, A, B, ids = _case(4, T, N, K, D, r)
    ids[2] = -1
    dense = [oracle.lora.dense_update(A[m], B[m]).astype(np.float32) for m in range(D)]
    y = oracle.lora.lora_sbmm(x, A, B, ids)
    y_c = oracle.c.linear(x, None, dense, ids.astype(np.int32), acc64=True)
    np.testing.assert_allclose(y, y_c, rtol=0, atol=2e-6)          # dense was rounded to fp32 once
    # and every request uses its own adapter: make them very different
    A2 = [a * np.float16(4.0 ** m) for m, a in enumerate(A)]
    y2 = oracle.lora.lora_sbmm(x, A2, B, ids)
    for t in range(T):
        if ids[t] >= 0:
            np.testing.assert_allclose(y2[t], y[t] * 4.0 ** ids[t], rtol=1e-12, atol=0)
