"""GPU: dz_compress_delta is bit-exact against the compressor oracle (2:4 magnitude pruning and group-wise
asymmetric round to nearest; paper Section 4.1 steps 2-3), and its tables serve through dz_pack_delta and
dz_sbmm like any others."""
import numpy as np
import pytest
import torch

import dz_synth as S
import oracle
from dzcase import assert_close

pytestmark = pytest.mark.gpu


def _compress(dz, ctx, d_dev, N, K, bits, G):
    codes = torch.full((N, K // 2), 0xFF, dtype=torch.uint8, device="cuda")
    idx = torch.full((N, K // 2), 0xFF, dtype=torch.uint8, device="cuda")
    scale = torch.full((N, K // G), float("nan"), dtype=torch.float16, device="cuda")
    zero = torch.full((N, K // G), float("nan"), dtype=torch.float16, device="cuda")
    dz.dz_compress_delta(ctx, d_dev, N, K, bits, G, codes, idx, scale, zero)
    torch.cuda.synchronize()
    return codes, idx, scale, zero


def _assert_tables_equal(got, want):
    codes, idx, scale, zero = (t.cpu().numpy() for t in got)
    wc, wi, ws, wz = want
    assert np.array_equal(idx, wi)
    assert np.array_equal(scale.view(np.uint16), ws.view(np.uint16))
    assert np.array_equal(zero.view(np.uint16), wz.view(np.uint16))
    assert np.array_equal(codes, wc)


@pytest.mark.parametrize("N,K,bits,G,std", [(16, 256, 4, 64, 0.002), (48, 768, 4, 128, 0.002), (32, 512, 2, 128, 0.002),
                                             (80, 1024, 2, 64, 0.01), (1024, 2816, 4, 128, 0.002),
                                             (512, 4096, 2, 128, 0.0005)])
def test_bit_exact_against_the_oracle(dz, N, K, bits, G, std):
    print(f"case N={N} K={K} bits={bits} G={G}", flush=True)
    d = S._normal_f16((N, K), std, S.stream(11, "dense delta", N, K, bits, G))
    want = oracle.compress_.compress(d.numpy(), bits, G)
    with dz.Context(0) as c:
        got = _compress(dz, c.h, d.cuda(), N, K, bits, G)
        _assert_tables_equal(got, want)
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_ties_zeros_and_tiny_values(dz):
    """Equal magnitudes (the lower position wins), all-zero groups (scale 1, zero 0, codes 0), one-sided
    groups (the grid still contains zero), subnormal values, and a group whose scale underflows to zero in
    fp16."""
    N, K, bits, G = 16, 256, 4, 64
    d = torch.zeros(N, K, dtype=torch.float16)
    d[0] = 1.0                                     # all equal: positions 0, 1 everywhere
    d[1, ::2] = -0.5; d[1, 1::2] = 0.5             # equal magnitudes, mixed signs
    d[2, :64] = torch.linspace(0.001, 0.02, 64).half()       # one-sided positive group
    d[3, :64] = -torch.linspace(0.001, 0.02, 64).half()      # one-sided negative group
    d[4, :64] = 6e-8                               # the smallest subnormal: (hi - lo) / 15 rounds to zero in fp16
    d[5, :64] = torch.linspace(-6e-5, 6e-5, 64).half()       # subnormal range
    d[6] = S._normal_f16((K,), 0.002, S.stream(12, "row"))
    d[6, 3::4] = d[6, 2::4]                        # tie between positions 2 and 3 in every group
    d[7, 0] = 65504.0; d[7, 1] = -65504.0          # hi - lo overflows fp16 but not fp32; s = f16(131008/15)
    want = oracle.compress_.compress(d.numpy(), bits, G)
    with dz.Context(0) as c:
        got = _compress(dz, c.h, d.cuda(), N, K, bits, G)
        _assert_tables_equal(got, want)
    assert want[1][0].reshape(-1, 2).tolist() == [[0, 1]] * (K // 4)
    assert want[2][4, 0] == 1.0 and want[3][4, 0] == 0.0 and not want[0][4, :32].any()


def test_compressed_delta_serves_through_pack_and_sbmm(dz):
    """dense delta -> dz_compress_delta -> dz_pack_delta -> dz_sbmm against the oracle chain
    compress -> dequant -> selective product on the same inputs."""
    T, N, K, D, bits, G = 24, 96, 1024, 3, 4, 128
    x = S.make_x(T, K, S.stream(13, "x"))
    ids = S.ids_uniform(T, D, S.stream(13, "ids")).to(torch.int32)
    dense_in = [S._normal_f16((N, K), 0.002, S.stream(13, "delta", m)) for m in range(D)]
    dense_ref = []
    for d in dense_in:
        codes, idx, scale, zero = oracle.compress_.compress(d.numpy(), bits, G)
        dense_ref.append(oracle.c.dequant(codes, idx, scale, zero, bits, G))
    want = oracle.c.linear(x.numpy(), None, dense_ref, ids.numpy())
    with dz.Context(0) as c:
        packed = []
        for d in dense_in:
            codes, idx, scale, zero = _compress(dz, c.h, d.cuda(), N, K, bits, G)
            p = torch.empty(dz.dz_packed_bytes(N, K, bits, G), dtype=torch.uint8, device="cuda")
            dz.dz_pack_delta(c.h, codes, idx, scale, zero, N, K, bits, G, p)
            packed.append(p)
        out = torch.empty(T, N, dtype=torch.float16, device="cuda")
        dz.dz_sbmm(c.h, x.cuda(), packed, ids.cuda(), out, T, N, K, bits, G, 0)
        torch.cuda.synchronize()
        assert_close(out, want, "compress -> pack -> sbmm")
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_argument_errors(dz):
    with dz.Context(0) as c:
        d = torch.zeros(16, 256, dtype=torch.float16, device="cuda")
        b = torch.zeros(16 * 128, dtype=torch.uint8, device="cuda")
        h = torch.zeros(64, dtype=torch.float16, device="cuda")
        assert dz.dz_compress_delta(c.h, d, 16, 256, 3, 64, b, b, h, h, check=False) == dz.DZ_ERR_BITS
        assert dz.dz_compress_delta(c.h, d, 16, 200, 4, 64, b, b, h, h, check=False) == dz.DZ_ERR_SHAPE
        assert dz.dz_compress_delta(c.h, d, 16, 256, 4, 32, b, b, h, h, check=False) == dz.DZ_ERR_SHAPE
        assert dz.dz_compress_delta(c.h, None, 16, 256, 4, 64, b, b, h, h, check=False) == dz.DZ_ERR_ARG
        assert dz.dz_compress_delta(c.h, d.view(-1)[1:], 16, 256, 4, 64, b, b, h, h, check=False) == dz.DZ_ERR_ALIGN
