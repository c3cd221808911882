"""GPU: the quantisation-only format (paper Section 4.1 step 3 without the 2:4 pruning of step 2) and the
merged weight of one variant (Section 5.1 Eq. (2)), against their oracles: pack / unpack bit-exact,
dz_qsbmm / dz_qlinear and base-product-of-the-merged-weight within the output tolerance."""
import numpy as np
import pytest
import torch

import dz_synth as S
import oracle
from dzcase import assert_close

pytestmark = pytest.mark.gpu


def _ids(kind, T, D, seed):
    g = S.stream(seed, "ids")
    v = {"uniform": lambda: S.ids_uniform(T, D, g), "zipf": lambda: S.ids_zipf(T, D, 1.5, g),
         "segments": lambda: S.ids_segments(T, D, g)}[kind]()
    return torch.as_tensor(np.asarray(v), dtype=torch.int32)


@pytest.mark.parametrize("N,K,bits,G", [(16, 256, 4, 64), (48, 768, 4, 128), (32, 512, 2, 128), (80, 1024, 2, 64),
                                         (1024, 2816, 4, 128)])
def test_qpack_qunpack_roundtrip_bit_exact(dz, N, K, bits, G):
    print(f"case N={N} K={K} bits={bits} G={G}", flush=True)
    t = S.make_dense_tables(N, K, bits, G, S.stream(41, "qpack", N, K, bits, G))
    with dz.Context(0) as c:
        d = t.to("cuda")
        nbytes = dz.dz_qpacked_bytes(N, K, bits, G)
        assert nbytes == S.qpacked_bytes(N, K, bits, G)
        guard = 64
        buf = torch.full((nbytes + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
        packed = buf[guard:guard + nbytes]
        dz.dz_qpack_delta(c.h, d.codes, d.scale, d.zero, N, K, bits, G, packed)
        codes = torch.full_like(d.codes, 0xFF)
        scale = torch.zeros_like(d.scale); zero = torch.zeros_like(d.zero)
        dense = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
        dz.dz_qunpack_delta(c.h, packed, N, K, bits, G, codes, scale, zero, dense)
        torch.cuda.synchronize()
        assert (buf[:guard] == 0xA5).all() and (buf[guard + nbytes:] == 0xA5).all()
        assert torch.equal(codes.cpu(), t.codes)
        assert scale.cpu().view(torch.int16).equal(t.scale.view(torch.int16))
        assert zero.cpu().view(torch.int16).equal(t.zero.view(torch.int16))
        ref = oracle.quant.dequant_dense(t.codes.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G)
        assert dense.cpu().numpy().tobytes() == ref.tobytes()
        buf2 = torch.zeros_like(buf)                    # every byte of the blob is written
        dz.dz_qpack_delta(c.h, d.codes, d.scale, d.zero, N, K, bits, G, buf2[guard:guard + nbytes])
        torch.cuda.synchronize()
        assert torch.equal(buf2[guard:guard + nbytes], packed)
        assert dz.dz_check(c.h) == dz.DZ_OK


CASES = [
    # name            T    N     K    D  bits  G   ids
    ("tiny",          8,  256,  256,  4, 4,  64, "uniform"),
    ("b4g128_t32",   32,   96, 1024,  8, 4, 128, "uniform"),
    ("b2g128_t64z",  64,  160, 1536, 32, 2, 128, "zipf"),
    ("b2g64_t7",      7,   48,  768,  3, 2,  64, "uniform"),
    ("b4g64_t1",      1,   32,  512,  2, 4,  64, "uniform"),
    ("b4g128_t17",   17,  208,  512,  5, 4, 128, "uniform"),
    ("b4g128_t100", 100,   64, 1024,  6, 4, 128, "uniform"),       # large batch: tiled kernel, mixed tiles
    ("b2g128_t200s", 200, 128,  512,  7, 2, 128, "segments"),
    ("b4g128_t300w", 300, 512, 1024,  2, 4, 128, "segments"),      # tiles whose rows all name one delta
    ("b2g64_t520",  520,  272,  768,  3, 2,  64, "segments"),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_parity(dz, case):
    name, T, N, K, D, bits, G, kind = case
    print(f"case {name}", flush=True)
    W = S.make_base(N, K, S.stream(42, "W"))
    x = S.make_x(T, K, S.stream(42, "x"))
    tabs = [S.make_dense_tables(N, K, bits, G, S.stream(42, "qdelta", m), std=0.002) for m in range(D)]
    ids = _ids(kind, T, D, 42)
    if T > 2:
        ids[1] = -1
    dense = [oracle.quant.dequant_dense(t.codes.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G) for t in tabs]
    y = oracle.c.linear(x.numpy(), W.numpy(), dense, ids.numpy())
    y_delta = oracle.c.linear(x.numpy(), None, dense, ids.numpy())
    with dz.Context(0) as c:
        packed = []
        for t in tabs:
            d = t.to("cuda")
            p = torch.empty(dz.dz_qpacked_bytes(N, K, bits, G), dtype=torch.uint8, device="cuda")
            dz.dz_qpack_delta(c.h, d.codes, d.scale, d.zero, N, K, bits, G, p)
            packed.append(p)
        dx, dW, did = x.cuda(), W.cuda(), ids.cuda()
        o = torch.full((T, N), 7.0, dtype=torch.float16, device="cuda")
        dz.dz_qsbmm(c.h, dx, packed, did, o, T, N, K, bits, G, 0)
        assert_close(o, y_delta, name + " qsbmm")
        o = torch.full((T, N), 7.0, dtype=torch.float16, device="cuda")
        dz.dz_qlinear(c.h, dx, dW, packed, did, o, T, N, K, bits, G)
        r = assert_close(o, y, name + " qlinear")
        print(f"  qlinear max_rel={r[0]:.2e} mean_abs={r[1]:.2e}", flush=True)
        o2 = torch.empty(T, N, dtype=torch.float16, device="cuda")
        dz.dz_base_gemm(c.h, dx, dW, o2, T, N, K)
        dz.dz_qsbmm(c.h, dx, packed, did, o2, T, N, K, bits, G, 1)
        assert_close(o2, y, name + " base then qsbmm(accumulate)")
        assert dz.dz_check(c.h) == dz.DZ_OK


@pytest.mark.parametrize("N,K,bits,G,T", [(48, 768, 4, 128, 24), (256, 1024, 2, 64, 300), (1024, 4096, 4, 128, 64)])
def test_merged_weight(dz, N, K, bits, G, T):
    """dz_merge_delta is bit-exact against the correctly rounded W + delta; the base product of the merged
    weight serves a batch of that one variant within the output tolerance of the exact layer."""
    print(f"case N={N} K={K} bits={bits} G={G} T={T}", flush=True)
    W = S.make_base(N, K, S.stream(43, "W", N))
    x = S.make_x(T, K, S.stream(43, "x", N))
    t = S.make_delta_tables(N, K, bits, G, S.stream(43, "delta", N))
    dense = oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G)
    want_m = oracle.quant.merged_weight(W.numpy(), dense)
    y = oracle.c.linear(x.numpy(), W.numpy(), [dense], np.zeros(T, np.int32))
    with dz.Context(0) as c:
        d = t.to("cuda")
        p = torch.empty(dz.dz_packed_bytes(N, K, bits, G), dtype=torch.uint8, device="cuda")
        dz.dz_pack_delta(c.h, d.codes, d.idx, d.scale, d.zero, N, K, bits, G, p)
        m = torch.full((N, K), float("nan"), dtype=torch.float16, device="cuda")
        dz.dz_merge_delta(c.h, W.cuda(), p, N, K, bits, G, m)
        torch.cuda.synchronize()
        assert m.cpu().numpy().tobytes() == want_m.tobytes()
        o = torch.empty(T, N, dtype=torch.float16, device="cuda")
        dz.dz_base_gemm(c.h, x.cuda(), m, o, T, N, K)
        assert_close(o, y, "base product of the merged weight")
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_two_of_four_delta_written_densely_serves_the_same(dz):
    """Dense-expanded serving of a 2:4 delta: the same delta written into the quantisation-only format
    (pruned columns carry the zero-point as their code) goes through dz_qsbmm at the dense rate and must
    match both the oracle and, to rounding, dz_sbmm on the 2:4 blob."""
    T, N, K, D, bits, G = 48, 128, 1024, 3, 4, 128
    x = S.make_x(T, K, S.stream(44, "x"))
    ids = _ids("uniform", T, D, 44)
    tabs = [S.make_delta_tables(N, K, bits, G, S.stream(44, "delta", m)) for m in range(D)]
    dense = [oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G) for t in tabs]
    want = oracle.c.linear(x.numpy(), None, dense, ids.numpy())
    with dz.Context(0) as c:
        sp, qp = [], []
        for t in tabs:
            d = t.to("cuda")
            p = torch.empty(dz.dz_packed_bytes(N, K, bits, G), dtype=torch.uint8, device="cuda")
            dz.dz_pack_delta(c.h, d.codes, d.idx, d.scale, d.zero, N, K, bits, G, p)
            sp.append(p)
            codes = np.repeat(t.zero.numpy().astype(np.uint8), G, axis=1)
            cols = (np.arange(K // 2) // 2 * 4)[None, :] + t.idx.numpy().astype(np.int64)
            np.put_along_axis(codes, cols, t.codes.numpy(), axis=1)
            q = torch.empty(dz.dz_qpacked_bytes(N, K, bits, G), dtype=torch.uint8, device="cuda")
            dz.dz_qpack_delta(c.h, torch.from_numpy(codes).cuda(), d.scale, d.zero, N, K, bits, G, q)
            qp.append(q)
        o_s = torch.empty(T, N, dtype=torch.float16, device="cuda")
        o_q = torch.empty(T, N, dtype=torch.float16, device="cuda")
        dz.dz_sbmm(c.h, x.cuda(), sp, ids.cuda(), o_s, T, N, K, bits, G, 0)
        dz.dz_qsbmm(c.h, x.cuda(), qp, ids.cuda(), o_q, T, N, K, bits, G, 0)
        torch.cuda.synchronize()
        assert_close(o_s, want, "2:4 blob")
        assert_close(o_q, want, "the same delta, dense-expanded")
        # identical dequantised values, identical k order inside a step: the two differ by summation order only
        assert (o_s.float() - o_q.float()).abs().max().item() <= 2.0 ** -9 * float(np.abs(want).max())
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_argument_errors(dz):
    with dz.Context(0) as c:
        z = torch.zeros(16 * 256, dtype=torch.uint8, device="cuda")
        h = torch.zeros(64, dtype=torch.float16, device="cuda")
        assert dz.dz_qpacked_bytes(256, 256, 3, 64) == 0 and dz.dz_qpacked_bytes(250, 256, 4, 64) == 0
        assert dz.dz_qpack_delta(c.h, z, h, h, 16, 256, 3, 64, z, check=False) == dz.DZ_ERR_BITS
        assert dz.dz_qpack_delta(c.h, z, h, h, 16, 200, 4, 64, z, check=False) == dz.DZ_ERR_SHAPE
        assert dz.dz_qpack_delta(c.h, z, h, h, 16, 256, 4, 64, z[1:], check=False) == dz.DZ_ERR_ALIGN
        assert dz.dz_qunpack_delta(c.h, None, 16, 256, 4, 64, check=False) == dz.DZ_ERR_ARG
        assert dz.dz_merge_delta(c.h, None, z, 16, 256, 4, 64, z, check=False) == dz.DZ_ERR_ARG
