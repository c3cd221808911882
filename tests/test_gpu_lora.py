"""GPU: dz_lora_sbmm against the low-rank adapter oracle, y[t] = B_m (A_m x[t]) with m = Idx[t] (paper
Section 3.2, Section 6.4; the selective batched product of Section 5.2 with a low-rank matrix in place
of a delta)."""
import numpy as np
import pytest
import torch

import dz_synth as S
import oracle
from dzcase import assert_close

pytestmark = pytest.mark.gpu


def _case(seed, T, N, K, D, r, ids="uniform", std=0.05):
    x = S.make_x(T, K, S.stream(seed, "x"))
    A = [S.make_base(r, K, S.stream(seed, "A", m), std) for m in range(D)]
    B = [S.make_base(N, r, S.stream(seed, "B", m), std) for m in range(D)]
    g = S.stream(seed, "ids")
    idv = {"uniform": lambda: S.ids_uniform(T, D, g), "zipf": lambda: S.ids_zipf(T, D, 1.5, g),
           "segments": lambda: S.ids_segments(T, D, g)}[ids]()
    return x, A, B, torch.as_tensor(np.asarray(idv), dtype=torch.int32)


CASES = [
    # name        T     N     K    D   r  ids
    ("tiny",      4,    8,   64,   2,  8, "uniform"),
    ("r16",      32,  256,  512,   4, 16, "uniform"),
    ("r64_zipf", 64, 1024, 4096,  16, 64, "zipf"),
    ("ragged",   37, 1028,  520,   5, 24, "uniform"),       # N not a multiple of the 1024-wide block, K of 512
    ("t1",        1, 4096, 4096,   3, 16, "uniform"),
    ("t300",    300,  132, 1024,   7,  8, "segments"),
    ("wide",     16, 13824, 5120,  8, 16, "uniform"),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_parity(dz, case):
    name, T, N, K, D, r, ids = case
    print(f"case {name}", flush=True)
    x, A, B, idv = _case(21, T, N, K, D, r, ids)
    if T > 3:
        idv[2] = -1                                 # a request with no adapter
    want = oracle.lora.lora_sbmm(x.numpy(), [a.numpy() for a in A], [b.numpy() for b in B], idv.numpy())
    with dz.Context(0) as c:
        dA, dB = [a.cuda() for a in A], [b.cuda() for b in B]
        out = torch.full((T, N), 7.0, dtype=torch.float16, device="cuda")
        dz.dz_lora_sbmm(c.h, x.cuda(), dA, dB, r, idv.cuda(), out, T, N, K, 0)
        torch.cuda.synchronize()
        max_rel, mean_abs = assert_close(out, want, name)
        print(f"  max_rel={max_rel:.2e} mean_abs={mean_abs:.2e}", flush=True)
        if T > 3:
            assert not out[2].any()
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_accumulate_completes_a_base_product(dz):
    """out = x W^T first, then out += B_m A_m x: equals the oracle's linear layer with the dense update
    B_m A_m in the delta's place (two roundings, inside the tolerance)."""
    T, N, K, D, r = 24, 192, 1024, 3, 16
    x, A, B, idv = _case(22, T, N, K, D, r, std=0.02)
    W = S.make_base(N, K, S.stream(22, "W"), 0.02)
    dense = [oracle.lora.dense_update(a.numpy(), b.numpy()).astype(np.float32) for a, b in zip(A, B)]
    want = oracle.c.linear(x.numpy(), W.numpy(), dense, idv.numpy())
    with dz.Context(0) as c:
        out = torch.empty(T, N, dtype=torch.float16, device="cuda")
        dz.dz_base_gemm(c.h, x.cuda(), W.cuda(), out, T, N, K)
        dz.dz_lora_sbmm(c.h, x.cuda(), [a.cuda() for a in A], [b.cuda() for b in B], r, idv.cuda(), out, T, N, K, 1)
        torch.cuda.synchronize()
        assert_close(out, want, "base then lora(accumulate)")


def test_adapters_beside_deltas_in_one_batch(dz):
    """A batch that mixes delta-served and adapter-served requests (Section 3.2): dz_linear with the delta
    indices (adapter requests carry -1 there), then dz_lora_sbmm accumulating with the adapter indices."""
    T, N, K, D, r, bits, G = 32, 96, 1024, 3, 8, 4, 128
    x, A, B, _ = _case(23, T, N, K, D, r, std=0.02)
    W = S.make_base(N, K, S.stream(23, "W"), 0.02)
    tabs = [S.make_delta_tables(N, K, bits, G, S.stream(23, "delta", m)) for m in range(D)]
    which = S.ids_uniform(T, 2 * D, S.stream(23, "which")).numpy()
    delta_ids = np.where(which < D, which, -1).astype(np.int32)
    lora_ids = np.where(which >= D, which - D, -1).astype(np.int32)
    dense_d = [oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G) for t in tabs]
    dense_l = [oracle.lora.dense_update(a.numpy(), b.numpy()).astype(np.float32) for a, b in zip(A, B)]
    want = oracle.c.linear(x.numpy(), W.numpy(), dense_d + dense_l, which.astype(np.int32))
    with dz.Context(0) as c:
        packed = []
        for t in tabs:
            dt = t.to("cuda")
            p = torch.empty(dz.dz_packed_bytes(N, K, bits, G), dtype=torch.uint8, device="cuda")
            dz.dz_pack_delta(c.h, dt.codes, dt.idx, dt.scale, dt.zero, N, K, bits, G, p)
            packed.append(p)
        out = torch.empty(T, N, dtype=torch.float16, device="cuda")
        dx = x.cuda()
        dz.dz_linear(c.h, dx, W.cuda(), packed, torch.from_numpy(delta_ids).cuda(), out, T, N, K, bits, G)
        dz.dz_lora_sbmm(c.h, dx, [a.cuda() for a in A], [b.cuda() for b in B], r, torch.from_numpy(lora_ids).cuda(), out,
                        T, N, K, 1)
        torch.cuda.synchronize()
        assert_close(out, want, "deltas and adapters in one batch")
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_argument_errors_and_bad_indices(dz):
    with dz.Context(0) as c:
        T, N, K, r = 4, 8, 64, 8
        x, A, B, idv = _case(24, T, N, K, 2, r)
        dA, dB = [a.cuda() for a in A], [b.cuda() for b in B]
        out = torch.zeros(T, N, dtype=torch.float16, device="cuda")
        dx, did = x.cuda(), idv.cuda()
        assert dz.dz_lora_sbmm(c.h, dx, dA, dB, 12, did, out, T, N, K, check=False) == dz.DZ_ERR_SHAPE
        assert dz.dz_lora_sbmm(c.h, dx, dA, dB, 72, did, out, T, N, K, check=False) == dz.DZ_ERR_SHAPE
        assert dz.dz_lora_sbmm(c.h, dx, dA, dB, r, did, out, T, N, 60, check=False) == dz.DZ_ERR_SHAPE
        assert dz.dz_lora_sbmm(c.h, dx, dA, dB, r, did, out, T, 6, K, check=False) == dz.DZ_ERR_SHAPE
        assert dz.dz_lora_sbmm(c.h, None, dA, dB, r, did, out, T, N, K, check=False) == dz.DZ_ERR_ARG
        assert dz.dz_lora_sbmm(c.h, dx, dA, dB, r, did, out, 0, N, K, check=False) == dz.DZ_OK      # empty batch
        bad = torch.tensor([0, 5, 1, -1], dtype=torch.int32, device="cuda")
        dz.dz_lora_sbmm(c.h, dx, dA, dB, r, bad, out, T, N, K)
        torch.cuda.synchronize()
        assert not out[1].any() and not out[3].any()
        assert dz.dz_check(c.h) == dz.DZ_ERR_INDEX
