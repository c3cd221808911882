"""GPU parity: dz_base_gemm, dz_sbmm and dz_linear against the CPU oracle on the same seeded inputs
(paper Section 5.1 Eq. (2), Section 5.2).  Sizes the oracle finishes in seconds, chosen to span
several row tiles, k tiles, column blocks, split and unsplit k, and ragged request counts."""
import numpy as np
import pytest
import torch

import dz_synth as S
from dzcase import Case, assert_close

pytestmark = pytest.mark.gpu

CASES = [
    # name,            T,   N,    K,   D, bits, G,  ids
    ("tiny",           8,  256,  256,  4, 4,  64, "uniform"),
    ("b4g128_t32",    32,   96, 1024,  8, 4, 128, "uniform"),
    ("b2g128_t64z",   64,  160, 1536, 32, 2, 128, "zipf"),
    ("b2g64_t7",       7,   48,  768,  3, 2,  64, "uniform"),
    ("b4g64_t1",       1,   32,  512,  2, 4,  64, "uniform"),
    ("b4g128_t17",    17,  208,  512,  5, 4, 128, "uniform"),
    ("b4g128_t100",  100,   64, 1024,  6, 4, 128, "uniform"),
    ("b2g128_t200s", 200,  128,  512,  7, 2, 128, "segments"),
    ("b4g128_t64u4",  64,  272, 2048,  4, 4, 128, "uniform"),
]


def _run_all(dz, c, cs, tag):
    o = cs.out(fill=7.0)
    dz.dz_base_gemm(c.h, cs.dx, cs.dW, o, cs.T, cs.N, cs.K)
    assert_close(o, cs.y_base, tag + " base")
    o = cs.out(fill=7.0)
    dz.dz_sbmm(c.h, cs.dx, cs.packed, cs.dids, o, cs.T, cs.N, cs.K, cs.bits, cs.G, 0)
    assert_close(o, cs.y_delta, tag + " sbmm")
    o = cs.out(fill=7.0)
    dz.dz_linear(c.h, cs.dx, cs.dW, cs.packed, cs.dids, o, cs.T, cs.N, cs.K, cs.bits, cs.G)
    r = assert_close(o, cs.y, tag + " linear")
    # accumulate: base first, then out += delta part (two roundings)
    o2 = cs.out()
    dz.dz_base_gemm(c.h, cs.dx, cs.dW, o2, cs.T, cs.N, cs.K)
    dz.dz_sbmm(c.h, cs.dx, cs.packed, cs.dids, o2, cs.T, cs.N, cs.K, cs.bits, cs.G, 1)
    assert_close(o2, cs.y, tag + " base then sbmm(accumulate)")
    assert dz.dz_check(c.h) == dz.DZ_OK
    return r


@pytest.mark.parametrize("splits", ["auto", "1", "3"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_parity_small(dz, case, splits):
    name, T, N, K, D, bits, G, ids = case
    print(f"case {name} splits={splits}", flush=True)
    with dz.Context(0) as c:
        if splits != "auto":
            c.set_option(dz.DZ_OPT_SPLIT_K, int(splits))
        cs = Case(dz, c.h, 0, T, N, K, D, bits, G, ids)
        max_rel, mean_abs = _run_all(dz, c, cs, name)
        print(f"  linear max_rel={max_rel:.2e} mean_abs={mean_abs:.2e}", flush=True)


def test_single_rounding_is_tight(dz):
    """fp32 accumulation and one rounding: every output is within about one fp16 step of the
    oracle value, and most equal its fp16 rounding (the kernels round each dequantised delta value to fp16,
    a 2^-11 relative perturbation of the delta term, which moves a few results across a rounding
    boundary)."""
    with dz.Context(0) as c:
        cs = Case(dz, c.h, 3, 32, 96, 1024, 8, 4, 128, "uniform")
        o = cs.out()
        dz.dz_linear(c.h, cs.dx, cs.dW, cs.packed, cs.dids, o, cs.T, cs.N, cs.K, cs.bits, cs.G)
        torch.cuda.synchronize()
        ref16 = torch.from_numpy(cs.y).to(torch.float16)
        same = (o.cpu() == ref16).float().mean().item()
        assert same > 0.85, same
        ref = torch.from_numpy(cs.y).double()
        rms = ref.pow(2).mean().sqrt()
        rel = ((o.cpu().double() - ref).abs() / torch.maximum(ref.abs(), rms)).max().item()
        assert rel <= 2.0 ** -9, rel          # about one fp16 step at the output's own magnitude


def test_base_only_requests_and_bad_indices(dz):
    with dz.Context(0) as c:
        T, N, K, D = 12, 64, 512, 3
        ids = np.array([0, -1, 2, 1, -1, -1, 0, 2, 2, -1, 1, 0], np.int32)
        cs = Case(dz, c.h, 5, T, N, K, D, 4, 128, ids)
        _run_all(dz, c, cs, "minus-one")
        base_rows = torch.as_tensor(ids == -1)
        o = cs.out(fill=7.0)
        dz.dz_sbmm(c.h, cs.dx, cs.packed, cs.dids, o, T, N, K, 4, 128, 0)
        torch.cuda.synchronize()
        assert (o.cpu()[base_rows] == 0).all()
        # all requests base-only
        cs2 = Case(dz, c.h, 6, 5, N, K, D, 4, 128, np.full(5, -1, np.int32))
        _run_all(dz, c, cs2, "all-base")
        # an index outside [-1, D): served base-only, reported by dz_check
        bad = ids.copy(); bad[3] = 3; bad[7] = -2
        cs3 = Case(dz, c.h, 5, T, N, K, D, 4, 128, bad)
        o = cs3.out()
        dz.dz_linear(c.h, cs3.dx, cs3.dW, cs3.packed, cs3.dids, o, T, N, K, 4, 128)
        assert_close(o, cs3.y, "bad ids")          # the oracle treats them as base-only too
        assert dz.dz_check(c.h) == dz.DZ_ERR_INDEX
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_degenerate_calls(dz):
    with dz.Context(0) as c:
        cs = Case(dz, c.h, 7, 4, 32, 256, 2, 4, 64, "uniform")
        o = cs.out(fill=3.0)
        # T == 0: nothing happens
        assert dz.dz_linear(c.h, cs.dx, cs.dW, cs.packed, cs.dids, o, 0, cs.N, cs.K, 4, 64) == dz.DZ_OK
        torch.cuda.synchronize()
        assert (o == 3.0).all()
        # D == 0: the base product alone; SBMM gives zeros
        dz.dz_linear(c.h, cs.dx, cs.dW, [], cs.dids, o, cs.T, cs.N, cs.K, 4, 64)
        assert_close(o, cs.y_base, "D=0 linear")
        dz.dz_sbmm(c.h, cs.dx, [], cs.dids, o, cs.T, cs.N, cs.K, 4, 64, 0)
        torch.cuda.synchronize()
        assert (o == 0).all()
        # argument errors
        assert dz.dz_linear(c.h, cs.dx, cs.dW, cs.packed, cs.dids, o, cs.T, cs.N, 200, 4, 64, check=False) == dz.DZ_ERR_SHAPE
        assert dz.dz_linear(c.h, cs.dx, cs.dW, cs.packed, cs.dids, o, cs.T, cs.N, cs.K, 3, 64, check=False) == dz.DZ_ERR_BITS
        assert dz.dz_linear(c.h, cs.dx, None, cs.packed, cs.dids, o, cs.T, cs.N, cs.K, 4, 64, check=False) == dz.DZ_ERR_ARG
        assert dz.dz_linear(c.h, cs.dx, cs.dW, cs.packed * 65, cs.dids, o, cs.T, cs.N, cs.K, 4, 64, check=False) == dz.DZ_ERR_ARG
        assert dz.dz_base_gemm(c.h, cs.dx.view(-1)[1:], cs.dW, o, 1, cs.N, cs.K, check=False) == dz.DZ_ERR_ALIGN
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_maximum_tables(dz):
    """The sizes that fill the kernels' tables: DZ_MAX_DELTAS resident deltas, 64 requests that all
    name different deltas (64 one-row segments), and a batch where every request names the same one."""
    with dz.Context(0) as c:
        T, N, K, D = 64, 32, 256, dz.DZ_MAX_DELTAS
        ids = (np.arange(T, dtype=np.int32) * 2 + 1)[::-1].copy()        # 64 distinct deltas, descending order
        cs = Case(dz, c.h, 11, T, N, K, D, 2, 64, ids)
        _run_all(dz, c, cs, "64 segments of 128 deltas")
        cs.ids = torch.full((T,), D - 1, dtype=torch.int32)
        cs.dids = cs.ids.cuda()
        import oracle
        ref = oracle.c.linear(cs.x.numpy(), cs.W.numpy(), cs.dense, cs.ids.numpy())
        o = cs.out(fill=7.0)
        dz.dz_linear(c.h, cs.dx, cs.dW, cs.packed, cs.dids, o, T, N, K, 2, 64)
        assert_close(o, ref, "one segment of 64 rows, last delta")
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_tiles_of_one_delta(dz):
    """Large batches whose 128-row tiles each belong to one delta (the fused path of the tiled
    kernel), next to tiles that mix deltas and base-only requests (the general path)."""
    with dz.Context(0) as c:
        T, N, K, D = 300, 96, 768, 3
        ids = np.concatenate([np.zeros(256, np.int32), np.full(44, 2, np.int32)])
        for bits, G in ((4, 128), (2, 64)):
            cs = Case(dz, c.h, 21, T, N, K, D, bits, G, ids)
            _run_all(dz, c, cs, f"one delta per tile b{bits}")
        # the same rows in scrambled order with base-only requests among them: after sorting, the
        # first tile is all delta 0, the second mixes delta 0 and delta 2, the third ends in rows
        # that name no delta
        rng = np.random.default_rng(5)
        ids2 = np.concatenate([np.zeros(200, np.int32), np.full(80, 2, np.int32), np.full(20, -1, np.int32)])
        rng.shuffle(ids2)
        cs = Case(dz, c.h, 22, T, N, K, D, 4, 128, ids2)
        _run_all(dz, c, cs, "mixed tiles")


@pytest.mark.parametrize("opts", [{"DZ_OPT_WIDE_TILE": 2}, {"DZ_OPT_WIDE_TILE": 2, "DZ_OPT_SPLIT_K": 3},
                                  {"DZ_OPT_WIDE_TILE": 2, "DZ_OPT_SPLIT_K": 1}, {}],
                         ids=["wide", "wide_splits3", "wide_whole", "default"])
def test_base_gemm_of_a_large_batch_over_several_tiles(dz, opts):
    """The base product of a large batch (Eq. (2), first term): several 256 x 256 tiles with ragged
    last tiles in both directions, whole and cut into k slices (DZ_OPT_WIDE_TILE = 2 sends every such
    call to the 256 x 256 kernel, which by default only takes calls with many tiles), and the default
    route."""
    import oracle
    T, N, K = 600, 784, 1024
    print(f"wide base gemm {opts}", flush=True)
    with dz.Context(0) as c:
        for k, v in opts.items():
            c.set_option(getattr(dz, k), v)
        W = S.make_base(N, K, S.stream(70, "W"), 0.02)
        x = S.make_x(T, K, S.stream(70, "x"))
        ref = oracle.c.linear(x.numpy(), W.numpy(), None, None)
        o = torch.full((T, N), 7.0, dtype=torch.float16, device="cuda")
        dz.dz_base_gemm(c.h, x.cuda(), W.cuda(), o, T, N, K)
        assert dz.dz_check(c.h) == dz.DZ_OK
        assert_close(o, ref, f"base gemm {opts}")


@pytest.mark.parametrize("tiles", [1, 2, 3])
@pytest.mark.parametrize("case", [("b4g128_t32", 32, 96, 2048, 8, 4, 128, "uniform"), ("b2g128_t64z", 64, 160, 2304, 32, 2, 128, "zipf"),
                                  ("b4g64_t9", 9, 272, 2816, 3, 4, 64, "uniform"), ("b2g64_t40", 40, 48, 1792, 5, 2, 64, "uniform")],
                         ids=lambda c: c[0])
def test_short_rounds(dz, case, tiles):
    """DZ_OPT_ROUND_TILES below what the LDS buffers hold: many rounds per workgroup, so the two x buffers
    swap several times inside a row block, with and without split k."""
    name, T, N, K, D, bits, G, ids = case
    print(f"case {name} round tiles {tiles}", flush=True)
    for splits in (0, 1, 2):
        with dz.Context(0) as c:
            c.set_option(dz.DZ_OPT_ROUND_TILES, tiles)
            if splits:
                c.set_option(dz.DZ_OPT_SPLIT_K, splits)
            cs = Case(dz, c.h, 5, T, N, K, D, bits, G, ids)
            _run_all(dz, c, cs, f"{name} round tiles {tiles} splits {splits}")


def test_options_are_validated(dz):
    with dz.Context(0) as c:
        assert c.set_option(dz.DZ_OPT_SPLIT_K, 3) == dz.DZ_OK
        assert dz.dz_set_option(c.h, dz.DZ_OPT_WIDE_TILE, 3, check=False) == dz.DZ_ERR_ARG
        assert dz.dz_set_option(c.h, 99, 1, check=False) == dz.DZ_ERR_ARG
        assert dz.dz_set_option(c.h, dz.DZ_OPT_SPLIT_K, -1, check=False) == dz.DZ_ERR_ARG


def test_large_batch_calls_of_one_layer_share_one_sort(dz):
    """DZ_OPT_REUSE_SEGMENTS: consecutive large-batch calls with the same index vector reuse the
    sorted order; a changed vector at another address, another T or a reset option sorts again."""
    with dz.Context(0) as c:
        c.set_option(dz.DZ_OPT_REUSE_SEGMENTS, 1)
        a = Case(dz, c.h, 31, 300, 64, 512, 5, 4, 128, "segments")
        b = Case(dz, c.h, 32, 300, 96, 512, 5, 4, 128, "uniform")
        for rep in range(2):
            for cs in (a, a, b, a):
                o = cs.out(fill=7.0)
                dz.dz_linear(c.h, cs.dx, cs.dW, cs.packed, cs.dids, o, cs.T, cs.N, cs.K, cs.bits, cs.G)
                assert_close(o, cs.y, "reuse")
        # same address, new contents: the caller must reset the option (its promise no longer holds)
        a.dids.copy_(b.dids)
        c.set_option(dz.DZ_OPT_REUSE_SEGMENTS, 1)
        import oracle
        ref = oracle.c.linear(a.x.numpy(), a.W.numpy(), a.dense, b.ids.numpy())
        o = a.out(fill=7.0)
        dz.dz_linear(c.h, a.dx, a.dW, a.packed, a.dids, o, a.T, a.N, a.K, a.bits, a.G)
        assert_close(o, ref, "after reset")
        assert dz.dz_check(c.h) == dz.DZ_OK
