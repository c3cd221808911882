"""GPU parity: dz_linear_group -- several projections that share x and the request indices, one
call -- against the CPU oracle, projection by projection (each is the linear layer of paper
Section 5.1 Eq. (2); stacking them along the output dimension changes no result)."""
import pytest
import torch

from dzcase import Case, assert_close

pytestmark = pytest.mark.gpu

GROUPS = [
    # name,          T,  K,    D, bits, G,  ids,       N of each projection
    ("qkv_b4",      32, 1024,  8, 4, 128, "uniform", [256, 64, 64]),
    ("ragged_b4",    5,  512,  3, 4,  64, "uniform", [272, 48, 128, 16]),
    ("gateup_b2",   64, 1536, 32, 2, 128, "zipf",    [160, 160]),
    ("single_b2",   17,  768,  4, 2,  64, "uniform", [208]),
    ("tiled_b4",   150,  512,  6, 4, 128, "segments", [128, 64]),
]


def _make(dz, c, g):
    name, T, K, D, bits, G, ids, Ns = g
    cases = [Case(dz, c.h, 10 + p, T, N, K, D, bits, G, ids) for p, N in enumerate(Ns)]
    # one x and one index vector for the whole group: take the first projection's
    for cs in cases[1:]:
        cs.dx, cs.dids, cs.x, cs.ids = cases[0].dx, cases[0].dids, cases[0].x, cases[0].ids
    return cases


def _oracle(cs, x, ids):
    import oracle
    return oracle.c.linear(x.numpy(), cs.W.numpy(), cs.dense, ids.numpy())


@pytest.mark.parametrize("splits", ["auto", "1", "3"])
@pytest.mark.parametrize("group", GROUPS, ids=[g[0] for g in GROUPS])
def test_group_matches_oracle(dz, group, splits):
    name, T, K, D, bits, G, ids, Ns = group
    print(f"group {name} splits={splits}", flush=True)
    with dz.Context(0) as c:
        if splits != "auto":
            c.set_option(dz.DZ_OPT_SPLIT_K, int(splits))
        cases = _make(dz, c, group)
        x, idv = cases[0].x, cases[0].ids
        outs = [cs.out(fill=7.0) for cs in cases]
        dz.dz_linear_group(c.h, cases[0].dx, [cs.dW for cs in cases], [cs.packed for cs in cases], cases[0].dids,
                           outs, T, Ns, K, bits, G)
        assert dz.dz_check(c.h) == dz.DZ_OK
        for p, cs in enumerate(cases):
            ref = _oracle(cs, x, idv)
            assert_close(outs[p], ref, f"{name} projection {p}")
            # and the single-projection entry point agrees to within the same bar
            o1 = cs.out(fill=7.0)
            dz.dz_linear(c.h, cases[0].dx, cs.dW, cs.packed, cases[0].dids, o1, T, cs.N, K, bits, G)
            assert_close(o1, ref, f"{name} projection {p} alone")
            assert (outs[p].float() - o1.float()).abs().max().item() <= 2e-2 * max(1.0, float(abs(ref).max()))


def test_group_argument_errors(dz):
    with dz.Context(0) as c:
        cs = Case(dz, c.h, 1, 4, 32, 256, 2, 4, 64, "uniform")
        o = cs.out()
        # no projections, too many projections
        assert dz.dz_linear_group(c.h, cs.dx, [], [], cs.dids, [], 4, [], 256, 4, 64, check=False) == dz.DZ_ERR_ARG
        P = dz.DZ_MAX_GROUP + 1
        assert dz.dz_linear_group(c.h, cs.dx, [cs.dW] * P, [cs.packed] * P, cs.dids, [o] * P, 4, [32] * P, 256, 4, 64,
                                  check=False) == dz.DZ_ERR_ARG
        # a projection with a shape the kernels do not take
        assert dz.dz_linear_group(c.h, cs.dx, [cs.dW, cs.dW], [cs.packed, cs.packed], cs.dids, [o, o], 4, [32, 40],
                                  256, 4, 64, check=False) == dz.DZ_ERR_SHAPE
        # T == 0 is a no-op
        assert dz.dz_linear_group(c.h, cs.dx, [cs.dW], [cs.packed], cs.dids, [o], 0, [32], 256, 4, 64) == dz.DZ_OK
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_group_at_the_pointer_limit(dz):
    """Three projections x DZ_MAX_DELTAS deltas = the most packed-delta pointers one launch carries."""
    import oracle
    with dz.Context(0) as c:
        T, K, D = 24, 256, dz.DZ_MAX_DELTAS
        g = ("limit", T, K, D, 4, 128, "uniform", [16, 32, 16])
        cases = _make(dz, c, g)
        outs = [cs.out(fill=7.0) for cs in cases]
        dz.dz_linear_group(c.h, cases[0].dx, [cs.dW for cs in cases], [cs.packed for cs in cases], cases[0].dids,
                           outs, T, g[7], K, 4, 128)
        assert dz.dz_check(c.h) == dz.DZ_OK
        for p, cs in enumerate(cases):
            assert_close(outs[p], _oracle(cs, cases[0].x, cases[0].ids), f"limit projection {p}")
        # one projection more would not fit
        P = 4
        assert dz.dz_linear_group(c.h, cases[0].dx, [cases[0].dW] * P, [cases[0].packed] * P, cases[0].dids,
                                  [outs[0]] * P, T, [16] * P, K, 4, 128, check=False) == dz.DZ_ERR_ARG
