"""GPU parity on seeded random shapes: dz_base_gemm, dz_sbmm, dz_linear (and the accumulate form) against
the CPU oracle (paper Section 5.1 Eq. (2), Section 5.2) on shapes nobody picked by hand -- batch sizes
around the points where the library changes kernels (64 / 65 rows) or tile counts (multiples of 16 and
128), ragged row counts of N, odd numbers of k tiles, request vectors with base-only (-1) entries and
deltas nobody names.  Every case is a valid call; sizes are kept to what the oracle does in about a second."""
import numpy as np
import pytest
import torch

import dz_synth as S
from dzcase import Case, assert_close
from test_gpu_linear import _run_all

pytestmark = pytest.mark.gpu

T_CHOICES = [1, 2, 15, 16, 17, 31, 33, 48, 63, 64, 65, 80, 127, 128, 129, 191, 257, 300]


def _draw(i):
    r = np.random.default_rng(20231205 + i)
    T = int(r.choice(T_CHOICES))
    N = 16 * int(r.integers(1, 26))                 # 16 .. 400: one to several row blocks, ragged last block
    K = 256 * int(r.integers(1, 10))                # 1 .. 9 k tiles
    while T * N * K > 60_000_000:                   # keep the oracle to about a second per product
        K = max(256, K - 256)
        if K == 256:
            N = max(16, N - 64)
    D = int(r.choice([0, 1, 2, 3, 5, 8, 13, 24, 40]))
    bits = int(r.choice([2, 4]))
    G = int(r.choice([64, 128]))
    kind = str(r.choice(["uniform", "zipf", "segments", "holes"]))
    return T, N, K, D, bits, G, kind


def _ids(kind, T, D, seed):
    g = S.stream(seed, "ids")
    if D == 0:
        return np.full(T, -1, np.int32)
    if kind == "uniform":
        return S.ids_uniform(T, D, g)
    if kind == "zipf":
        return S.ids_zipf(T, D, 1.5, g)
    if kind == "segments":
        return S.ids_segments(T, D, g)
    # holes: a third of the requests take the base model only, and only every other delta is named
    r = np.random.default_rng(seed)
    ids = r.integers(0, max(1, (D + 1) // 2), size=T).astype(np.int32) * 2
    ids = np.minimum(ids, D - 1)
    ids[r.random(T) < 0.33] = -1
    return ids


@pytest.mark.parametrize("i", range(24))
def test_random_shape(dz, i):
    T, N, K, D, bits, G, kind = _draw(i)
    tag = f"random[{i}] T={T} N={N} K={K} D={D} bits={bits} G={G} ids={kind}"
    print(tag, flush=True)
    with dz.Context(0) as c:
        cs = Case(dz, c.h, 1000 + i, T, N, K, D, bits, G, _ids(kind, T, D, 1000 + i))
        max_rel, mean_abs = _run_all(dz, c, cs, tag)
        print(f"  linear max_rel={max_rel:.2e} mean_abs={mean_abs:.2e}", flush=True)


@pytest.mark.parametrize("i", range(24, 32))
def test_random_shape_through_the_streaming_kernel_at_any_batch_size(dz, i):
    """The same sweep with large batches forced through the streaming kernel, 64 rows at a time."""
    T, N, K, D, bits, G, kind = _draw(i)
    T = max(T, 65 + 7 * (i - 24))
    while T * N * K > 60_000_000:
        N = max(16, N - 64)
    tag = f"random-streaming[{i}] T={T} N={N} K={K} D={D} bits={bits} G={G} ids={kind}"
    print(tag, flush=True)
    with dz.Context(0) as c:
        c.set_option(dz.DZ_OPT_LARGE_BATCH_STREAMING, 1)
        cs = Case(dz, c.h, 2000 + i, T, N, K, D, bits, G, _ids(kind, T, D, 2000 + i))
        _run_all(dz, c, cs, tag)


@pytest.mark.parametrize("i", range(32, 44))
def test_random_group(dz, i):
    """dz_linear_group on 1..4 random projections that share x and the request vector, each against the oracle."""
    import oracle
    r = np.random.default_rng(20231205 + i)
    T, _, K, D, bits, G, kind = _draw(i)
    P = int(r.integers(1, 5))
    Ns = [16 * int(r.integers(1, 18)) for _ in range(P)]
    D = min(D, 24)
    while T * sum(Ns) * K > 80_000_000:
        K = max(256, K - 256)
        if K == 256:
            T = max(1, T // 2)
    tag = f"random-group[{i}] T={T} K={K} D={D} bits={bits} G={G} ids={kind} N={Ns}"
    print(tag, flush=True)
    with dz.Context(0) as c:
        ids = _ids(kind, T, D, 3000 + i)
        cases = [Case(dz, c.h, 3000 + 10 * i + p, T, N, K, D, bits, G, ids) for p, N in enumerate(Ns)]
        first = cases[0]
        outs = [cs.out(fill=7.0) for cs in cases]
        dz.dz_linear_group(c.h, first.dx, [cs.dW for cs in cases], [cs.packed for cs in cases], first.dids, outs, T, Ns,
                           K, bits, G)
        assert dz.dz_check(c.h) == dz.DZ_OK
        for p, cs in enumerate(cases):
            ref = oracle.c.linear(first.x.numpy(), cs.W.numpy(), cs.dense, first.ids.numpy())
            assert_close(outs[p], ref, f"{tag} projection {p}")
