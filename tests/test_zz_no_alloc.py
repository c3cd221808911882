"""GPU: dz_linear_static -- the fused linear layer on the library's static device workspace, for
callers that cannot allocate -- against dz_linear on the same inputs, through the C ABI.  Both run
the same kernels with the same decomposition, so the outputs must be identical bit for bit; the
oracle bounds both.  Two calls in a row, the second with a smaller input (the static workspace
keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from dzcase import Case, assert_close

pytestmark = pytest.mark.gpu


def _both(dz, c, cs, tag):
    ref = cs.out(fill=7.0)
    dz.dz_linear(c.h, cs.dx, cs.dW, cs.packed, cs.dids, ref, cs.T, cs.N, cs.K, cs.bits, cs.G)
    got = cs.out(fill=5.0)
    dz.dz_linear_static(0, cs.dx, cs.dW, cs.packed, cs.dids, got, cs.T, cs.N, cs.K, cs.bits, cs.G)
    assert dz.dz_check(c.h) == dz.DZ_OK
    assert_close(got, cs.y, tag + " static vs oracle")
    assert_close(ref, cs.y, tag + " context vs oracle")
    assert torch.equal(got, ref), tag


def test_static_entry_point_matches_dz_linear(dz):
    with dz.Context(0) as c:
        # split k on both (partial sums and counters in use), then a smaller call right after
        first = Case(dz, c.h, 80, 64, 272, 2048, 4, 4, 128, "uniform")
        second = Case(dz, c.h, 81, 17, 96, 1024, 5, 2, 64, "zipf")
        print("static: first call", flush=True)
        _both(dz, c, first, "first")
        print("static: second, smaller call", flush=True)
        _both(dz, c, second, "second")
        print("static: first again", flush=True)
        _both(dz, c, first, "first again")
        # an index outside [-1, D) is served base-only and reported by dz_check
        bad = first.ids.clone(); bad[5] = 9
        got = first.out()
        dz.dz_linear_static(0, first.dx, first.dW, first.packed, bad.cuda(), got, first.T, first.N, first.K, first.bits, first.G)
        assert dz.dz_check(c.h) == dz.DZ_ERR_INDEX
        assert dz.dz_check(c.h) == dz.DZ_OK
        # limits: larger batches and partial sums beyond the static array are refused
        assert dz.dz_linear_static(0, first.dx, first.dW, first.packed, first.dids, got, 65, first.N, first.K, first.bits,
                                   first.G, check=False) == dz.DZ_ERR_LIMIT
        # 71744 x 512 at 64 rows: two workgroups share every row block, 2 x 64 x 71744 x 4 bytes = 35 MiB of
        # partial sums against the array's 32 MiB (real buffers of that size, so the call is legal either way)
        T, N, K = 64, 71744, 512
        W = torch.zeros(N, K, dtype=torch.float16, device="cuda")
        x = torch.zeros(T, K, dtype=torch.float16, device="cuda")
        o = torch.empty(T, N, dtype=torch.float16, device="cuda")
        ids = torch.full((T,), -1, dtype=torch.int32, device="cuda")
        assert dz.dz_linear_static(0, x, W, [], ids, o, T, N, K, 4, 128, check=False) == dz.DZ_ERR_LIMIT
        dz.dz_linear(c.h, x, W, [], ids, o, T, N, K, 4, 128)       # the context's workspace grows instead
        assert dz.dz_check(c.h) == dz.DZ_OK
