"""GPU: the compute calls can be recorded into a HIP graph and replayed (serving loops replay a
decode step that way).  After one eager call at the same shapes the library allocates nothing and
never synchronises, so a capture holds only its kernels; every replay -- with new activations
written into the same buffers and eager work in between -- must match the CPU oracle like the
eager call does (paper Section 5.1 Eq. (2) per projection)."""
import numpy as np
import pytest
import torch

import dz_synth as S
from dzcase import Case, assert_close

pytestmark = pytest.mark.gpu

SHAPES = [
    # name,      T,   K,   D, bits, G,  ids,        N of each projection
    ("decode",   32, 1024, 8, 4, 128, "uniform",  [256, 64, 64]),
    ("tiled",   150,  512, 6, 4, 128, "segments", [128, 64]),
    ("decode2",  64,  768, 5, 2,  64, "zipf",     [96]),
]


@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_replays_match_oracle(dz, shape):
    import oracle
    name, T, K, D, bits, G, ids, Ns = shape
    print(f"graph {name}", flush=True)
    with dz.Context(0) as c:
        cases = [Case(dz, c.h, 40 + p, T, N, K, D, bits, G, ids) for p, N in enumerate(Ns)]
        x0, idv = cases[0].x, cases[0].ids
        dx, dids = cases[0].dx, cases[0].dids
        outs = [cs.out(fill=7.0) for cs in cases]
        sb = cases[0].out(fill=7.0)          # dz_sbmm of the first projection rides along

        def calls():
            if len(cases) > 1:
                dz.dz_linear_group(c.h, dx, [cs.dW for cs in cases], [cs.packed for cs in cases], dids, outs, T, Ns, K,
                                   bits, G)
            else:
                dz.dz_linear(c.h, dx, cases[0].dW, cases[0].packed, dids, outs[0], T, Ns[0], K, bits, G)
            dz.dz_sbmm(c.h, dx, cases[0].packed, dids, sb, T, Ns[0], K, bits, G, accumulate=0)

        def check(x, what):
            assert dz.dz_check(c.h) == dz.DZ_OK
            for p, cs in enumerate(cases):
                assert_close(outs[p], oracle.c.linear(x.numpy(), cs.W.numpy(), cs.dense, idv.numpy()), f"{name} {what} p{p}")
            assert_close(sb, oracle.c.linear(x.numpy(), None, cases[0].dense, idv.numpy()), f"{name} {what} sbmm")

        calls()                              # eager: sizes the workspace
        torch.cuda.synchronize()
        check(x0, "eager")

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            calls()
        for rep in range(3):
            x = S.make_x(T, K, S.stream(90 + rep, "x"))
            dx.copy_(x)                      # new activations, same buffers
            for o in outs + [sb]:
                o.fill_(7.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            check(x, f"replay {rep}")
            # eager work of the same context between replays
            dx.copy_(x0)
            calls()
            torch.cuda.synchronize()
            check(x0, f"eager after replay {rep}")


def test_growth_during_capture_is_an_error(dz):
    """A call that would have to grow the workspace cannot do so inside a capture: it reports a
    runtime failure, leaves the capture valid, and works again outside."""
    with dz.Context(0) as c:
        small = Case(dz, c.h, 50, 8, 32, 256, 2, 4, 64, "uniform")
        o = small.out()
        dz.dz_linear(c.h, small.dx, small.dW, small.packed, small.dids, o, 8, 32, 256, 4, 64)
        torch.cuda.synchronize()
        big = Case(dz, c.h, 51, 5000, 32, 256, 2, 4, 64, "segments")     # needs a larger segment workspace
        ob = big.out()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ob.zero_()
            rc = dz.dz_linear(c.h, big.dx, big.dW, big.packed, big.dids, ob, 5000, 32, 256, 4, 64, check=False)
        assert rc == dz.DZ_ERR_HIP
        msg = dz.dz_strerror(rc)                     # the runtime's own text travels with the code
        assert msg.startswith("HIP runtime failure: ") and len(msg) > len("HIP runtime failure: "), msg
        assert dz.lib().dz_last_hip_error(c.h).decode() in msg
        torch.cuda.synchronize()
        dz.dz_linear(c.h, big.dx, big.dW, big.packed, big.dids, ob, 5000, 32, 256, 4, 64)
        assert dz.dz_check(c.h) == dz.DZ_OK
        assert_close(ob, big.y, "after failed capture")


def test_replay_after_the_workspace_grew(dz):
    """A graph recorded before the workspace grows still replays correctly afterwards: the buffers a
    growth replaces stay allocated until dz_destroy (the graph's kernel nodes hold their addresses)."""
    import oracle
    with dz.Context(0) as c:
        c.set_option(dz.DZ_OPT_SPLIT_K, 3)               # split k: the launch uses partial sums and counters
        small = Case(dz, c.h, 52, 32, 96, 1536, 4, 4, 128, "uniform")
        o = small.out(fill=7.0)
        dz.dz_linear(c.h, small.dx, small.dW, small.packed, small.dids, o, 32, 96, 1536, 4, 128)
        torch.cuda.synchronize()
        assert_close(o, small.y, "eager")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            dz.dz_linear(c.h, small.dx, small.dW, small.packed, small.dids, o, 32, 96, 1536, 4, 128)
        # an eager call whose partial sums exceed the initial workspace (8 slices x 64 x 20480 x 4 bytes = 40 MiB)
        c.set_option(dz.DZ_OPT_SPLIT_K, 8)
        T, N, K = 64, 20480, 2048
        W = S.make_base(N, K, S.stream(53, "W"), 0.02).cuda()
        x = S.make_x(T, K, S.stream(53, "x")).cuda()
        big = torch.empty(T, N, dtype=torch.float16, device="cuda")
        print("growing the workspace", flush=True)
        dz.dz_base_gemm(c.h, x, W, big, T, N, K)
        assert dz.dz_check(c.h) == dz.DZ_OK
        rows = torch.arange(0, N, 997, device="cuda")
        assert_close(big[:, rows], oracle.c.linear(x.cpu().numpy(), W[rows].cpu().numpy(), None, None), "big base")
        for rep in range(2):
            xn = S.make_x(32, 1536, S.stream(54 + rep, "x"))
            small.dx.copy_(xn)
            o.fill_(7.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert dz.dz_check(c.h) == dz.DZ_OK
            assert_close(o, oracle.c.linear(xn.numpy(), small.W.numpy(), small.dense, small.ids.numpy()), f"replay {rep} after growth")
