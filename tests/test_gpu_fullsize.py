"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.

Inputs are generated on the GPU with the seeded generator; the oracle cannot redo a whole layer
in seconds, so it recomputes a sample of output features (rows of W and of every delta, chosen to
include tile and matrix edges) for ALL requests, from canonical tables copied back to the host.
Rows are independent of each other in the definition (paper Section 5.1 Eq. (2)), so a row subset
is itself a complete, smaller instance of the problem."""
import numpy as np
import pytest
import torch

import dz_synth as S
import oracle
from dzcase import assert_close

pytestmark = pytest.mark.gpu

CASES = [
    ("7b_decode", 4096, 4096), ("7b_decode", 11008, 4096), ("7b_decode", 4096, 11008),
    ("7b_decode_many", 4096, 4096), ("7b_decode_many", 4096, 11008),
    ("13b_prefill", 5120, 5120), ("13b_prefill", 13824, 5120), ("13b_prefill", 5120, 13824),
    ("70b_stack", 8192, 8192), ("70b_stack", 1024, 8192), ("70b_stack", 28672, 8192), ("70b_stack", 8192, 28672),
]


def _sample_rows(N, n=48, seed=0):
    g = np.random.default_rng(seed)
    fixed = [0, 1, 15, 16, 17, 127, 128, 129, N // 2 - 1, N // 2, N - 129, N - 128, N - 17, N - 16, N - 1]
    rnd = g.choice(N, size=n, replace=False).tolist()
    return sorted(set(int(r) for r in fixed + rnd if 0 <= r < N))


@pytest.mark.parametrize("cfgname,N,K", CASES, ids=[f"{c}-{n}x{k}" for c, n, k in CASES])
def test_fullsize_sampled_rows(dz, cfgname, N, K):
    print(f"case {cfgname} {N}x{K}", flush=True)
    cfg = S.config(cfgname)
    with dz.Context(0) as c:
        p = S.make_projection(cfg, 0, 0, f"full{N}x{K}", N, K, device="cuda")
        ids = cfg.make_ids(S.stream(0, cfg.name, "ids"))
        d_ids = ids.cuda()
        nbytes = dz.dz_packed_bytes(N, K, cfg.bits, cfg.group)
        packed = []
        for t in p.tabs:
            buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            dz.dz_pack_delta(c.h, t.codes, t.idx, t.scale, t.zero, N, K, cfg.bits, cfg.group, buf)
            packed.append(buf)
        out = torch.full((cfg.T, N), 7.0, dtype=torch.float16, device="cuda")
        dz.dz_linear(c.h, p.x, p.W, packed, d_ids, out, cfg.T, N, K, cfg.bits, cfg.group)
        assert dz.dz_check(c.h) == dz.DZ_OK
        assert torch.isfinite(out.float()).all()
        rows = _sample_rows(N)
        ridx = torch.as_tensor(rows, device="cuda")
        Wn = p.W[ridx].cpu().numpy()
        xn = p.x.cpu().numpy()
        dense = []
        for t in p.tabs:
            s = t.rows(ridx).to("cpu")
            assert oracle.c.validate(s.codes.numpy(), s.idx.numpy(), s.scale.numpy(), s.zero.numpy(), cfg.bits, cfg.group) == 0
            dense.append(oracle.c.dequant(s.codes.numpy(), s.idx.numpy(), s.scale.numpy(), s.zero.numpy(), cfg.bits, cfg.group))
        ref = oracle.c.linear(xn, Wn, dense, ids.numpy())
        got = out[:, ridx]
        max_rel, mean_abs = assert_close(got, ref, f"{cfgname} {N}x{K}")
        print(f"  max_rel={max_rel:.2e} mean_abs={mean_abs:.2e}", flush=True)
        # the delta term really is in there: compare against the base-only oracle too
        ref_base = oracle.c.linear(xn, Wn, None, None)
        assert np.abs(ref - ref_base).max() > 10 * np.abs(got.float().cpu().numpy() - ref).max()


@pytest.mark.parametrize("N,K", [(5120, 5120), (13824, 5120), (5120, 13824)], ids=lambda v: str(v))
def test_fullsize_base_product_of_the_prefill_batch(dz, N, K):
    """dz_base_gemm alone at the prefill workload's sizes (the route bench.py --path base times: the
    256 x 256 tile kernel where it has enough tiles), sampled output features against the oracle."""
    print(f"case 13b_prefill base {N}x{K}", flush=True)
    cfg = S.config("13b_prefill")
    with dz.Context(0) as c:
        W = S.make_base(N, K, S.stream(3, "W", N, K), 0.02).cuda()
        x = S.make_x(cfg.T, K, S.stream(3, "x", K)).cuda()
        out = torch.full((cfg.T, N), 7.0, dtype=torch.float16, device="cuda")
        dz.dz_base_gemm(c.h, x, W, out, cfg.T, N, K)
        assert dz.dz_check(c.h) == dz.DZ_OK
        assert torch.isfinite(out.float()).all()
        rows = _sample_rows(N)
        ridx = torch.as_tensor(rows, device="cuda")
        ref = oracle.c.linear(x.cpu().numpy(), W[ridx].cpu().numpy(), None, None)
        max_rel, mean_abs = assert_close(out[:, ridx], ref, f"base {N}x{K}")
        print(f"  max_rel={max_rel:.2e} mean_abs={mean_abs:.2e}", flush=True)
