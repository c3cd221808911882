"""GPU parity at the full sizes of the five workloads.

bench.py issues q,k,v as one dz_linear_group call, gate,up as another, and o and down as dz_linear
calls.  test_fullsize_grouped_launches makes exactly those grouped calls (same generator keys, the
first projection's x for the group, same entry point) for every workload; test_fullsize_sampled_rows
covers every projection shape through dz_linear, which is also how bench.py issues o and down.

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


def _oracle_rows(cfg, p, x, ids, rows):
    """Oracle outputs of the sampled output features `rows` of projection p for all requests."""
    ridx = torch.as_tensor(rows, device="cuda")
    Wn = p.W[ridx].cpu().numpy()
    dense = []
    for t in p.tabs:
        s = t.rows(ridx).to("cpu")
        assert oracle.c.validate(s.codes.numpy(), s.idx.numpy(), s.scale.numpy(), s.zero.numpy(), cfg.bits, cfg.group) == 0
        dense.append(oracle.c.dequant(s.codes.numpy(), s.idx.numpy(), s.scale.numpy(), s.zero.numpy(), cfg.bits, cfg.group))
    return ridx, oracle.c.linear(x.cpu().numpy(), Wn, dense, ids.numpy())


def _grouped_cases():
    out = []
    for name in ("7b_decode", "7b_decode_many", "70b_stack", "13b_prefill"):
        cfg = S.config(name)
        projs = S.projections_of(cfg)
        for g in S.launch_groups(cfg):
            if len(g) > 1:
                out.append((name, tuple(g), "+".join(str(projs[i][1]) for i in g) + f"x{projs[g[0]][2]}"))
    return out


GROUPED = _grouped_cases()


@pytest.mark.parametrize("cfgname,gidx,label", GROUPED, ids=[f"{c}-{l}" for c, _, l in GROUPED])
def test_fullsize_grouped_launches(dz, cfgname, gidx, label):
    """The launches bench.py times: one dz_linear_group call over the projections that share x, at
    full size, with the workgroup ranges crossing row-block and projection boundaries and split-k
    partial sums meeting; every projection's sampled output features against the oracle."""
    print(f"grouped {cfgname} {label}", flush=True)
    cfg = S.config(cfgname)
    projs = S.projections_of(cfg)
    ids = cfg.make_ids(S.stream(0, cfg.name, "ids"))
    d_ids = ids.cuda()
    with dz.Context(0) as c:
        sel = []
        for i in gidx:
            name, N, K = projs[i]
            p = S.make_projection(cfg, 0, 0, name, N, K, device="cuda")
            nbytes = dz.dz_packed_bytes(N, K, cfg.bits, cfg.group)
            packed = []
            for t in p.tabs:
                buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
                dz.dz_pack_delta(c.h, t.codes, t.idx, t.scale, t.zero, N, K, cfg.bits, cfg.group, buf)
                packed.append(buf)
            sel.append((p, packed, torch.full((cfg.T, N), 7.0, dtype=torch.float16, device="cuda")))
        x = sel[0][0].x                       # bench.py: the first projection's x stands for the shared input
        K = sel[0][0].K
        dz.dz_linear_group(c.h, x, [p.W for p, _, _ in sel], [pk for _, pk, _ in sel], d_ids, [o for _, _, o in sel],
                           cfg.T, [p.N for p, _, _ in sel], K, cfg.bits, cfg.group)
        assert dz.dz_check(c.h) == dz.DZ_OK
        for j, (p, _, o) in enumerate(sel):
            assert torch.isfinite(o.float()).all()
            ridx, ref = _oracle_rows(cfg, p, x, ids, _sample_rows(p.N, seed=j))
            max_rel, mean_abs = assert_close(o[:, ridx], ref, f"{cfgname} {label} projection {j}")
            print(f"  projection {j} ({p.N}x{K}): max_rel={max_rel:.2e} mean_abs={mean_abs:.2e}", flush=True)
            ref_base = oracle.c.linear(x.cpu().numpy(), p.W[ridx].cpu().numpy(), None, None)
            assert np.abs(ref - ref_base).max() > 10 * np.abs(o[:, ridx].float().cpu().numpy() - ref).max()


def test_grouped_split_k_launch_is_reproducible(dz):
    """Split-k partial sums meet in a fixed order, whoever arrives last: fifty repeats of one grouped
    full-size launch give the same bits every time."""
    cfg = S.config("7b_decode")
    projs = S.projections_of(cfg)
    gidx = S.launch_groups(cfg)[0]
    ids = cfg.make_ids(S.stream(0, cfg.name, "ids")).cuda()
    with dz.Context(0) as c:
        Ws, packs, Ns = [], [], []
        x = None
        for i in gidx:
            name, N, K = projs[i]
            p = S.make_projection(cfg, 0, 0, name, N, K, device="cuda")
            nbytes = dz.dz_packed_bytes(N, K, cfg.bits, cfg.group)
            packed = []
            for t in p.tabs:
                buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
                dz.dz_pack_delta(c.h, t.codes, t.idx, t.scale, t.zero, N, K, cfg.bits, cfg.group, buf)
                packed.append(buf)
            Ws.append(p.W); packs.append(packed); Ns.append(N)
            x = p.x if x is None else x
            del p
        first = None
        for rep in range(50):
            outs = [torch.full((cfg.T, N), 7.0, dtype=torch.float16, device="cuda") for N in Ns]
            dz.dz_linear_group(c.h, x, Ws, packs, ids, outs, cfg.T, Ns, projs[gidx[0]][2], cfg.bits, cfg.group)
            torch.cuda.synchronize()
            if first is None:
                first = outs
                continue
            for a, b in zip(first, outs):
                assert torch.equal(a, b), f"repeat {rep} differs"
        assert dz.dz_check(c.h) == dz.DZ_OK


@pytest.mark.parametrize("cfgname,N,K", [("7b_decode", 11008, 4096), ("70b_stack", 8192, 8192), ("13b_prefill", 5120, 5120)],
                         ids=lambda v: str(v))
def test_fullsize_quantisation_only(dz, cfgname, N, K):
    """dz_qlinear at workload sizes (quantisation-only deltas: Section 4.1 step 3 without step 2), sampled
    output features against the oracle; the deltas are quantised on the GPU by the seeded generator."""
    print(f"case {cfgname} quant-only {N}x{K}", flush=True)
    cfg = S.config(cfgname)
    D = min(cfg.D, 4)
    with dz.Context(0) as c:
        W = S.make_base(N, K, S.stream(0, cfgname, "qfull", "W", device="cuda"))
        x = S.make_x(cfg.T, K, S.stream(0, cfgname, "qfull", "x", device="cuda"))
        tabs = [S.make_dense_tables(N, K, cfg.bits, cfg.group, S.stream(0, cfgname, "qfull", m, device="cuda")) for m in range(D)]
        ids = cfg.make_ids(S.stream(0, cfg.name, "ids")) % D
        ids = ids.to(torch.int32)
        packed = []
        for t in tabs:
            p = torch.empty(dz.dz_qpacked_bytes(N, K, cfg.bits, cfg.group), dtype=torch.uint8, device="cuda")
            dz.dz_qpack_delta(c.h, t.codes, t.scale, t.zero, N, K, cfg.bits, cfg.group, p)
            packed.append(p)
        out = torch.full((cfg.T, N), 7.0, dtype=torch.float16, device="cuda")
        dz.dz_qlinear(c.h, x, W, packed, ids.cuda(), out, cfg.T, N, K, cfg.bits, cfg.group)
        assert dz.dz_check(c.h) == dz.DZ_OK
        rows = _sample_rows(N)
        ridx = torch.as_tensor(rows, device="cuda")
        dense = [oracle.quant.dequant_dense(t.codes[ridx].cpu().numpy(), t.scale[ridx].cpu().numpy(),
                                            t.zero[ridx].cpu().numpy(), cfg.bits, cfg.group) for t in tabs]
        ref = oracle.c.linear(x.cpu().numpy(), W[ridx].cpu().numpy(), dense, ids.numpy())
        max_rel, mean_abs = assert_close(out[:, ridx], ref, f"{cfgname} quant-only {N}x{K}")
        print(f"  max_rel={max_rel:.2e} mean_abs={mean_abs:.2e}", flush=True)


def test_fullsize_adapters_and_compressor(dz):
    """dz_lora_sbmm with 128 adapters of rank 64 on a 7B projection, and dz_compress_delta on a whole
    4096 x 4096 delta (bit-exact against the oracle on sampled rows, which are independent of each other)."""
    T, N, K, D, r = 64, 4096, 4096, 128, 64
    with dz.Context(0) as c:
        x = S.make_x(T, K, S.stream(0, "lora full", "x", device="cuda"))
        A = [S.make_base(r, K, S.stream(0, "lora full", "A", m, device="cuda"), 0.05) for m in range(D)]
        B = [S.make_base(N, r, S.stream(0, "lora full", "B", m, device="cuda"), 0.05) for m in range(D)]
        ids = S.ids_uniform(T, D, S.stream(0, "lora full", "ids")).to(torch.int32)
        out = torch.empty(T, N, dtype=torch.float16, device="cuda")
        dz.dz_lora_sbmm(c.h, x, A, B, r, ids.cuda(), out, T, N, K, 0)
        torch.cuda.synchronize()
        used = sorted(set(int(v) for v in ids.tolist()))
        remap = {m: i for i, m in enumerate(used)}
        ref = oracle.lora.lora_sbmm(x.cpu().numpy(), [A[m].cpu().numpy() for m in used], [B[m].cpu().numpy() for m in used],
                                    np.asarray([remap[int(v)] for v in ids.tolist()], np.int32))
        assert_close(out, ref, "128 adapters of rank 64")
        d = S._normal_f16((N, K), 0.002, S.stream(0, "compress full", device="cuda"))
        codes = torch.empty(N, K // 2, dtype=torch.uint8, device="cuda"); idx = torch.empty_like(codes)
        scale = torch.empty(N, K // 128, dtype=torch.float16, device="cuda"); zero = torch.empty_like(scale)
        dz.dz_compress_delta(c.h, d, N, K, 4, 128, codes, idx, scale, zero)
        torch.cuda.synchronize()
        rows = torch.as_tensor(_sample_rows(N), device="cuda")
        wc, wi, ws, wz = oracle.compress_.compress(d[rows].cpu().numpy(), 4, 128)
        assert np.array_equal(codes[rows].cpu().numpy(), wc) and np.array_equal(idx[rows].cpu().numpy(), wi)
        assert np.array_equal(scale[rows].cpu().numpy().view(np.uint16), ws.view(np.uint16))
        assert np.array_equal(zero[rows].cpu().numpy().view(np.uint16), wz.view(np.uint16))
        assert dz.dz_check(c.h) == dz.DZ_OK
