"""The synthetic stand-in for the offline compressor (paper Section 4.1 steps 2-3) makes legal
tables: magnitude 2:4 prune, then group-wise asymmetric round-to-nearest."""
import numpy as np
import torch

import dz_synth as S
import oracle


def test_prune_keeps_two_largest_with_low_index_ties():
    d = torch.tensor([[1, -3, 2, 0.5, 2, 2, 2, 2, 0, 0, 0, 1, -1, 1, -1, 1]], dtype=torch.float16)
    kept, idx = S.prune_2of4(d)
    assert idx.tolist() == [[1, 2, 0, 1, 0, 3, 0, 1]]
    assert kept.tolist() == [[-3, 2, 2, 2, 0, 1, -1, 1]]


def test_rtn_bound_and_ranges():
    for bits, G in [(4, 64), (2, 128), (4, 128)]:
        N, K = 64, 512
        gen = S.stream(5, bits, G)
        d = S._normal_f16((N, K), 0.002, gen)
        kept, idx = S.prune_2of4(d)
        q, s, z = S.quantize_groups(kept, bits, G)
        assert q.max() <= (1 << bits) - 1
        assert (z == z.round()).all() and z.min() >= 0 and z.max() <= (1 << bits) - 1
        per = G // 2
        sf = s.float().repeat_interleave(per, 1)
        zf = z.float().repeat_interleave(per, 1)
        rec = (q.float() - zf) * sf
        err = (kept.float() - rec).abs()
        inside = (q > 0) & (q < (1 << bits) - 1)
        assert (err[inside] <= 0.5 * sf[inside] * 1.002 + 1e-9).all()
        # pruned entries are never larger than kept ones of the same group of four
        a = d.abs().float().reshape(N, K // 4, 4)
        km = torch.zeros_like(a, dtype=torch.bool)
        km.scatter_(-1, idx.reshape(N, K // 4, 2).long(), True)
        assert (a.masked_fill(km, 0).amax(-1) <= a.masked_fill(~km, 9).amin(-1)).all()
        t = S.DeltaTables(q, idx, s, z, bits, G)
        assert oracle.c.validate(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G) == 0


def test_streams_are_reproducible_and_independent():
    a = S.make_x(4, 8, S.stream(0, "x", 1))
    b = S.make_x(4, 8, S.stream(0, "x", 1))
    c = S.make_x(4, 8, S.stream(0, "x", 2))
    assert torch.equal(a, b) and not torch.equal(a, c)


def test_configs_match_the_five_workloads():
    c = S.CONFIGS
    assert [(s.N, s.K, s.count) for s in c["7b_decode"].shapes] == [(4096, 4096, 4), (11008, 4096, 2), (4096, 11008, 1)]
    assert [(s.N, s.K, s.count) for s in c["70b_stack"].shapes] == [(8192, 8192, 2), (1024, 8192, 2), (28672, 8192, 2), (8192, 28672, 1)]
    ids = c["13b_prefill"].make_ids(S.stream(0, "ids"))
    assert ids.shape == (2048,) and (ids[1:] >= ids[:-1]).all() and ids.unique().numel() == 16
    z = c["7b_decode_many"].make_ids(S.stream(0, "ids"))
    assert z.shape == (64,) and z.min() >= 0 and z.max() < 32
