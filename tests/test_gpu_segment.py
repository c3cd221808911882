"""GPU: dz_segment equals the oracle's stable counting sort bit for bit (paper Section 5.2, request
reordering)."""
import numpy as np
import pytest
import torch

import dz_synth as S
import oracle

pytestmark = pytest.mark.gpu


def _run(dz, c, ids, D):
    ids = np.asarray(ids, np.int32)
    T = len(ids)
    d = torch.as_tensor(ids, device="cuda") if T else torch.zeros(1, dtype=torch.int32, device="cuda")
    counts = torch.full((max(D, 1),), -7, dtype=torch.int32, device="cuda")
    offsets = torch.full((D + 1,), -7, dtype=torch.int32, device="cuda")
    perm = torch.full((max(T, 1),), -7, dtype=torch.int32, device="cuda")
    dz.dz_segment(c.h, d, T, D, counts, offsets, perm)
    torch.cuda.synchronize()
    rc, ro, rp = oracle.c.segment(ids, D)
    assert counts.cpu().numpy()[:D].tolist() == rc.tolist()
    assert offsets.cpu().numpy().tolist() == ro.tolist()
    assert perm.cpu().numpy()[:T].tolist() == rp.tolist()


def test_segment_matches_oracle(dz):
    with dz.Context(0) as c:
        _run(dz, c, [], 3)
        _run(dz, c, [0], 1)
        _run(dz, c, [2, 2, 2], 3)
        _run(dz, c, [1, -1, 0, 1, 0, -1, 2], 3)
        _run(dz, c, S.ids_uniform(8, 4, S.stream(0, "u")).numpy(), 4)
        _run(dz, c, S.ids_uniform(32, 8, S.stream(0, "u")).numpy(), 8)
        _run(dz, c, S.ids_zipf(64, 32, 1.5, S.stream(0, "z")).numpy(), 32)
        _run(dz, c, S.ids_segments(2048, 16, S.stream(0, "s")).numpy(), 16)
        _run(dz, c, S.ids_uniform(5000, 100, S.stream(1, "u")).numpy(), 100)
        _run(dz, c, S.ids_uniform(1000, 300, S.stream(2, "u")).numpy(), 300)
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_out_of_range_index_is_reported_once(dz):
    with dz.Context(0) as c:
        _run(dz, c, [1, 5, 0, -3, 2], 3)          # 5 and -3 are outside [-1, 3)
        assert dz.dz_check(c.h) == dz.DZ_ERR_INDEX
        assert dz.dz_check(c.h) == dz.DZ_OK       # sticky until read, then cleared
        _run(dz, c, [1, -1, 0], 3)
        assert dz.dz_check(c.h) == dz.DZ_OK
