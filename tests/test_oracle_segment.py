"""Pins for request reordering (paper Section 5.2: requests of the same delta are grouped together
before the delta product)."""
import numpy as np

import dz_synth as S
import oracle


def _check(ids, D):
    ids = np.asarray(ids, np.int32)
    T = len(ids)
    counts, offsets, perm = oracle.c.segment(ids, D)
    assert sorted(perm.tolist()) == list(range(T))
    valid = (ids >= 0) & (ids < D)
    assert counts.sum() == valid.sum() and offsets[0] == 0 and offsets[D] == valid.sum()
    assert (np.diff(offsets) == counts).all()
    key = np.where(valid, ids, D)
    assert (np.diff(key[perm]) >= 0).all()
    for m in range(D):
        seg = perm[offsets[m]:offsets[m + 1]]
        assert (ids[seg] == m).all() and (np.diff(seg) > 0).all()       # stable
    tail = perm[offsets[D]:]
    assert (np.diff(tail) > 0).all() and not valid[tail].any()
    c2, o2, p2 = oracle.np_.segment(ids, D)
    assert (c2 == counts).all() and (o2 == offsets).all() and (p2 == perm).all()
    assert (perm == np.argsort(key, kind="stable")).all()


def test_segment_cases():
    _check([], 3)
    _check([0], 1)
    _check([2, 2, 2], 3)
    _check([1, -1, 0, 5, 1, 0, -7, 2], 3)
    _check(S.ids_uniform(32, 8, S.stream(0, "u")).numpy(), 8)
    _check(S.ids_zipf(64, 32, 1.5, S.stream(0, "z")).numpy(), 32)
    _check(S.ids_segments(2048, 16, S.stream(0, "s")).numpy(), 16)
    _check(S.ids_uniform(777, 5, S.stream(1, "u")).numpy(), 3)         # ids 3,4 out of range
