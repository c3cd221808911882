"""Pins for the oracle's dense dequantisation (what a compressed delta stands for).

Paper Section 4.1: step 2 keeps two of every four consecutive entries and stores their 2-bit
positions; step 3 stores each kept value as a b-bit code.  Nothing here calls the GPU library.
"""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _tables(N, K, G, codes, idx, scale, zero):
    return (np.asarray(codes, np.uint8).reshape(N, K // 2), np.asarray(idx, np.uint8).reshape(N, K // 2),
            np.asarray(scale, np.float16).reshape(N, K // G), np.asarray(zero, np.float16).reshape(N, K // G))


def _gold_rows(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


@pytest.mark.parametrize("impl", ["c", "np"])
def test_closed_form_values(impl):
    deq = oracle.c.dequant if impl == "c" else oracle.np_.dequant
    for bits, s, z, code, want in _gold_rows("dequant_closed_form.txt"):
        bits, code = int(bits), int(code)
        # one row, one group of 4 columns, kept values at positions 1 and 3; second code = zero-point
        codes, idx, scale, zero = _tables(1, 4, 4, [code, int(float(z))], [1, 3], [float(s)], [float(z)])
        d = deq(codes, idx, scale, zero, bits, 4)
        assert d.dtype == np.float32 and d.shape == (1, 4)
        assert d[0].tolist() == [0.0, float(want), 0.0, 0.0], (bits, s, z, code)


@pytest.mark.parametrize("impl", ["c", "np"])
def test_six_position_pairs(impl):
    deq = oracle.c.dequant if impl == "c" else oracle.np_.dequant
    a, b = 3.0, -5.0     # scale 1, zero 8 -> codes 11 and 3
    for i0, i1, *pat in _gold_rows("two_of_four_patterns.txt"):
        want = [{"a": a, "b": b, "0": 0.0}[p] for p in pat]
        codes, idx, scale, zero = _tables(1, 4, 4, [11, 3], [int(i0), int(i1)], [1.0], [8.0])
        assert deq(codes, idx, scale, zero, 4, 4)[0].tolist() == want


@pytest.mark.parametrize("impl", ["c", "np"])
def test_group_boundaries_rows_and_columns(impl):
    """Scale/zero change every G dense columns and every row; a transposed or off-by-one group
    index would move a value onto the wrong grid."""
    deq = oracle.c.dequant if impl == "c" else oracle.np_.dequant
    N, K, G = 3, 16, 8
    codes = np.full((N, K // 2), 1, np.uint8)
    idx = np.tile(np.array([0, 1], np.uint8), (N, K // 4))
    scale = np.array([[1, 2], [4, 8], [16, 32]], np.float16)
    zero = np.zeros((N, 2), np.float16)
    d = deq(codes, idx, scale, zero, 4, G)
    for n in range(N):
        for k in range(K):
            want = float(scale[n, k // G]) if k % 4 < 2 else 0.0
            assert d[n, k] == want, (n, k)


def test_c_and_numpy_agree_bit_for_bit_and_invariants():
    import torch
    import dz_synth as S
    for bits, G, N, K in [(4, 64, 48, 256), (2, 128, 32, 512), (4, 128, 16, 1024)]:
        t = S.make_delta_tables(N, K, bits, G, S.stream(0, "deq", bits, G))
        args = (t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G)
        assert oracle.c.validate(*args) == 0
        dc = oracle.c.dequant(*args)
        dn = oracle.np_.dequant(*args)
        assert dc.tobytes() == dn.tobytes()
        # the product is exact in fp32: fp64 evaluation rounds to the same fp32
        d64 = oracle.np_.dequant(*args, dtype=np.float64)
        assert (d64.astype(np.float32) == dc).all() and (d64 == dc.astype(np.float64)).all()
        # 2:4 invariant on the dense matrix and on the metadata
        nz = (dc.reshape(N, K // 4, 4) != 0).sum(-1)
        assert nz.max() <= 2
        i = t.idx.numpy().reshape(N, K // 4, 2)
        assert (i[..., 0] < i[..., 1]).all() and i.max() <= 3
        # every stored position that holds a non-zero code-minus-zero shows up in the dense matrix
        stored = np.zeros((N, K // 4, 4), bool)
        np.put_along_axis(stored, i.astype(np.int64), True, axis=-1)
        assert stored.sum(-1).min() == 2 and stored.sum(-1).max() == 2
        assert not (dc.reshape(N, K // 4, 4)[~stored] != 0).any()


def test_validate_rejects_bad_tables():
    codes, idx, scale, zero = _tables(1, 8, 4, [1, 2, 3, 4], [0, 1, 2, 3], [1.0, 1.0], [0.0, 0.0])
    assert oracle.c.validate(codes, idx, scale, zero, 4, 4) == 0
    bad = codes.copy(); bad[0, 0] = 16
    assert oracle.c.validate(bad, idx, scale, zero, 4, 4) == 4
    assert oracle.c.validate(codes, idx, scale, zero, 2, 4) == 4      # code 4 does not fit 2 bits
    bi = idx.copy(); bi[0, 0], bi[0, 1] = 1, 1
    assert oracle.c.validate(codes, bi, scale, zero, 4, 4) == 5       # equal positions
    bi = idx.copy(); bi[0, 0], bi[0, 1] = 2, 1
    assert oracle.c.validate(codes, bi, scale, zero, 4, 4) == 5       # descending
    bz = zero.copy(); bz[0, 0] = 0.5
    assert oracle.c.validate(codes, idx, scale, bz, 4, 4) == 6
    bs = scale.copy(); bs[0, 1] = np.inf
    assert oracle.c.validate(codes, idx, bs, zero, 4, 4) == 7
    assert oracle.c.validate(codes, idx, scale, zero, 3, 4) == 2
