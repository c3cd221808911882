"""Pins for the quantisation-only and merged-weight oracles (paper Section 4.1 step 3; Section 5.1
Eq. (2)).  Nothing here calls the GPU library."""
import numpy as np
import torch

import dz_synth as S
import oracle

Q = oracle.quant


def test_closed_form_tables():
    """b = 4, s = 0.5, z = 8: codes 0..15 stand for -4.0 .. 3.5 in steps of 0.5; b = 2, s = 0.25, z = 1:
    {-0.25, 0, 0.25, 0.5}.  Two rows and two groups with different (s, z) show that row and group are
    indexed the right way round."""
    codes = np.tile(np.arange(16, dtype=np.uint8), (2, 2))            # [2][32], G = 16
    scale = np.array([[0.5, 0.25], [2.0, 1.0]], np.float16)
    zero = np.array([[8, 0], [15, 1]], np.float16)
    d = Q.dequant_dense(codes, scale, zero, 4, 16)
    c = np.arange(16, dtype=np.float32)
    assert np.array_equal(d[0, :16], (c - 8) * 0.5) and np.array_equal(d[0, 16:], c * 0.25)
    assert np.array_equal(d[1, :16], (c - 15) * 2.0) and np.array_equal(d[1, 16:], c - 1.0)
    assert d[0, 0] == -4.0 and d[0, 15] == 3.5
    d2 = Q.dequant_dense(np.arange(4, dtype=np.uint8)[None, :], np.array([[0.25]], np.float16),
                         np.array([[1]], np.float16), 2, 4)
    assert d2.tolist() == [[-0.25, 0.0, 0.25, 0.5]]


def test_a_two_of_four_table_written_densely_gives_the_same_matrix():
    """A 2:4 delta is a dense delta whose pruned columns carry the zero-point as their code: the dense
    dequantiser must then reproduce the (separately pinned) 2:4 dequantiser bit for bit."""
    N, K, bits, G = 12, 256, 4, 64
    t = S.make_delta_tables(N, K, bits, G, S.stream(31, "delta"))
    sparse = oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G)
    codes = np.repeat(t.zero.numpy().astype(np.uint8), G, axis=1)           # every column at the zero-point
    cols = (np.arange(K // 2) // 2 * 4)[None, :] + t.idx.numpy().astype(np.int64)
    np.put_along_axis(codes, cols, t.codes.numpy(), axis=1)
    dense = Q.dequant_dense(codes, t.scale.numpy(), t.zero.numpy(), bits, G)
    assert dense.tobytes() == sparse.tobytes()


def test_quantizer_hand_worked_and_round_to_nearest():
    """One group of four by hand: v = (-1, 0.5, 0.25, 1), b = 2: lo -1, hi 1, s = f16(2/3) = 0.66650390625,
    z = rint(1.5004) = 2; codes rint(v / s) + 2 = (-2, 1, 0, 2) + 2 -> (0, 3, 2, 4 -> 3)."""
    v = np.array([[-1.0, 0.5, 0.25, 1.0]], np.float16)
    codes, scale, zero = Q.quantize_dense(v, 2, 4)
    assert scale[0, 0] == 0.66650390625 and zero[0, 0] == 2.0 and codes.tolist() == [[0, 3, 2, 3]]
    # random deltas: every value whose code is not at an end of the range is reproduced within half a step
    for bits, G in ((4, 128), (2, 64)):
        d = S._normal_f16((16, 512), 0.002, S.stream(32, "d", bits)).numpy()
        codes, scale, zero = Q.quantize_dense(d, bits, G)
        deq = Q.dequant_dense(codes, scale, zero, bits, G)
        s = np.repeat(scale.astype(np.float32), G, axis=1)
        inner = (codes > 0) & (codes < (1 << bits) - 1)
        assert (np.abs(d.astype(np.float32) - deq)[inner] <= 0.5 * s[inner] * (1 + 1e-3)).all()
        assert zero.view(np.uint16).max() < 0x8000 and (zero == np.rint(zero)).all()
        # the generator's own (torch) writing of the rule gives the same tables
        t = S.make_dense_tables(16, 512, bits, G, S.stream(32, "d", bits))
        assert np.array_equal(t.codes.numpy(), codes)
        assert np.array_equal(t.scale.numpy().view(np.uint16), scale.view(np.uint16))
        assert np.array_equal(t.zero.numpy().view(np.uint16), zero.view(np.uint16))
        assert S.qpacked_bytes(16, 512, bits, G) == 16 * 512 * bits // 8 + 4 * 16 * 512 // G


def test_merged_weight_is_the_correctly_rounded_sum():
    W = np.array([[1.0, 0.5, -2.0, 1024.0]], np.float16)
    d = np.array([[2.0 ** -11, 2.0 ** -12, 0.0, 0.5]], np.float32)
    m = Q.merged_weight(W, d)
    # 1 + 2^-11 is a tie between 1 and 1 + 2^-10 -> even (1.0); 0.5 + 2^-12 is a tie -> 0.5; 1024.5 -> tie -> 1024
    assert m.tolist() == [[1.0, 0.5, -2.0, 1024.0]]
    m = Q.merged_weight(W, np.array([[2.0 ** -10, 2.0 ** -11 + 2.0 ** -20, 0.25, 1.0]], np.float32))
    assert m.tolist() == [[1.0 + 2.0 ** -10, 0.5 + 2.0 ** -11, -1.75, 1025.0]]
    # and serving from it equals serving base + delta up to that rounding: a variant's product through the
    # merged weight stays within the fp16 step of W times |x|_1 of the exact one
    t = S.make_delta_tables(8, 256, 4, 64, S.stream(33, "delta"))
    dense = oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), 4, 64)
    Wb = S.make_base(8, 256, S.stream(33, "W")).numpy()
    x = S.make_x(3, 256, S.stream(33, "x")).numpy()
    ids = np.zeros(3, np.int32)
    exact = oracle.c.linear(x, Wb, [dense], ids)
    via = oracle.c.linear(x, Q.merged_weight(Wb, dense), None, None)
    bound = np.abs(x.astype(np.float64)).sum(1)[:, None] * (np.abs(Wb).max() * 2.0 ** -11)
    assert (np.abs(via.astype(np.float64) - exact) <= bound + 1e-6).all()
