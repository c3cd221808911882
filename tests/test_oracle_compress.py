"""Pins for the data-free compressor oracle (2:4 magnitude pruning + group-wise asymmetric round to
nearest; paper Section 4.1 steps 2-3, with the mask and grid rule this build states).  Nothing here
calls the GPU library."""
import numpy as np
import torch

import dz_synth as S
import oracle

C = oracle.compress_


def test_hand_worked_groups():
    """Worked by hand from the rule.  Row 0: magnitudes 0.5, 1.0, 0.25, 1.0 -> keep positions 1 and 3;
    row 1: all equal -> ties go to the lower positions 0 and 1; row 2: keep positions 0 and 2."""
    d = np.array([[0.5, -1.0, 0.25, 1.0], [1.0, 1.0, 1.0, 1.0], [-3.0, 0.5, 2.0, 1.0]], np.float16)
    kept, idx = C.prune_2of4(d)
    assert idx.tolist() == [[1, 3], [0, 1], [0, 2]]
    assert kept.tolist() == [[-1.0, 1.0], [1.0, 1.0], [-3.0, 2.0]]
    # 2-bit grid over one group of 4 dense columns (2 kept values), by hand:
    #  row 0: lo -1, hi 1 -> s = f16(2/3) = 0.66650390625, z = rint(1/s) = rint(1.5004) = 2,
    #         q = clamp(rint(-1.5004) + 2, 0, 3) = 0 and clamp(rint(1.5004) + 2) = clamp(4) = 3
    #  row 1: lo 0, hi 1 -> s = f16(1/3) = 0.333251953125, z = 0, q = rint(3.0007) = 3 twice
    #  row 2: lo -3, hi 2 -> s = f16(5/3) = 1.6669921875, z = rint(1.79966) = 2, q = rint(-1.79966)+2 = 0, rint(1.19977)+2 = 3
    codes, scale, zero = C.quantize(kept, 2, 4)
    assert scale[:, 0].tolist() == [0.66650390625, 0.333251953125, 1.6669921875]
    assert zero[:, 0].tolist() == [2.0, 0.0, 2.0]
    assert codes.tolist() == [[0, 3], [3, 3], [0, 3]]
    # a one-sided positive group has zero-point +0: the zero-point is one of the 2^b codes, never a negative zero
    assert zero.view(np.uint16)[1, 0] == 0
    # an all-zero group: scale 1, zero 0, codes 0
    codes, scale, zero = C.quantize(np.zeros((1, 2), np.float16), 4, 4)
    assert (scale[0, 0], zero[0, 0], codes.tolist()) == (1.0, 0.0, [[0, 0]])


def test_invariants_on_random_deltas():
    for bits, G in ((4, 128), (2, 64), (4, 64), (2, 128)):
        d = S._normal_f16((24, 512), 0.002, S.stream(7, "delta", bits, G)).numpy()
        codes, idx, scale, zero = C.compress(d, bits, G)
        assert oracle.c.validate(codes, idx, scale, zero, bits, G) == 0
        dense = oracle.c.dequant(codes, idx, scale, zero, bits, G)
        # exactly two stored positions per group of four, at most two non-zeros
        nz = (dense.reshape(24, -1, 4) != 0).sum(-1)
        assert nz.max() <= 2
        # the dropped entries are the two smallest magnitudes of their group
        mag = np.abs(d.astype(np.float32)).reshape(24, -1, 4)
        keep = np.zeros_like(mag, bool)
        np.put_along_axis(keep, idx.reshape(24, -1, 2).astype(np.int64), True, axis=-1)
        assert (np.where(keep, mag, np.inf).min(-1) >= np.where(keep, -np.inf, mag).max(-1)).all()
        # round to nearest: a kept value whose code is not at the end of the code range is reproduced to
        # within half a grid step
        qg = (np.arange(256) // 2 * 4) // G
        s = scale.astype(np.float32)[:, qg]
        kept = np.take_along_axis(d.reshape(24, -1, 4), idx.reshape(24, -1, 2).astype(np.int64), -1).reshape(24, -1)
        deq = np.take_along_axis(dense.reshape(24, -1, 4), idx.reshape(24, -1, 2).astype(np.int64), -1).reshape(24, -1)
        inner = (codes > 0) & (codes < (1 << bits) - 1)
        err = np.abs(kept.astype(np.float32) - deq)
        assert (err[inner] <= 0.5 * s[inner] * (1 + 1e-3)).all()


def test_agrees_with_the_input_generator_bit_for_bit():
    """The seeded input generator has its own vectorised writing of the same rule (torch); two
    independent writings must give identical tables."""
    for bits, G in ((4, 128), (2, 64)):
        d = S._normal_f16((40, 1024), 0.002, S.stream(8, "delta", bits))
        kept_t, idx_t = S.prune_2of4(d)
        q_t, s_t, z_t = S.quantize_groups(kept_t, bits, G)
        codes, idx, scale, zero = C.compress(d.numpy(), bits, G)
        assert np.array_equal(idx, idx_t.numpy())
        assert np.array_equal(codes, q_t.numpy())
        assert np.array_equal(scale.view(np.uint16), s_t.numpy().view(np.uint16))
        assert np.array_equal(zero.view(np.uint16), z_t.numpy().view(np.uint16))
    # ties and zeros
    d = torch.tensor([[1.0, -1.0, 1.0, -1.0, 0.0, 0.0, 0.0, 0.0]], dtype=torch.float16)
    kept_t, idx_t = S.prune_2of4(d)
    kept, idx = C.prune_2of4(d.numpy())
    assert idx.tolist() == idx_t.tolist() == [[0, 1, 0, 1]]
