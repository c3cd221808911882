"""GPU: dz_pack_delta / dz_unpack_delta are bit-exact against the canonical tables and the oracle's
dense dequantisation (paper Section 4.1 steps 2-3)."""
import numpy as np
import pytest
import torch

import dz_synth as S
import oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,K,bits,G", [(256, 256, 4, 64), (48, 768, 4, 128), (32, 512, 2, 128),
                                         (80, 1024, 2, 64), (4096, 4096, 4, 128), (1024, 2816, 2, 128)])
def test_pack_unpack_roundtrip_bit_exact(dz, N, K, bits, G):
    print(f"case N={N} K={K} bits={bits} G={G}", flush=True)
    with dz.Context(0) as c:
        t = S.make_delta_tables(N, K, bits, G, S.stream(0, "pack", N, K, bits, G))
        d = t.to("cuda")
        nbytes = dz.dz_packed_bytes(N, K, bits, G)
        assert nbytes == N * K * (2 * bits + 4) // 32 + 4 * N * K // G
        guard = 64
        buf = torch.full((nbytes + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
        packed = buf[guard:guard + nbytes]
        assert packed.data_ptr() % 16 == 0
        dz.dz_pack_delta(c.h, d.codes, d.idx, d.scale, d.zero, N, K, bits, G, packed)
        codes = torch.full_like(d.codes, 0xFF); idx = torch.full_like(d.idx, 0xFF)
        scale = torch.zeros_like(d.scale); zero = torch.zeros_like(d.zero)
        dense = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
        dz.dz_unpack_delta(c.h, packed, N, K, bits, G, codes, idx, scale, zero, dense)
        torch.cuda.synchronize()
        assert (buf[:guard] == 0xA5).all() and (buf[guard + nbytes:] == 0xA5).all()      # stays in bounds
        assert torch.equal(codes.cpu(), t.codes) and torch.equal(idx.cpu(), t.idx)
        assert scale.cpu().view(torch.int16).equal(t.scale.view(torch.int16))
        assert zero.cpu().view(torch.int16).equal(t.zero.view(torch.int16))
        ref = oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G)
        assert dense.cpu().numpy().tobytes() == ref.tobytes()
        # every byte of the blob is written (no holes): packing twice over different fill gives same bytes
        buf2 = torch.zeros_like(buf)
        p2 = buf2[guard:guard + nbytes]
        dz.dz_pack_delta(c.h, d.codes, d.idx, d.scale, d.zero, N, K, bits, G, p2)
        torch.cuda.synchronize()
        assert torch.equal(p2, packed)
        assert dz.dz_check(c.h) == dz.DZ_OK


def test_argument_errors(dz):
    with dz.Context(0) as c:
        z = torch.zeros(4096, dtype=torch.uint8, device="cuda")
        h = torch.zeros(64, dtype=torch.float16, device="cuda")
        assert dz.dz_packed_bytes(256, 256, 3, 64) == 0 and dz.dz_packed_bytes(250, 256, 4, 64) == 0
        assert dz.dz_packed_bytes(256, 128, 4, 64) == 0 and dz.dz_packed_bytes(256, 256, 4, 32) == 0
        assert dz.dz_pack_delta(c.h, z, z, h, h, 16, 256, 3, 64, z, check=False) == dz.DZ_ERR_BITS
        assert dz.dz_pack_delta(c.h, z, z, h, h, 16, 200, 4, 64, z, check=False) == dz.DZ_ERR_SHAPE
        assert dz.dz_pack_delta(c.h, z, z, h, h, 16, 256, 4, 64, z[1:], check=False) == dz.DZ_ERR_ALIGN
        assert dz.dz_pack_delta(c.h, None, z, h, h, 16, 256, 4, 64, z, check=False) == dz.DZ_ERR_ARG
        assert dz.dz_unpack_delta(c.h, None, 16, 256, 4, 64, check=False) == dz.DZ_ERR_ARG
        assert "bits" in dz.dz_strerror(dz.DZ_ERR_BITS)
