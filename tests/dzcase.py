"""Shared scaffolding for the GPU parity tests: build one seeded case on the host, run the oracle
on it, upload it, pack the deltas through the C ABI."""
from __future__ import annotations

import numpy as np
import torch

import dz_synth as S
import oracle

MAX_REL = 1e-2      # max |gpu - ref| / max(|ref|, rms(ref))   (spec tolerance for fp16 outputs)
MEAN_ABS = 1e-3     # mean |gpu - ref|


def errors(got_f16: torch.Tensor, ref_f32: np.ndarray):
    got = got_f16.detach().float().cpu().numpy().astype(np.float64)
    ref = ref_f32.astype(np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), max(rms, 1e-30))
    diff = np.abs(got - ref)
    return (float((diff / den).max()) if ref.size else 0.0, float(diff.mean()) if ref.size else 0.0, rms)


def assert_close(got_f16, ref_f32, what=""):
    assert tuple(got_f16.shape) == tuple(ref_f32.shape), (what, got_f16.shape, ref_f32.shape)
    assert torch.isfinite(got_f16.float()).all(), what
    max_rel, mean_abs, rms = errors(got_f16, ref_f32)
    assert max_rel <= MAX_REL, f"{what}: max rel err {max_rel:.3e} > {MAX_REL} (rms {rms:.3e})"
    assert mean_abs <= MEAN_ABS, f"{what}: mean abs err {mean_abs:.3e} > {MEAN_ABS}"
    return max_rel, mean_abs


class Case:
    """One linear layer, D deltas, T requests; host copies, oracle results, device copies."""

    def __init__(self, dz, ctx, seed, T, N, K, D, bits, G, ids, delta_std=0.002, base_std=0.02, device="cuda"):
        self.T, self.N, self.K, self.D, self.bits, self.G = T, N, K, D, bits, G
        self.W = S.make_base(N, K, S.stream(seed, "W"), base_std)
        self.x = S.make_x(T, K, S.stream(seed, "x"))
        self.tabs = [S.make_delta_tables(N, K, bits, G, S.stream(seed, "delta", m), std=delta_std) for m in range(D)]
        if isinstance(ids, str):
            g = S.stream(seed, "ids")
            ids = {"uniform": lambda: S.ids_uniform(T, D, g), "zipf": lambda: S.ids_zipf(T, D, 1.5, g),
                   "segments": lambda: S.ids_segments(T, D, g)}[ids]()
        self.ids = torch.as_tensor(np.asarray(ids), dtype=torch.int32)
        # oracle
        self.dense = [oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), bits, G)
                      for t in self.tabs]
        xn, Wn, idn = self.x.numpy(), self.W.numpy(), self.ids.numpy()
        self.y_base = oracle.c.linear(xn, Wn, None, None)
        self.y_delta = oracle.c.linear(xn, None, self.dense, idn) if D else np.zeros((T, N), np.float32)
        self.y = oracle.c.linear(xn, Wn, self.dense, idn)
        # device
        self.dW, self.dx, self.dids = self.W.to(device), self.x.to(device), self.ids.to(device)
        self.packed = []
        nbytes = dz.dz_packed_bytes(N, K, bits, G)
        for t in self.tabs:
            dt = t.to(device)
            p = torch.empty(nbytes, dtype=torch.uint8, device=device)
            dz.dz_pack_delta(ctx, dt.codes, dt.idx, dt.scale, dt.zero, N, K, bits, G, p)
            self.packed.append(p)
        torch.cuda.synchronize()

    def out(self, fill=None):
        o = torch.empty(self.T, self.N, dtype=torch.float16, device="cuda")
        if fill is not None:
            o.fill_(fill)
        return o
