"""Seeded synthetic inputs for the delta-serving hot path.

This module only *makes inputs*: base weights, activations, request->delta index vectors and
"canonical" compressed-delta tables.  It is the one module that both the CPU oracle's tests and the
GPU library's tests import; it contains none of the serving arithmetic (no dequantization, no matmul,
no segmentation).  Everything is written with torch ops so the same code runs on the CPU (small
cases) and on the GPU (full-size layers that would take minutes to draw on the host).

The canonical tables stand in for the output of the paper's offline compressor (Section 4.1, steps 2
and 3: 2:4 structured pruning, then low-bit quantization and packing).  The real compressor needs
calibration data and trained weights; here step 2 is a magnitude 2:4 prune and step 3 is group-wise
asymmetric round-to-nearest, which yields tables of the same shape, bit-width and sparsity pattern.

Canonical tables of one delta for one linear layer with weight shape [N][K] (out x in features):
  codes u8 [N][K/2]   b-bit code of each kept value, two per group of four consecutive k
  idx   u8 [N][K/2]   position (0..3) of each kept value inside its group of four, ascending pairs
  scale f16[N][K/G]   step of the quantisation grid of the G dense columns a group spans
  zero  f16[N][K/G]   integer zero-point of that grid (stored as an exactly-representable fp16)
The value the tables stand for is (code - zero) * scale at column 4*g + idx, and 0 elsewhere.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import torch

__all__ = [
    "DeltaTables", "LayerSpec", "CONFIGS", "stream", "make_base", "make_x", "make_delta_tables",
    "prune_2of4", "quantize_groups", "ids_uniform", "ids_zipf", "ids_segments", "config",
]


def stream(seed: int, *key, device: str = "cpu") -> torch.Generator:
    """Independent generator for the sub-stream named by `key` (config, layer, projection, ...)."""
    h = hashlib.sha256(repr((int(seed),) + tuple(key)).encode()).digest()
    g = torch.Generator(device=device)
    g.manual_seed(int.from_bytes(h[:8], "little") & ((1 << 63) - 1))
    return g


def _normal_f16(shape, std: float, gen: torch.Generator) -> torch.Tensor:
    """Draw N(0, std) in fp32 from the seeded stream, round once to fp16 (nearest-even)."""
    t = torch.empty(shape, dtype=torch.float32, device=gen.device)
    t.normal_(0.0, std, generator=gen)
    return t.to(torch.float16)


def make_base(N: int, K: int, gen: torch.Generator, std: float = 0.02) -> torch.Tensor:
    """Base weight W[N][K], fp16."""
    return _normal_f16((N, K), std, gen)


def make_x(T: int, K: int, gen: torch.Generator, std: float = 1.0) -> torch.Tensor:
    """Activations x[T][K], fp16."""
    return _normal_f16((T, K), std, gen)


@dataclass
class DeltaTables:
    codes: torch.Tensor   # u8 [N][K/2]
    idx: torch.Tensor     # u8 [N][K/2]
    scale: torch.Tensor   # f16 [N][K/G]
    zero: torch.Tensor    # f16 [N][K/G]
    bits: int
    group: int

    @property
    def N(self) -> int:
        return self.codes.shape[0]

    @property
    def K(self) -> int:
        return self.codes.shape[1] * 2

    def to(self, device) -> "DeltaTables":
        return DeltaTables(self.codes.to(device), self.idx.to(device), self.scale.to(device),
                           self.zero.to(device), self.bits, self.group)

    def rows(self, rows) -> "DeltaTables":
        """Tables of a subset of output rows (rows are independent of each other)."""
        return DeltaTables(self.codes[rows].contiguous(), self.idx[rows].contiguous(),
                           self.scale[rows].contiguous(), self.zero[rows].contiguous(),
                           self.bits, self.group)


def prune_2of4(delta: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    """Magnitude 2:4 prune along k.  Returns (kept values [N][K/2] in the input dtype, idx u8
    [N][K/2]).  In every group of four consecutive k the two largest |v| are kept; ties go to the
    lower position; kept entries are emitted in ascending position."""
    N, K = delta.shape
    assert K % 4 == 0
    v = delta.reshape(N, K // 4, 4)
    a = v.abs().to(torch.float32)
    pos = torch.arange(4, device=delta.device)
    # beats[i][j]: element i outranks element j (strict total order: magnitude, then lower position)
    ai, aj = a.unsqueeze(-1), a.unsqueeze(-2)
    pi, pj = pos.view(4, 1), pos.view(1, 4)
    beats = (ai > aj) | ((ai == aj) & (pi < pj))
    wins = beats.sum(-1)                      # 3,2,1,0 in some order
    keep = wins >= 2                          # exactly two per group
    # ascending positions of the two kept entries
    first = keep.to(torch.uint8).argmax(-1)   # lowest kept position
    last = 3 - keep.flip(-1).to(torch.uint8).argmax(-1)
    idx = torch.stack([first, last], -1).to(torch.uint8)        # [N][K/4][2]
    kept = torch.gather(v, -1, idx.to(torch.int64))
    return kept.reshape(N, K // 2), idx.reshape(N, K // 2)


def quantize_groups(kept: torch.Tensor, bits: int, group: int):
    """Asymmetric round-to-nearest over the kept values of each (row, group of `group` dense
    columns = group/2 kept values).  The grid always contains 0.  Returns codes u8, scale f16,
    zero f16 (integer-valued)."""
    N, K2 = kept.shape
    per = group // 2
    assert K2 % per == 0
    qmax = float((1 << bits) - 1)
    v = kept.to(torch.float32).reshape(N, K2 // per, per)
    lo = torch.clamp(v.amin(-1), max=0.0)
    hi = torch.clamp(v.amax(-1), min=0.0)
    s16 = ((hi - lo) / qmax).to(torch.float16)
    dead = s16 == 0
    s16 = torch.where(dead, torch.ones_like(s16), s16)
    s = s16.to(torch.float32)
    z = torch.clamp(torch.round((0.0 - lo) / s), 0.0, qmax)      # torch.round is round-half-even
    z = torch.where(dead, torch.zeros_like(z), z)
    q = torch.clamp(torch.round(v / s.unsqueeze(-1)) + z.unsqueeze(-1), 0.0, qmax)
    return (q.to(torch.uint8).reshape(N, K2), s16, z.to(torch.float16))


def make_delta_tables(N: int, K: int, bits: int, group: int, gen: torch.Generator,
                      std: float = 0.002, row_chunk: int = 2048) -> DeltaTables:
    """Draw a delta ~ N(0, std) -> fp16 -> 2:4 magnitude prune -> group-wise asymmetric RTN."""
    assert K % group == 0 and group % 4 == 0
    codes, idxs, scales, zeros = [], [], [], []
    for r0 in range(0, N, row_chunk):     # chunked only to bound peak memory; stream order is fixed
        r1 = min(N, r0 + row_chunk)
        d = _normal_f16((r1 - r0, K), std, gen)
        kept, idx = prune_2of4(d)
        q, s, z = quantize_groups(kept, bits, group)
        codes.append(q); idxs.append(idx); scales.append(s); zeros.append(z)
    return DeltaTables(torch.cat(codes), torch.cat(idxs), torch.cat(scales), torch.cat(zeros),
                       bits, group)


@dataclass
class DenseTables:
    """A quantisation-only delta (no 2:4 pruning): a code for every column."""
    codes: torch.Tensor   # u8 [N][K]
    scale: torch.Tensor   # f16 [N][K/G]
    zero: torch.Tensor    # f16 [N][K/G]
    bits: int
    group: int

    def to(self, device) -> "DenseTables":
        return DenseTables(self.codes.to(device), self.scale.to(device), self.zero.to(device), self.bits, self.group)


def make_dense_tables(N: int, K: int, bits: int, group: int, gen: torch.Generator, std: float = 0.002,
                      row_chunk: int = 2048) -> DenseTables:
    """Draw a delta ~ N(0, std) -> fp16 -> group-wise asymmetric RTN over all `group` values of a group."""
    assert K % group == 0
    codes, scales, zeros = [], [], []
    for r0 in range(0, N, row_chunk):
        r1 = min(N, r0 + row_chunk)
        d = _normal_f16((r1 - r0, K), std, gen)
        q, s, z = quantize_groups(d, bits, 2 * group)      # quantize_groups counts `group // 2` values per group
        codes.append(q); scales.append(s); zeros.append(z)
    return DenseTables(torch.cat(codes), torch.cat(scales), torch.cat(zeros), bits, group)


def qpacked_bytes(N: int, K: int, bits: int, group: int) -> int:
    """Bytes of a quantisation-only delta: b bits per weight plus one fp16 (scale, zero) pair per group."""
    return N * K * bits // 8 + 4 * N * K // group


# ----------------------------------------------------------------------------- request -> delta ids
def ids_uniform(T: int, D: int, gen: torch.Generator) -> torch.Tensor:
    return torch.randint(0, D, (T,), generator=gen, device=gen.device, dtype=torch.int64).to(torch.int32)


def ids_zipf(T: int, D: int, s: float, gen: torch.Generator) -> torch.Tensor:
    """Popularity p(rank r) ~ r^-s over D deltas (rank 1 = delta 0), iid per token."""
    w = torch.arange(1, D + 1, dtype=torch.float64, device=gen.device) ** (-s)
    return torch.multinomial((w / w.sum()).to(torch.float32), T, replacement=True,
                             generator=gen).to(torch.int32)


def ids_segments(T: int, D: int, gen: torch.Generator) -> torch.Tensor:
    """D contiguous segments with positive random lengths summing to T (a random composition),
    segment i served by delta i: the shape of a prefill batch of D prompts."""
    assert T >= D
    cuts = (torch.randperm(T - 1, generator=gen, device=gen.device)[: D - 1] + 1).sort().values
    bounds = torch.cat([torch.zeros(1, dtype=cuts.dtype, device=cuts.device), cuts,
                        torch.full((1,), T, dtype=cuts.dtype, device=cuts.device)])
    lens = bounds[1:] - bounds[:-1]
    return torch.repeat_interleave(torch.arange(D, device=gen.device), lens).to(torch.int32)


# ------------------------------------------------------------------------------------- the configs
@dataclass
class LayerSpec:
    name: str
    N: int
    K: int
    count: int = 1      # how many projections of this shape one transformer layer has


@dataclass
class Config:
    name: str
    shapes: List[LayerSpec]
    D: int
    bits: int
    group: int
    delta_std: float
    T: int
    ids: str                    # "uniform" | "zipf1.5" | "segments"
    layers: int = 1             # transformer layers in the model the shapes come from
    base_std: float = 0.02

    def make_ids(self, gen: torch.Generator) -> torch.Tensor:
        if self.ids == "uniform":
            return ids_uniform(self.T, self.D, gen)
        if self.ids == "zipf1.5":
            return ids_zipf(self.T, self.D, 1.5, gen)
        if self.ids == "segments":
            return ids_segments(self.T, self.D, gen)
        raise ValueError(self.ids)


def _llama(h: int, ffn: int, kv: Optional[int] = None) -> List[LayerSpec]:
    kv = h if kv is None else kv
    if kv == h:
        return [LayerSpec("qkvo", h, h, 4), LayerSpec("gate_up", ffn, h, 2), LayerSpec("down", h, ffn, 1)]
    return [LayerSpec("qo", h, h, 2), LayerSpec("kv", kv, h, 2), LayerSpec("gate_up", ffn, h, 2),
            LayerSpec("down", h, ffn, 1)]


CONFIGS: Dict[str, Config] = {
    "tiny": Config("tiny", [LayerSpec("lin", 256, 256, 1)], D=4, bits=4, group=64, delta_std=0.002,
                   T=8, ids="uniform"),
    "7b_decode": Config("7b_decode", _llama(4096, 11008), D=8, bits=4, group=128, delta_std=0.002,
                        T=32, ids="uniform", layers=32),
    "7b_decode_many": Config("7b_decode_many", _llama(4096, 11008), D=32, bits=2, group=128,
                             delta_std=0.001, T=64, ids="zipf1.5", layers=32),
    "13b_prefill": Config("13b_prefill", _llama(5120, 13824), D=16, bits=4, group=128,
                          delta_std=0.002, T=2048, ids="segments", layers=40),
    "70b_stack": Config("70b_stack", _llama(8192, 28672, kv=1024), D=4, bits=2, group=128,
                        delta_std=0.002, T=64, ids="uniform", layers=80),
}


def config(name: str) -> Config:
    return CONFIGS[name]


# ------------------------------------------------------------------- whole projections of a config
@dataclass
class Projection:
    """Inputs of one linear layer of a config: base weight, D delta tables, activations."""
    name: str
    N: int
    K: int
    W: torch.Tensor
    tabs: List[DeltaTables]
    x: torch.Tensor


def projections_of(cfg: Config) -> List[Tuple[str, int, int]]:
    """(name, N, K) of every linear projection of one transformer layer, in execution order."""
    out = []
    for s in cfg.shapes:
        for i in range(s.count):
            out.append((f"{s.name}{i}", s.N, s.K))
    return out


def launch_groups(cfg: Config) -> List[List[int]]:
    """Indices into projections_of(cfg), grouped by the activation they read: q, k and v read the
    layer input, gate and up read the attention block's output, o and down read tensors of their
    own.  Projections of one group can be served by one grouped call."""
    names = [n for n, _, _ in projections_of(cfg)]
    first = {"qkvo0": "qkv", "qkvo1": "qkv", "qkvo2": "qkv", "qo0": "qkv", "kv0": "qkv", "kv1": "qkv",
             "gate_up0": "gate_up", "gate_up1": "gate_up"}
    groups: Dict[str, List[int]] = {}
    order: List[List[int]] = []
    for i, n in enumerate(names):
        key = first.get(n)
        if key is None:
            order.append([i])
        elif key in groups:
            groups[key].append(i)
        else:
            groups[key] = [i]
            order.append(groups[key])
    return order


def make_projection(cfg: Config, seed: int, layer: int, name: str, N: int, K: int,
                    device: str = "cpu", with_tables: bool = True) -> Projection:
    """All tensors of one projection, each from its own sub-stream keyed by
    (config, layer, projection, tensor kind, delta id)."""
    key = (cfg.name, layer, name)
    W = make_base(N, K, stream(seed, *key, "W", device=device), cfg.base_std)
    x = make_x(cfg.T, K, stream(seed, *key, "x", device=device))
    tabs = []
    if with_tables:
        tabs = [make_delta_tables(N, K, cfg.bits, cfg.group, stream(seed, *key, "delta", m, device=device),
                                  std=cfg.delta_std) for m in range(cfg.D)]
    return Projection(name, N, K, W, tabs, x)


def algorithmic_bytes(N: int, K: int, T: int, bits: int, group: int, n_active: int) -> int:
    """Bytes one fused linear call must move at least: the base weight, the packed deltas that
    have at least one request, x, out and the index vector."""
    packed = N * K * (2 * bits + 4) // 32 + 4 * N * K // group
    return 2 * N * K + n_active * packed + 2 * T * K + 2 * T * N + 4 * T
