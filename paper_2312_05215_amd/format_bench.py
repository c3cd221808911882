"""Compressed-matmul comparison on one matrix (paper Section 4.1: 2:4 sparsity + quantisation against
quantisation alone and against fp16, at inputs of 1 .. 4096 rows), on this library's kernels:

  fp16      dz_base_gemm            x . W^T                       2 N K bytes,   2 T N K flops
  sparse    dz_sbmm                 x . delta^T, 2:4 + b bits     N K (2b+4)/32 + 4 N K / G bytes, T N K flops (kept values)
  quant     dz_qsbmm                x . delta^T, b bits only      N K b / 8 + 4 N K / G bytes,     2 T N K flops
  linear    dz_linear               x . W^T + x . delta^T (2:4), one fused launch
  qlinear   dz_qlinear              the same with the quantisation-only delta
  merged    dz_base_gemm on f16(W + delta) (one dense product; forming the merged weight with
            dz_merge_delta is timed separately: it is paid once per variant, not per call)

Every request of the batch names the one delta.  Each timed call reads a different copy of the matrix
(enough copies to exceed the 256 MB last-level cache), inputs are random codes: only the timing matters
here, parity is the tests' business.  Prints one table per shape and bit width.

    python -m paper_2312_05215_amd.format_bench [--shapes 4096x4096,13824x5120] [--bits 4,2] [--iters 40]
"""
from __future__ import annotations

import argparse

import torch

from . import binding as dz


def _time(fn, n_copies, iters, stream):
    for i in range(min(3, iters)):
        fn(i % n_copies)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(iters):
        fn(i % n_copies)
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters          # microseconds per call


def run(N, K, bits, G, Ts, iters):
    dev = "cuda"
    stream = torch.cuda.current_stream()
    w_bytes = 2 * N * K
    n_copies = max(2, (600 << 20) // w_bytes + 1)
    gen = torch.Generator(device=dev).manual_seed(0)
    rows = []
    with dz.Context(0) as c:
        W = [torch.randn(N, K, device=dev, dtype=torch.float16, generator=gen) * 0.02 for _ in range(n_copies)]
        scale = torch.full((N, K // G), 2e-4, dtype=torch.float16, device=dev)
        zero = torch.full((N, K // G), float((1 << bits) // 2), dtype=torch.float16, device=dev)
        pairs = torch.tensor([[0, 1], [0, 2], [0, 3], [1, 2], [1, 3], [2, 3]], dtype=torch.uint8, device=dev)
        sp, qp = [], []
        for _ in range(n_copies):
            codes = torch.randint(0, 1 << bits, (N, K // 2), device=dev, dtype=torch.uint8, generator=gen)
            idx = pairs[torch.randint(0, 6, (N, K // 4), device=dev, generator=gen)].reshape(N, K // 2).contiguous()
            p = torch.empty(dz.dz_packed_bytes(N, K, bits, G), dtype=torch.uint8, device=dev)
            dz.dz_pack_delta(c.h, codes, idx, scale, zero, N, K, bits, G, p)
            sp.append(p)
            qcodes = torch.randint(0, 1 << bits, (N, K), device=dev, dtype=torch.uint8, generator=gen)
            q = torch.empty(dz.dz_qpacked_bytes(N, K, bits, G), dtype=torch.uint8, device=dev)
            dz.dz_qpack_delta(c.h, qcodes, scale, zero, N, K, bits, G, q)
            qp.append(q)
            del codes, idx, qcodes
        merged = torch.empty(N, K, dtype=torch.float16, device=dev)
        t_merge = _time(lambda i: dz.dz_merge_delta(c.h, W[i], sp[i], N, K, bits, G, merged), n_copies, iters, stream)
        for T in Ts:
            x = torch.randn(T, K, device=dev, dtype=torch.float16, generator=gen)
            ids = torch.zeros(T, dtype=torch.int32, device=dev)
            out = torch.empty(T, N, dtype=torch.float16, device=dev)
            t = {
                "fp16": _time(lambda i: dz.dz_base_gemm(c.h, x, W[i], out, T, N, K), n_copies, iters, stream),
                "sparse": _time(lambda i: dz.dz_sbmm(c.h, x, [sp[i]], ids, out, T, N, K, bits, G, 0), n_copies, iters, stream),
                "quant": _time(lambda i: dz.dz_qsbmm(c.h, x, [qp[i]], ids, out, T, N, K, bits, G, 0), n_copies, iters, stream),
                "linear": _time(lambda i: dz.dz_linear(c.h, x, W[i], [sp[i]], ids, out, T, N, K, bits, G), n_copies, iters, stream),
                "qlinear": _time(lambda i: dz.dz_qlinear(c.h, x, W[i], [qp[i]], ids, out, T, N, K, bits, G), n_copies, iters, stream),
            }
            rows.append((T, t))
        assert dz.dz_check(c.h) == dz.DZ_OK
    sp_bytes, q_bytes = dz.dz_packed_bytes(N, K, bits, G), dz.dz_qpacked_bytes(N, K, bits, G)
    print(f"\n{N}x{K}, {bits}-bit, group {G}: fp16 {w_bytes / 1e6:.1f} MB, 2:4+quant {sp_bytes / 1e6:.2f} MB, "
          f"quant-only {q_bytes / 1e6:.2f} MB; dz_merge_delta {t_merge:.1f} us (once per variant)")
    print("| T | fp16 us | sparse us | quant us | quant/sparse | linear us | qlinear us | merged us (= fp16) | "
          "sparse GB/s | quant GB/s | sparse TF/s (TNK) | quant TF/s (2TNK) | linear TF/s (3TNK) | merged TF/s (2TNK) |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    for T, t in rows:
        tnk = T * N * K
        print(f"| {T} | {t['fp16']:.1f} | {t['sparse']:.1f} | {t['quant']:.1f} | {t['quant'] / t['sparse']:.2f} | "
              f"{t['linear']:.1f} | {t['qlinear']:.1f} | {t['fp16']:.1f} | {sp_bytes / t['sparse'] / 1e3:.0f} | "
              f"{q_bytes / t['quant'] / 1e3:.0f} | {tnk / t['sparse'] / 1e6:.1f} | {2 * tnk / t['quant'] / 1e6:.1f} | "
              f"{3 * tnk / t['linear'] / 1e6:.1f} | {2 * tnk / t['fp16'] / 1e6:.1f} |")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shapes", default="4096x4096,13824x5120")
    ap.add_argument("--bits", default="4,2")
    ap.add_argument("--group", type=int, default=128)
    ap.add_argument("--rows", default="1,4,16,64,256,2048")
    ap.add_argument("--iters", type=int, default=40)
    a = ap.parse_args()
    print(f"device: {torch.cuda.get_device_name(0)}; us per call, mean of {a.iters} calls over distinct copies")
    for shp in a.shapes.split(","):
        N, K = (int(v) for v in shp.split("x"))
        for b in a.bits.split(","):
            run(N, K, int(b), a.group, [int(v) for v in a.rows.split(",")], a.iters)
            print(f"  done {shp} {b}-bit", flush=True)


if __name__ == "__main__":
    main()
