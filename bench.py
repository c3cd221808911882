#!/usr/bin/env python3
"""Benchmark: decode throughput of the base-GEMM + SBMM linear layers on one MI355X.

Workload (`7b_decode`): a Llama-7B-shaped stack of linear projections per transformer layer --
q,k,v,o 4096x4096, gate,up 11008x4096, down 4096x11008, fp16 base ~N(0,0.02) -- with 8 resident
deltas (4-bit codes, 2:4 sparse, group 128) and a decode batch of 32 request rows whose delta ids
are uniform over the 8 deltas.  One *step* is one pass over all linear projections of all 32
layers -- request reordering, base product, SBMM and merge for all 224 projections, issued as 128
calls (q,k,v share one dz_linear_group call, gate,up another; --no-group issues 224) --, every layer
with its own weights and deltas resident in HBM (about 34 GB, far beyond the 256 MB last-level
cache).  Attention, norms, embeddings and sampling are not part of the path.  Inputs are seeded
and synthetic; no file is read.

`--workload` selects the other synthetic configurations (7b_decode_many: 32 deltas, 2-bit, Zipf ids,
64 rows; 70b_stack: Llama-70B shapes, 4 deltas; 13b_prefill: 2048 request rows in 16 prompt
segments, which runs the tiled MFMA kernel and is priced against the fp16 MFMA peak instead of HBM).

Prints ONE JSON line.  value = request rows (tokens) per second through the whole stack of layers;
roofline.achieved = algorithmic bytes (or flops) of all launches of a step / step time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="7b_decode",
                    choices=["7b_decode", "7b_decode_many", "13b_prefill", "70b_stack", "tiny"])
    ap.add_argument("--layers", type=int, default=0,
                    help="distinct resident layers (0 = all of the model; 4 for 13b_prefill and 8 for 70b_stack, "
                         "whose full stacks with all deltas would not leave room in 288 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-group", action="store_true",
                    help="one dz_linear call per projection instead of one dz_linear_group call for q,k,v and one for gate,up")
    ap.add_argument("--path", default="linear", choices=["linear", "base", "sbmm"],
                    help="which part of the layer is timed: the fused layer (default, the headline figure), "
                         "dz_base_gemm alone or dz_sbmm alone (one call per projection; for kernel profiles)")
    ap.add_argument("--graph", action="store_true",
                    help="record the step's launches into a HIP graph once and time its replays")
    ap.add_argument("--no-compare", action="store_true",
                    help="skip the extra timing of the other launch grouping (keeps a profile of the run to one kind of launch)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known traffic, for scaling rocprofv3 --pmc counters)")
    ap.add_argument("--seed", type=int, default=0)
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    import dz_synth as S
    import paper_2312_05215_amd as dz

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    cfg = S.config(args.workload)
    n_layers = args.layers if args.layers > 0 else {"13b_prefill": 4, "70b_stack": 8}.get(cfg.name, cfg.layers)
    projs = S.projections_of(cfg)
    ctx = dz.Context(0)
    nbytes = {(N, K): dz.dz_packed_bytes(N, K, cfg.bits, cfg.group) for _, N, K in projs}

    ids = cfg.make_ids(S.stream(args.seed, cfg.name, "ids"))
    n_active = int(ids.unique().numel())
    d_ids = ids.to(dev)

    t0 = time.time()
    layers = []          # per layer: list of (N, K, W, [packed], x, out)
    host_layer0 = None   # canonical tables of layer 0 for the CPU baseline
    for l in range(n_layers):
        row = []
        keep = []
        for name, N, K in projs:
            p = S.make_projection(cfg, args.seed, l, name, N, K, device=dev)
            packed = []
            for t in p.tabs:
                buf = torch.empty(nbytes[(N, K)], dtype=torch.uint8, device=dev)
                dz.dz_pack_delta(ctx.h, t.codes, t.idx, t.scale, t.zero, N, K, cfg.bits, cfg.group, buf)
                packed.append(buf)
            out = torch.empty(cfg.T, N, dtype=torch.float16, device=dev)
            row.append((N, K, p.W, packed, p.x, out))
            if l == 0 and not args.no_cpu_baseline:
                keep.append((name, N, K, p.W.cpu(), [t.to("cpu") for t in p.tabs], p.x.cpu()))
            del p
        if l == 0:
            host_layer0 = keep
        layers.append(row)
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    groups = S.launch_groups(cfg)

    def step_single():
        for row in layers:
            for N, K, W, packed, x, out in row:
                dz.dz_linear(ctx.h, x, W, packed, d_ids, out, cfg.T, N, K, cfg.bits, cfg.group)

    def step_grouped():
        # q,k,v read the same activation, so do gate and up: one call each (the x of the group's first
        # projection stands for the shared input); o and down go alone
        for row in layers:
            for gidx in groups:
                if len(gidx) == 1:
                    N, K, W, packed, x, out = row[gidx[0]]
                    dz.dz_linear(ctx.h, x, W, packed, d_ids, out, cfg.T, N, K, cfg.bits, cfg.group)
                else:
                    sel = [row[i] for i in gidx]
                    dz.dz_linear_group(ctx.h, sel[0][4], [r[2] for r in sel], [r[3] for r in sel], d_ids,
                                       [r[5] for r in sel], cfg.T, [r[0] for r in sel], sel[0][1], cfg.bits, cfg.group)

    def step_part():
        for row in layers:
            for N, K, W, packed, x, out in row:
                if args.path == "base":
                    dz.dz_base_gemm(ctx.h, x, W, out, cfg.T, N, K)
                else:
                    dz.dz_sbmm(ctx.h, x, packed, d_ids, out, cfg.T, N, K, cfg.bits, cfg.group, 0)

    grouped = not args.no_group and args.path == "linear"
    step = step_grouped if grouped else step_single
    if args.path != "linear":
        step = step_part
        args.no_compare = True

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)          # 1 GiB read + 1 GiB written by one elementwise kernel
        torch.cuda.synchronize()
        del src, dst

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        assert dz.dz_check(ctx.h) == dz.DZ_OK
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(steps):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        assert dz.dz_check(ctx.h) == dz.DZ_OK
        return ev0.elapsed_time(ev1) / steps

    if args.graph:
        step()                                  # eager once: sizes the library's workspace
        assert dz.dz_check(ctx.h) == dz.DZ_OK
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        ms_per_step = timed(graph.replay, args.steps, args.warmup)
    else:
        ms_per_step = timed(step, args.steps, args.warmup)
    # the same work as one call per projection, for comparison (not part of `value`)
    ms_other = None if args.no_compare else timed(step_single if grouped else step_grouped, max(1, args.steps // 2), 1)

    # a model pass over the cfg.layers layers: scale if fewer distinct layers were made resident
    ms_model = ms_per_step * cfg.layers / n_layers
    tokens_per_s = cfg.T / (ms_model * 1e-3)

    launches_per_step = n_layers * (len(groups) if grouped else len(projs))
    act = 0 if args.path == "base" else n_active
    bytes_per_step = n_layers * sum(S.algorithmic_bytes(N, K, cfg.T, cfg.bits, cfg.group, act) - (2 * N * K if args.path == "sbmm" else 0)
                                    for _, N, K in projs)
    avg_launch_us = ms_per_step * 1e3 / launches_per_step
    achieved = bytes_per_step / (ms_per_step * 1e-3) / 1e9
    # measured HBM bytes per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised under profiles/);
    # only quoted when the run launches the way the profiled run did
    traffic = None
    try:
        prof = {}
        for ln in open(os.path.join(ROOT, "profiles", "stream_kernel_7b_decode_pmc.txt")):
            if ln.startswith("traffic_"):
                k, v = ln.split(":")
                prof[k] = int(v)
        if cfg.name == "7b_decode" and prof.get("traffic_launches_per_layer") == launches_per_step // n_layers:
            traffic = prof.get("traffic_bytes_per_launch")
    except (OSError, ValueError):
        pass
    roofline = {"bound": "hbm", "kernel": "stream_kernel (fused base GEMM + SBMM)", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "bytes_per_launch_avg": bytes_per_step // launches_per_step,
                "avg_launch_us": round(avg_launch_us, 2), "launches_per_step": launches_per_step}
    if cfg.T > 64:
        # large batches run the tiled MFMA kernel: 2*T*N*K flops of the base product plus 2*T*N*K/2 of the
        # 2:4-sparse delta product for every request row that names a delta
        rows_with_delta = int(((ids >= 0) & (ids < cfg.D)).sum())
        dense_rows = 0 if args.path == "sbmm" else cfg.T
        sparse_rows = 0 if args.path == "base" else rows_with_delta
        flops_per_step = n_layers * sum(2.0 * N * K * (dense_rows + 0.5 * sparse_rows) for _, N, K in projs)
        tf = flops_per_step / (ms_per_step * 1e-3) / 1e12
        kname = {"linear": "prefill_kernel (fused base GEMM + SBMM)", "base": "tile_kernel (base GEMM)",
                 "sbmm": "prefill_kernel (SBMM)"}[args.path]
        roofline = {"bound": "mfma", "kernel": kname, "achieved": round(tf, 1),
                    "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / MFMA_F16_PEAK_TFLOPS, 4),
                    "traffic": None, "flops_per_launch_avg": int(flops_per_step // launches_per_step),
                    "avg_launch_us": round(avg_launch_us, 2), "launches_per_step": launches_per_step}

    cpu = None
    if not args.no_cpu_baseline and host_layer0:
        import numpy as np
        import oracle
        idn = ids.numpy()
        t1 = time.time()
        passes = 0
        while passes == 0 or time.time() - t1 < 10.0:      # about 10 s of CPU work, whole passes over layer 0
            for name, N, K, W, tabs, x in host_layer0:
                dense = [oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), cfg.bits, cfg.group)
                         for t in tabs]
                oracle.c.linear(x.numpy(), W.numpy(), dense, idn)
                del dense
            passes += 1
        cpu_s = (time.time() - t1) / passes
        cpu = {"value": round(cfg.T / (cpu_s * cfg.layers), 4), "unit": "tokens/s", "cores": oracle.c.num_threads(),
               "kind": "oracle",
               "sample": f"layer 0 of {cfg.layers} (all {len(projs)} projections: dense dequantisation of {cfg.D} deltas "
                         f"+ per-request dot products), {passes} passes, {cpu_s:.2f} s per pass; value extrapolates "
                         f"x{cfg.layers} layers"}

    line = {
        "metric": "SBMM+base decode tokens/s and achieved HBM GB/s (% of peak) per layer" if cfg.T <= 64 else
                  "SBMM+base prefill tokens/s and achieved fp16 MFMA TFLOP/s (% of peak) per layer",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": cfg.name, "layers": cfg.layers, "resident_layers": n_layers, "tokens": cfg.T,
                   "deltas": cfg.D, "active_deltas": n_active, "bits": cfg.bits, "group": cfg.group,
                   "projections_per_layer": len(projs), "launches_per_layer": len(groups) if grouped else len(projs),
                   "grouping": "q,k,v in one call; gate,up in one call" if grouped else "one call per projection",
                   "path": {"linear": "fused layer (dz_linear / dz_linear_group)", "base": "dz_base_gemm only",
                            "sbmm": "dz_sbmm only"}[args.path],
                   "submission": "replays of one HIP graph of the step" if args.graph else "eager launches",
                   "gen_seconds": round(gen_s, 1)},
        ("ms_per_step_one_call_per_projection" if grouped else "ms_per_step_grouped"):
            None if ms_other is None else round(ms_other, 4),
        "hbm_gbs": round(achieved, 1), "hbm_frac_of_peak": round(achieved / HBM_PEAK_GBS, 4),
        "us_per_layer": round(ms_per_step * 1e3 / n_layers, 2),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    ctx.close()


if __name__ == "__main__":
    main()
