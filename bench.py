#!/usr/bin/env python3
"""Benchmark: throughput of the base-GEMM + SBMM linear layers on one MI355X.

Headline workload (`7b_decode`): a Llama-7B-shaped stack of linear projections per transformer
layer -- q,k,v,o 4096x4096, gate,up 11008x4096, down 4096x11008, fp16 base ~N(0,0.02) -- with 8
resident deltas (4-bit codes, 2:4 sparse, group 128) and a decode batch of 32 request rows whose
delta ids are uniform over the 8 deltas.  One *step* is one pass over all linear projections of
all 32 layers -- request reordering, base product, SBMM and merge for all 224 projections, issued
as 128 calls (q,k,v share one dz_linear_group call, gate,up another; --no-group issues 224) --,
every layer with its own weights and deltas resident in HBM (about 34 GB, far beyond the 256 MB
last-level cache).  Attention, norms, embeddings and sampling are not part of the path.  Inputs are
seeded and synthetic; no file is read except the counter summaries under profiles/.

A default run (no --workload) times the headline workload and then, more briefly, the other three
performance configurations, whose figures go into the `workloads` object of the same JSON line:
7b_decode_many (32 deltas, 2-bit, Zipf ids, 64 rows, all 32 layers resident), 70b_stack (Llama-70B
shapes, 4 deltas, 2-bit, 64 rows, all 80 layers = 214 GB resident) and 13b_prefill (2048 request
rows in 16 prompt segments, all 40 layers resident; runs the tiled MFMA kernel and is priced against
the fp16 MFMA peak instead of HBM).  `--workload X` times X alone as the primary figure.

Prints ONE JSON line.  value = request rows (tokens) per second through the whole stack of layers;
roofline.achieved = algorithmic bytes (or flops) of all launches of a step / step time, so launch
gaps count against it; the measured ceilings of the device (a plain streaming read, a register-only
MFMA loop) are printed beside the nominal peaks.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
PERF_WORKLOADS = ["7b_decode", "7b_decode_many", "70b_stack", "13b_prefill"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, choices=PERF_WORKLOADS + ["tiny"],
                    help="time this workload alone (default: 7b_decode as the headline plus the other three, briefly)")
    ap.add_argument("--layers", type=int, default=0, help="distinct resident layers (0 = all of the model)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="default run: skip the three secondary workloads")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the streaming-read and MFMA-loop probes")
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
    ap.add_argument("--check", action="store_true",
                    help="after timing, compare sampled output features of layer 0 with the CPU oracle")
    ap.add_argument("--seed", type=int, default=0)
    return ap.parse_args()


def profile_traffic(kernel: str, workload: str, launches_per_layer: int):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this kernel and workload, if one exists
    for the same launch grouping.  A stored figure of an earlier run of the same command, not measured in this run."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    try:
        prof = {}
        for ln in open(path):
            if ln.startswith("traffic_"):
                k, v = ln.split(":")
                prof[k] = int(v)
        if prof.get("traffic_launches_per_layer") == launches_per_layer:
            return prof.get("traffic_bytes_per_launch"), os.path.relpath(path, ROOT)
    except (OSError, ValueError):
        pass
    return None, None


def run_workload(args, name, steps, warmup, with_cpu, primary):
    """Build the workload in HBM, time `steps` steps, return its result dictionary (and free everything)."""
    import torch
    import dz_synth as S
    import paper_2312_05215_amd as dz

    dev = "cuda"
    cfg = S.config(name)
    n_layers = args.layers if (args.layers > 0 and primary) else cfg.layers
    projs = S.projections_of(cfg)
    ctx = dz.Context(0)
    if cfg.T > 64:
        ctx.set_option(dz.DZ_OPT_REUSE_SEGMENTS, 1)      # the projections of a layer share one index vector
    nbytes = {(N, K): dz.dz_packed_bytes(N, K, cfg.bits, cfg.group) for _, N, K in projs}

    ids = cfg.make_ids(S.stream(args.seed, cfg.name, "ids"))
    n_active = int(ids[(ids >= 0) & (ids < cfg.D)].unique().numel())
    d_ids = ids.to(dev)

    t0 = time.time()
    layers = []          # per layer: list of (N, K, W, [packed], x, out)
    host_layer0 = None   # canonical tables of layer 0 on the host, for the CPU baseline
    check_layer0 = []    # layer 0's projections as generated, for the output check
    for l in range(n_layers):
        row = []
        keep = []
        for pname, N, K in projs:
            p = S.make_projection(cfg, args.seed, l, pname, N, K, device=dev)
            packed = []
            for t in p.tabs:
                buf = torch.empty(nbytes[(N, K)], dtype=torch.uint8, device=dev)
                dz.dz_pack_delta(ctx.h, t.codes, t.idx, t.scale, t.zero, N, K, cfg.bits, cfg.group, buf)
                packed.append(buf)
            out = torch.empty(cfg.T, N, dtype=torch.float16, device=dev)
            row.append((N, K, p.W, packed, p.x, out))
            if l == 0 and with_cpu:
                keep.append((pname, N, K, p.W.cpu(), [t.to("cpu") for t in p.tabs], p.x.cpu()))
            if l == 0 and args.check and primary:
                check_layer0.append((pname, N, K, p))
            del p
        if l == 0:
            host_layer0 = keep
        layers.append(row)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    resident_bytes = sum(W.numel() * 2 + sum(pk.numel() for pk in packed) for row in layers for _, _, W, packed, _, _ in row)

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

    path = args.path if primary else "linear"
    grouped = not args.no_group and path == "linear"
    step = step_grouped if grouped else step_single
    no_compare = args.no_compare or not primary
    if path != "linear":
        step = step_part
        no_compare = True

    if args.copy_calibration and primary:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)          # 1 GiB read + 1 GiB written by one elementwise kernel
        torch.cuda.synchronize()
        del src, dst

    # events are recorded on torch's current stream, which is the stream the binding launches on
    def timed(fn, n, w):
        for _ in range(w):
            fn()
        assert dz.dz_check(ctx.h) == dz.DZ_OK
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(n):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        assert dz.dz_check(ctx.h) == dz.DZ_OK
        return ev0.elapsed_time(ev1) / n

    if args.graph and primary:
        step()                                  # eager once: sizes the library's workspace
        assert dz.dz_check(ctx.h) == dz.DZ_OK
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        ms_per_step = timed(graph.replay, steps, warmup)
    else:
        ms_per_step = timed(step, steps, warmup)
    # the same work as one call per projection, for comparison (not part of `value`)
    ms_other = None if no_compare else timed(step_single if grouped else step_grouped, max(1, steps // 2), 1)

    # a model pass over the cfg.layers layers: scale if fewer distinct layers were made resident
    ms_model = ms_per_step * cfg.layers / n_layers
    tokens_per_s = cfg.T / (ms_model * 1e-3)

    # kernel launches per layer: one per call for small batches; large batches run one tiled kernel per projection
    launches_per_layer = len(groups) if (grouped and cfg.T <= 64) else len(projs)
    launches_per_step = n_layers * launches_per_layer
    act = 0 if path == "base" else n_active
    bytes_per_step = n_layers * sum(S.algorithmic_bytes(N, K, cfg.T, cfg.bits, cfg.group, act) - (2 * N * K if path == "sbmm" else 0)
                                    for _, N, K in projs)
    avg_launch_us = ms_per_step * 1e3 / launches_per_step
    achieved = bytes_per_step / (ms_per_step * 1e-3) / 1e9
    traffic, traffic_src = (profile_traffic("stream_kernel" if cfg.T <= 64 else "prefill_kernel", cfg.name, launches_per_layer)
                            if path == "linear" else (None, None))
    roofline = {"bound": "hbm", "kernel": "stream_kernel (fused base GEMM + SBMM)", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": traffic_src,
                "bytes_per_launch_avg": bytes_per_step // launches_per_step,
                "avg_launch_us": round(avg_launch_us, 2), "launches_per_step": launches_per_step}
    if cfg.T > 64:
        # large batches run the tiled MFMA kernel: 2*T*N*K flops of the base product plus 2*T*N*K/2 of the
        # 2:4-sparse delta product for every request row that names a delta
        rows_with_delta = int(((ids >= 0) & (ids < cfg.D)).sum())
        dense_rows = 0 if path == "sbmm" else cfg.T
        sparse_rows = 0 if path == "base" else rows_with_delta
        flops_per_step = n_layers * sum(2.0 * N * K * (dense_rows + 0.5 * sparse_rows) for _, N, K in projs)
        tf = flops_per_step / (ms_per_step * 1e-3) / 1e12
        kname = {"linear": "prefill_kernel (fused base GEMM + SBMM)", "base": "tile_kernel (base GEMM)",
                 "sbmm": "prefill_kernel (SBMM)"}[path]
        roofline = {"bound": "mfma", "kernel": kname, "achieved": round(tf, 1),
                    "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / MFMA_F16_PEAK_TFLOPS, 4),
                    "traffic": traffic, "traffic_source": traffic_src,
                    "flops_per_launch_avg": int(flops_per_step // launches_per_step),
                    "avg_launch_us": round(avg_launch_us, 2), "launches_per_step": launches_per_step}

    checked = None
    if check_layer0:
        # sampled output features of every projection of layer 0, as the timed step left them, against the oracle
        import numpy as np
        import oracle
        step()                                  # the timed configuration once more: the comparison run above wrote `out` last
        torch.cuda.synchronize()
        worst = 0.0
        for j, (pname, N, K, p) in enumerate(check_layer0):
            out = layers[0][j][5]
            gi = next(g for g in groups if j in g)
            x = layers[0][gi[0] if grouped else j][4]
            rows = torch.as_tensor(sorted(set([0, 15, 16, N // 2, N - 17, N - 1] + list(range(7, N, max(1, N // 40))))), device=dev)
            dense = []
            for t in p.tabs:
                s = t.rows(rows).to("cpu")
                dense.append(oracle.c.dequant(s.codes.numpy(), s.idx.numpy(), s.scale.numpy(), s.zero.numpy(), cfg.bits, cfg.group))
            ref = oracle.c.linear(x.cpu().numpy(), p.W[rows].cpu().numpy(), dense, ids.numpy())
            got = out[:, rows].float().cpu().numpy()
            rms = float(np.sqrt((ref.astype(np.float64) ** 2).mean()))
            rel = float((np.abs(got - ref) / np.maximum(np.abs(ref), rms)).max())
            assert rel <= 1e-2 and float(np.abs(got - ref).mean()) <= 1e-3, (pname, rel)
            worst = max(worst, rel)
        checked = {"projections": len(check_layer0), "max_rel_err": worst}
        check_layer0 = []

    cpu = None
    if with_cpu and host_layer0:
        import oracle
        idn = ids.numpy()

        def one_projection(entry):
            pname, N, K, W, tabs, x = entry
            dense = [oracle.c.dequant(t.codes.numpy(), t.idx.numpy(), t.scale.numpy(), t.zero.numpy(), cfg.bits, cfg.group)
                     for t in tabs]
            oracle.c.linear(x.numpy(), W.numpy(), dense, idn)

        all_threads = oracle.c.num_threads()
        t1 = time.time()
        passes = 0
        while passes == 0 or time.time() - t1 < 10.0:      # about 10 s of CPU work, whole passes over layer 0
            for entry in host_layer0:
                one_projection(entry)
            passes += 1
        cpu_s = (time.time() - t1) / passes
        # one thread: the first projection only (its share of the layer's multiply-adds scales the time up)
        oracle.c.set_threads(1)
        t2 = time.time()
        one_projection(host_layer0[0])
        one_s = time.time() - t2
        oracle.c.set_threads(all_threads)
        share = host_layer0[0][1] * host_layer0[0][2] / sum(N * K for _, N, K in projs)
        model = "unknown"
        try:
            for ln in open("/proc/cpuinfo"):
                if ln.startswith("model name"):
                    model = ln.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        cpu = {"value": round(cfg.T / (cpu_s * cfg.layers), 4), "unit": "tokens/s", "cores": all_threads,
               "kind": "oracle", "cpu_model": model,
               "sample": f"layer 0 of {cfg.layers} (all {len(projs)} projections: dense dequantisation of {cfg.D} deltas "
                         f"+ per-request dot products), {passes} passes, {cpu_s:.2f} s per pass; value extrapolates "
                         f"x{cfg.layers} layers",
               "single_thread": {"value": round(cfg.T / (one_s / share * cfg.layers), 5), "unit": "tokens/s", "cores": 1,
                                 "sample": f"projection {host_layer0[0][0]} of layer 0 ({host_layer0[0][1]}x{host_layer0[0][2]}, "
                                           f"{share:.3f} of the layer's multiply-adds) in {one_s:.2f} s; value extrapolates to "
                                           f"the layer by that share and x{cfg.layers} layers"}}

    ceilings = None
    if primary and not args.no_ceilings:
        big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(3)     # 1 GiB: beyond every cache
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dz.dz_probe_read(ctx.h, big, big.numel())
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            dz.dz_probe_read(ctx.h, big, big.numel())
        e1.record()
        torch.cuda.synchronize()
        read_gbs = 5 * big.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del big
        dz.dz_probe_mfma(ctx.h, 64)
        torch.cuda.synchronize()
        e0.record()
        flops = dz.dz_probe_mfma(ctx.h, 4096)
        e1.record()
        torch.cuda.synchronize()
        mfma_tf = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
        ceilings = {"streaming_read_GBps": round(read_gbs, 1), "streaming_read_frac_of_peak": round(read_gbs / HBM_PEAK_GBS, 4),
                    "mfma_f16_loop_TFLOPps": round(mfma_tf, 1), "mfma_frac_of_peak": round(mfma_tf / MFMA_F16_PEAK_TFLOPS, 4),
                    "how": "dz_probe_read: 1 GiB read once per launch with 16-byte loads, 5 launches; dz_probe_mfma: 4096 x 32 "
                           "register-only 16x16x32 fp16 MFMAs per wave, 16 waves per CU"}

    res = {
        "metric": "SBMM+base decode tokens/s and achieved HBM GB/s (% of peak) per layer" if cfg.T <= 64 else
                  "SBMM+base prefill tokens/s and achieved fp16 MFMA TFLOP/s (% of peak) per layer",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": cfg.name, "layers": cfg.layers, "resident_layers": n_layers,
                   "resident_GB": round(resident_bytes / 1e9, 1), "tokens": cfg.T,
                   "deltas": cfg.D, "active_deltas": n_active, "bits": cfg.bits, "group": cfg.group,
                   "projections_per_layer": len(projs), "launches_per_layer": launches_per_layer,
                   "grouping": "q,k,v in one call; gate,up in one call" if grouped else "one call per projection",
                   "path": {"linear": "fused layer (dz_linear / dz_linear_group)", "base": "dz_base_gemm only",
                            "sbmm": "dz_sbmm only"}[path],
                   "submission": "replays of one HIP graph of the step" if (args.graph and primary) else "eager launches",
                   "gen_seconds": round(gen_s, 1)},
        ("ms_per_step_one_call_per_projection" if grouped else "ms_per_step_grouped"):
            None if ms_other is None else round(ms_other, 4),
        "hbm_gbs": round(achieved, 1), "hbm_frac_of_peak": round(achieved / HBM_PEAK_GBS, 4),
        "us_per_layer": round(ms_per_step * 1e3 / n_layers, 2),
        "roofline": roofline, "cpu_baseline": cpu, "ceilings": ceilings, "checked": checked,
    }
    ctx.close()
    del layers, host_layer0
    gc.collect()
    torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    head = args.workload or "7b_decode"
    r = run_workload(args, head, args.steps, args.warmup, with_cpu=not args.no_cpu_baseline, primary=True)
    line = {
        "metric": r["metric"], "value": r["value"], "unit": r["unit"], "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
    }
    for k, v in r.items():
        if k not in line:
            line[k] = v
    if args.workload is None and not args.no_others and args.path == "linear" and not args.graph:
        others = {}
        for name in PERF_WORKLOADS:
            if name == head:
                continue
            # few steps: these runs only have to be long enough to time (a 70B step is 80 layers)
            o = run_workload(args, name, max(3, args.steps // 4), 1, with_cpu=False, primary=False)
            others[name] = {k: o[k] for k in ("metric", "value", "unit", "steps", "ms_per_step", "us_per_layer", "config", "roofline")}
        line["workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
