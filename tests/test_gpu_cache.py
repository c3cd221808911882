"""GPU: the resident-delta cache in front of the hot path.  Packed deltas live in pinned host
memory; each batch acquires the deltas it names (copied in on a second stream, least recently used
evicted), and dz_linear runs on the addresses the cache returns.  Results must match the CPU oracle
batch by batch (paper Section 5.1 Eq. (2)); the bytes in a slot must be the packed delta bit for bit;
the decisions must be those of oracle/lru_oracle.py."""
import numpy as np
import pytest
import torch

import dz_synth as S
from dzcase import Case, assert_close

pytestmark = pytest.mark.gpu


def _host_copies(case):
    """Pinned host copies of the case's packed deltas."""
    out = []
    for p in case.packed:
        h = torch.empty(p.numel(), dtype=torch.uint8, pin_memory=True)
        h.copy_(p)
        out.append(h)
    torch.cuda.synchronize()
    return out


def test_swapped_deltas_serve_batches(dz):
    import oracle
    from oracle import lru_oracle
    T, N, K, D, bits, G = 24, 96, 512, 10, 4, 128
    with dz.Context(0) as c:
        case = Case(dz, c.h, 60, T, N, K, D, bits, G, "uniform")
        nbytes = dz.dz_packed_bytes(N, K, bits, G)
        host = _host_copies(case)
        slots = 6
        cache = dz.dz_cache_create(0, slots, nbytes)
        copy_stream = torch.cuda.Stream()
        rng = np.random.default_rng(5)
        # batches of requests, each naming at most 3 of the 10 deltas (so two consecutive batches fit 6 slots)
        batches = []
        for b in range(12):
            names = rng.choice(D, size=int(rng.integers(1, 4)), replace=False)
            ids = rng.choice(np.concatenate([names, [-1]]), size=T)
            batches.append((list(map(int, names)), ids.astype(np.int32)))
        ref_plan = lru_oracle.plan(slots, [names for names, _ in batches])
        try:
            dx = case.dx
            acquired = []
            # copies of batch b+1 are enqueued before the compute of batch b: they overlap it
            acquired.append(dz.dz_cache_acquire(cache, batches[0][0], [host[m] for m in batches[0][0]], nbytes, copy_stream))
            outs = []
            for b, (names, ids) in enumerate(batches):
                if b + 1 < len(batches):
                    nn = batches[b + 1][0]
                    acquired.append(dz.dz_cache_acquire(cache, nn, [host[m] for m in nn], nbytes, copy_stream))
                rc, ptrs, s, h, ticket = acquired[b]
                assert list(zip(s, h)) == ref_plan[b], f"batch {b}"
                local = {m: i for i, m in enumerate(names)}
                lid = torch.tensor([local.get(int(m), -1) for m in ids], dtype=torch.int32, device="cuda")
                o = case.out(fill=7.0)
                print(f"cache batch {b} deltas {names}", flush=True)
                dz.dz_cache_wait(cache, ticket)            # the compute stream waits for this batch's copies only
                dz.dz_linear(c.h, dx, case.dW, ptrs, lid, o, T, N, K, bits, G)
                dz.dz_cache_release(cache, ticket)         # later evictions of these slots wait for this point
                outs.append((o, ids))
            assert dz.dz_check(c.h) == dz.DZ_OK
            torch.cuda.synchronize()
            for b, (o, ids) in enumerate(outs):
                ref = oracle.c.linear(case.x.numpy(), case.W.numpy(), case.dense, ids)
                assert_close(o, ref, f"batch {b}")
            # what sits in the slots of the last batch is the packed delta, bit for bit
            rc, ptrs, s, h, _ = acquired[-1]
            for m, ptr in zip(batches[-1][0], ptrs):
                codes = torch.empty(N, K // 2, dtype=torch.uint8, device="cuda")
                idx = torch.empty(N, K // 2, dtype=torch.uint8, device="cuda")
                dz.dz_unpack_delta(c.h, ptr, N, K, bits, G, codes=codes, idx=idx)
                torch.cuda.synchronize()
                assert torch.equal(codes.cpu(), case.tabs[m].codes)
                assert torch.equal(idx.cpu(), case.tabs[m].idx)
            hits, misses, evictions = dz.dz_cache_stats(cache)
            flat = [hh for r in ref_plan for _, hh in r]
            assert (hits, misses) == (sum(flat), len(flat) - sum(flat))
        finally:
            torch.cuda.synchronize()
            dz.dz_cache_destroy(cache)


def test_swap_in_rate(dz):
    """Not a pass/fail figure: prints the host-to-device rate of cold acquires (all misses), next to
    the rate of a plain pinned-memory copy of the same bytes by torch."""
    nbytes = 32 << 20
    n = 8
    host = [torch.empty(nbytes, dtype=torch.uint8, pin_memory=True).fill_(i + 1) for i in range(2 * n)]
    cache = dz.dz_cache_create(0, 2 * n, nbytes)
    copy_stream = torch.cuda.Stream()
    try:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for rnd in range(2):
            keys = list(range(rnd * n, rnd * n + n))
            torch.cuda.synchronize()
            e0.record()
            rc, ptrs, s, h, ticket = dz.dz_cache_acquire(cache, keys, [host[k] for k in keys], nbytes, copy_stream)
            dz.dz_cache_wait(cache, ticket)
            e1.record()                  # the compute stream now waits for the copies, so this event closes them
            dz.dz_cache_release(cache, ticket)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            assert h == [0] * n and len(set(ptrs)) == n
            print(f"swap-in round {rnd}: {n} x {nbytes >> 20} MiB in {ms:.2f} ms = {n * nbytes / ms / 1e6:.1f} GB/s", flush=True)
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        e0.record()
        for k in range(n):
            dst.copy_(host[k], non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        print(f"torch pinned copy: {n * nbytes / e0.elapsed_time(e1) / 1e6:.1f} GB/s", flush=True)
        e0.record()
        keys = list(range(n, 2 * n))
        rc, ptrs2, s2, h2, t2 = dz.dz_cache_acquire(cache, keys, [host[k] for k in keys], nbytes, copy_stream)
        dz.dz_cache_wait(cache, t2)
        e1.record()
        torch.cuda.synchronize()
        assert h2 == [1] * n and ptrs2 == ptrs
        print(f"all hits: {e0.elapsed_time(e1) * 1e3:.1f} us", flush=True)
    finally:
        torch.cuda.synchronize()
        dz.dz_cache_destroy(cache)


def test_copies_of_the_next_batch_run_under_the_compute_of_this_one(dz):
    """The swap-in pipeline overlaps: with batch b+1 acquired before the compute of batch b is
    enqueued, the copy interval of batch b+1 and the compute interval of batch b -- both taken with
    events against one common start -- intersect, and the copies do not wait for that compute to
    finish.  An eviction still waits for the last reader of the slot it overwrites (checked by
    values: every batch's output matches the oracle)."""
    import oracle
    T, N, K, bits, G = 32, 4096, 4096, 4, 128
    D = 6
    with dz.Context(0) as c:
        case = Case(dz, c.h, 61, T, 64, K, D, bits, G, "uniform")      # oracle-sized rows ...
        # ... stretched to a layer wide enough that one batch computes for a while: the 64 rows repeat
        reps = N // 64
        W = case.dW.repeat(reps, 1).contiguous()
        nbytes = dz.dz_packed_bytes(N, K, bits, G)
        host = []
        for t in case.tabs:
            dt = t.to("cuda")
            rep = lambda a: a.repeat(reps, 1).contiguous()
            p = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            dz.dz_pack_delta(c.h, rep(dt.codes), rep(dt.idx), rep(dt.scale), rep(dt.zero), N, K, bits, G, p)
            h = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
            h.copy_(p)
            host.append(h)
        torch.cuda.synchronize()
        slots = 4
        cache = dz.dz_cache_create(0, slots, nbytes)
        copy_stream = torch.cuda.Stream()
        batches = [[0, 1], [2, 3], [4, 5], [0, 1], [2, 3]]             # every batch after the second evicts
        n_launch = 40                                                   # launches per batch: a few ms of compute
        try:
            ev = lambda: torch.cuda.Event(enable_timing=True)
            origin = ev()
            spans = []      # per batch: (copy start, copy end, compute start, compute end) events
            outs = []
            torch.cuda.synchronize()
            origin.record()
            acq = []
            c0, c1 = ev(), ev()
            c0.record(copy_stream)
            acq.append(dz.dz_cache_acquire(cache, batches[0], [host[m] for m in batches[0]], nbytes, copy_stream))
            c1.record(copy_stream)
            copy_ev = [(c0, c1)]
            for b, names in enumerate(batches):
                if b + 1 < len(batches):
                    nn = batches[b + 1]
                    c0, c1 = ev(), ev()
                    c0.record(copy_stream)
                    acq.append(dz.dz_cache_acquire(cache, nn, [host[m] for m in nn], nbytes, copy_stream))
                    c1.record(copy_stream)
                    copy_ev.append((c0, c1))
                rc, ptrs, s, h, ticket = acq[b]
                local = {m: i for i, m in enumerate(names)}
                ids = torch.tensor([names[i % 2] for i in range(T)], dtype=torch.int32)
                lid = torch.tensor([local[int(m)] for m in ids], dtype=torch.int32, device="cuda")
                o = torch.full((T, N), 7.0, dtype=torch.float16, device="cuda")
                k0, k1 = ev(), ev()
                dz.dz_cache_wait(cache, ticket)
                k0.record()
                for _ in range(n_launch):
                    dz.dz_linear(c.h, case.dx, W, ptrs, lid, o, T, N, K, bits, G)
                k1.record()
                dz.dz_cache_release(cache, ticket)
                spans.append((k0, k1))
                outs.append((o, ids))
            torch.cuda.synchronize()
            assert dz.dz_check(c.h) == dz.DZ_OK
            t = lambda e: origin.elapsed_time(e)
            overlapped = 0
            for b in range(len(batches) - 1):
                cs, ce = t(copy_ev[b + 1][0]), t(copy_ev[b + 1][1])     # copies of batch b+1
                ks, ke = t(spans[b][0]), t(spans[b][1])                 # compute of batch b
                print(f"batch {b}: compute [{ks:.2f}, {ke:.2f}] ms, copies of batch {b + 1} [{cs:.2f}, {ce:.2f}] ms", flush=True)
                if ce > cs and min(ce, ke) - max(cs, ks) > 0.25 * min(ce - cs, ke - ks):
                    overlapped += 1
                # the compute of batch b+1 starts only after its copies
                assert t(spans[b + 1][0]) >= ce - 1e-3
            assert overlapped >= len(batches) - 2, overlapped
            for b, (o, ids) in enumerate(outs):
                ref = oracle.c.linear(case.x.numpy(), case.W.numpy(), case.dense, ids.numpy())
                assert_close(o[:, :64], ref, f"overlap batch {b}")
                assert torch.equal(o[:, :64], o[:, N - 64:])
        finally:
            torch.cuda.synchronize()
            dz.dz_cache_destroy(cache)
