"""CPU: the resident-delta cache's decisions (no device: a cache created with device < 0 takes the
same decisions and copies nothing) against the plain statement of the rule in oracle/lru_oracle.py,
and that statement against what does not depend on it: the textbook LRU fault count, and invariants."""
import random

import pytest

import paper_2312_05215_amd as dz
from oracle import lru_oracle

# the classic page-reference string of operating-systems textbooks: 12 faults under LRU with 3 frames
TEXTBOOK = [7, 0, 1, 2, 0, 3, 0, 4, 2, 3, 0, 3, 2, 1, 2, 0, 1, 7, 0, 1]


def run_cache(slots, calls):
    c = dz.dz_cache_create(-1, slots, 1024)
    out = []
    try:
        for keys in calls:
            rc, ptrs, s, h, _ = dz.dz_cache_acquire(c, keys, None, 1024, check=False)
            if rc != dz.DZ_OK:
                assert rc == dz.DZ_ERR_ARG
                out.append(None)
            else:
                assert all(p == 0 for p in ptrs)
                out.append(list(zip(s, h)))
        stats = dz.dz_cache_stats(c)
    finally:
        dz.dz_cache_destroy(c)
    return out, stats


def test_oracle_is_textbook_lru_for_single_keys():
    res = lru_oracle.plan(3, [[k] for k in TEXTBOOK])
    assert sum(1 - hit for r in res for _, hit in r) == 12
    # and with 4 frames the same string faults 8 times
    res4 = lru_oracle.plan(4, [[k] for k in TEXTBOOK])
    assert sum(1 - hit for r in res4 for _, hit in r) == 8


def test_oracle_invariants():
    rng = random.Random(3)
    for trial in range(50):
        slots = rng.randint(2, 9)
        nkeys = rng.randint(1, 14)
        calls = [[rng.randrange(nkeys) for _ in range(rng.randint(1, 4))] for _ in range(40)]
        res = lru_oracle.plan(slots, calls)
        holder = {}                       # slot -> key, replayed from the decisions alone
        prev_slots = set()
        for keys, r in zip(calls, res):
            if r is None:
                continue
            assert len(r) == len(keys)
            now = set()
            for k, (s, hit) in zip(keys, r):
                assert 0 <= s < slots
                if hit:
                    assert holder.get(s) == k                 # a hit never moves a delta
                else:
                    assert k not in holder.values()           # a miss was really absent
                    assert s not in prev_slots and s not in now   # protected slots are not evicted
                    holder[s] = k
                now.add(s)
            prev_slots = now
        if nkeys <= slots:                # everything fits: each key is brought in once
            assert all(r is not None for r in res)
            assert sum(1 - hit for r in res for _, hit in r) == len({k for c in calls for k in c})


def test_library_matches_oracle_on_textbook_string():
    got, (hits, misses, evictions) = run_cache(3, [[k] for k in TEXTBOOK])
    assert got == lru_oracle.plan(3, [[k] for k in TEXTBOOK])
    assert (hits, misses, evictions) == (8, 12, 9)


@pytest.mark.parametrize("seed", range(8))
def test_library_matches_oracle_on_random_batches(seed):
    rng = random.Random(seed)
    slots = rng.randint(2, 12)
    nkeys = rng.randint(2, 30)
    calls = [[rng.randrange(nkeys) * 1000003 - 7 for _ in range(rng.randint(0, 5))] for _ in range(200)]
    got, (hits, misses, evictions) = run_cache(slots, calls)
    ref = lru_oracle.plan(slots, calls)
    assert [g if g else None for g in got] == [r if r else None for r in ref]
    flat = [h for r in ref if r for _, h in r]
    assert hits == sum(flat) and misses == len(flat) - sum(flat)


def test_argument_errors():
    with pytest.raises(dz.DzError):
        dz.dz_cache_create(-1, 0, 1024)
    c = dz.dz_cache_create(-1, 2, 1000)
    try:
        assert dz.dz_cache_acquire(c, [1, 2, 3], None, 1000, check=False)[0] == dz.DZ_ERR_ARG     # three keys, two slots
        assert dz.dz_cache_acquire(c, [1], None, 4096, check=False)[0] == dz.DZ_ERR_ARG           # larger than a slot
        assert dz.dz_cache_acquire(c, [1, 2], None, 1000)[0] == dz.DZ_OK
        # both slots belong to the previous call now: nothing new fits, and nothing changes
        assert dz.dz_cache_acquire(c, [3], None, 1000, check=False)[0] == dz.DZ_ERR_ARG
        rc, _, slots, hits, _ = dz.dz_cache_acquire(c, [2, 1], None, 1000)
        assert hits == [1, 1] and slots == [1, 0]
        assert dz.dz_cache_stats(c) == (2, 2, 0)
    finally:
        dz.dz_cache_destroy(c)
