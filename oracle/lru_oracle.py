"""Replacement rule of the resident-delta cache, written out plainly -- TEST INFRASTRUCTURE ONLY.

The serving engine keeps a bounded number of compressed deltas on the GPU and brings others in on
demand (paper Section 5.1; Section 5.4, paragraph "Scalability").  The paper fixes no replacement
rule; the reading taken is least-recently-used, with two additions the asynchronous copies need:
slots handed out by the current call or by the previous call are never evicted (their deltas may
still be read by work that has not run yet), and empty slots are filled before anything is evicted.

`plan(slots, calls)` replays a list of calls, each a list of keys, and returns per call the list of
(slot, hit) pairs -- the decisions dz_cache_acquire must take -- or None for a call that cannot be
served (more keys to bring in than slots outside this and the previous call's), which changes
nothing.

Pins (tests/test_cache_policy.py): with one key per call the rule is textbook LRU, whose fault
count on the classic 20-reference string with 3 frames is 12; hits never move a delta; with at
least as many slots as distinct keys nothing is ever evicted.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple


def plan(slots: int, calls: Sequence[Sequence[int]]) -> List[Optional[List[Tuple[int, int]]]]:
    key_of = [None] * slots          # delta held by each slot
    last_use = [0] * slots           # logical time the slot was last handed out
    call_of = [-2] * slots           # number of the call that last handed it out
    clock = 0
    call_no = 0
    out = []
    for keys in calls:
        if not keys:                 # a call without keys does nothing: it is not "the previous call" afterwards
            out.append([])
            continue
        wanted = set(keys)
        missing = sum(1 for k in wanted if k not in key_of)
        available = sum(1 for s in range(slots)
                        if key_of[s] is None or (call_of[s] != call_no and key_of[s] not in wanted))
        if missing > available:
            out.append(None)
            continue
        prev, call_no = call_no, call_no + 1
        res = []
        for k in keys:
            if k in key_of:
                s, hit = key_of.index(k), 1
            else:
                hit = 0
                empty = [t for t in range(slots) if key_of[t] is None]
                if empty:
                    s = empty[0]
                else:
                    cand = [t for t in range(slots)
                            if call_of[t] not in (prev, call_no) and key_of[t] not in wanted]
                    s = min(cand, key=lambda t: (last_use[t], t))
                key_of[s] = k
            clock += 1
            last_use[s] = clock
            call_of[s] = call_no
            res.append((s, hit))
        out.append(res)
    return out
