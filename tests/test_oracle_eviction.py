"""Pins of the oracle's KV-eviction plan (Sec. 2: local patterns allow evicting the cache beyond the
attention span; applied to the mask of Sec. 4.3) against brute force over the mask itself: the plan
must keep every cached key some future row still attends, nothing else, and give each a fixed slot."""
import numpy as np

import oracle


def random_flags(seed, Hq, P):
    rng = np.random.default_rng(seed)
    d = np.zeros((Hq, P), np.uint8)
    v = np.zeros((Hq, P), np.uint8)
    for h in range(Hq):
        d[h, :int(rng.integers(1, 30))] = 1
        if rng.random() < 0.5:
            a = int(rng.integers(30, 60))
            d[h, a:a + int(rng.integers(1, 8))] = 1
        v[h, :int(rng.integers(1, 5))] = 1
        v[h, rng.choice(P, size=6, replace=False)] = 1
    d[Hq - 1] = 0                                   # a head without any diagonal
    return d, v


def test_plan_is_exactly_what_future_rows_attend():
    Hq, Hkv, P = 6, 3, 260
    d, v = random_flags(1, Hq, P)
    art = oracle.from_patterns(d, v)
    G = Hq // Hkv
    for p in (70, 128, 199):
        plan = oracle.eviction_plan(d, v, Hkv, p)
        for g in range(Hkv):
            # brute force: keys <= p attended by any row i in [p, P) of any head of the group
            needed = set()
            for h in range(g * G, (g + 1) * G):
                for i in range(p, P):
                    needed.update(int(j) for j in oracle.kept_list(art, h, i) if j <= p)
            W = int(plan.window[g])
            live = set(int(c) for c in plan.cols[plan.col_ptr[g]:plan.col_ptr[g + 1]])
            live |= set(range(max(0, p - W + 1), p + 1)) if W > 0 else set()
            assert needed <= live, f"group {g} at p = {p}: a needed key would be evicted"
            # nothing superfluous, as long as the rows that need the oldest window keys still exist (i < P)
            if p + W <= P:
                assert live <= needed, f"group {g} at p = {p}: {sorted(live - needed)[:5]} kept for nothing"


def test_slots_are_distinct_fixed_and_dense():
    Hq, Hkv, P = 4, 2, 300
    d, v = random_flags(2, Hq, P)
    for g in range(Hkv):
        seen_at = {}
        for p in (100, 101, 150, 299):
            plan = oracle.eviction_plan(d, v, Hkv, p)
            W = int(plan.window[g])
            ncol = int(plan.col_ptr[g + 1] - plan.col_ptr[g])
            live = sorted(set(int(c) for c in plan.cols[plan.col_ptr[g]:plan.col_ptr[g + 1]]) |
                          (set(range(max(0, p - W + 1), p + 1)) if W > 0 else set()))
            slots = [oracle.eviction_slot(plan, g, j) for j in live]
            assert len(set(slots)) == len(slots), "two live keys share a row"
            assert all(0 <= s < ncol + W for s in slots)
            # a window key keeps its ring position while p advances (columns found later shift the ring's
            # base, which is why the ring offset is compared, not the absolute row)
            for j, s in zip(live, slots):
                if s >= ncol:
                    assert s - ncol == j % W
                    seen_at.setdefault(j, s - ncol)
                    assert seen_at[j] == s - ncol


def test_group_union_and_degenerate_heads():
    d = np.zeros((2, 50), np.uint8)
    v = np.zeros((2, 50), np.uint8)
    d[0, :3] = 1
    d[1, 9] = 1
    v[0, 4] = 1
    v[1, [4, 7, 40]] = 1
    plan = oracle.eviction_plan(d, v, 1, 20)
    assert plan.window[0] == 10                       # the largest offset of either head, plus the key itself
    assert list(plan.cols) == [4, 7]                  # union, ascending; column 40 lies beyond p
    assert oracle.eviction_slot(plan, 0, 7) == 1 and oracle.eviction_slot(plan, 0, 15) == 2 + 15 % 10
    empty = oracle.eviction_plan(np.zeros((2, 50), np.uint8), np.zeros((2, 50), np.uint8), 2, 20)
    assert (empty.window == 0).all() and len(empty.cols) == 0 and oracle.eviction_slot(empty, 1, 3) == -1
