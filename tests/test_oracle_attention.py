"""Pins of the oracle's masked attention (Sec. 3 and the end of Sec. 4.3) against library dense
causal attention, a brute-force dense softmax, and identities any correct implementation obeys."""
import numpy as np
import pytest
import torch

import oracle


def rand_qkv(rng, Hq, Hkv, S, d, scale=1.0):
    Q = (rng.standard_normal((Hq, S, d)) * scale).astype(np.float32)
    K = (rng.standard_normal((Hkv, S, d)) * scale).astype(np.float32)
    V = rng.standard_normal((Hkv, S, d)).astype(np.float32)
    return Q, K, V


def random_art(rng, H, S, L=0, p_diag=0.15, p_vert=0.1):
    d = (rng.random((H, S)) < p_diag).astype(np.uint8)
    v = (rng.random((H, S)) < p_vert).astype(np.uint8)
    tm = None
    if L:
        tm = (rng.random((H, L, L)) < 0.4).astype(np.uint8) * np.tril(np.ones((L, L), np.uint8))
    return oracle.from_patterns(d, v, tm)


def brute(Q, K, V, art, scale=None):
    """Dense logits, -inf fill from the dense mask, softmax, matmul; fp64 numpy."""
    Hq, S, d = Q.shape
    G = Hq // K.shape[0]
    sc = scale if scale else 1.0 / np.sqrt(d)
    O = np.zeros((Hq, S, d))
    lse = np.full((Hq, S), -np.inf)
    for h in range(Hq):
        M = oracle.rows(art, h, S, 0, S).astype(bool)
        s = (Q[h].astype(np.float64) @ K[h // G].astype(np.float64).T) * sc
        s = np.where(M, s, -np.inf)
        for i in range(S):
            if not M[i].any():
                continue
            mx = s[i].max()
            e = np.exp(s[i] - mx)
            O[h, i] = (e / e.sum()) @ V[h // G].astype(np.float64)
            lse[h, i] = mx + np.log(e.sum())
    return O, lse


def test_all_ones_mask_is_dense_causal_attention():
    rng = np.random.default_rng(10)
    Hq, Hkv, S, d = 4, 2, 65, 16
    Q, K, V = rand_qkv(rng, Hq, Hkv, S, d)
    art = oracle.from_patterns(np.ones((Hq, S), np.uint8), np.zeros((Hq, S), np.uint8))
    O, lse = oracle.attend_prefill(Q, K, V, art)
    tq = torch.from_numpy(Q).double()[None]
    tk = torch.from_numpy(K).double().repeat_interleave(Hq // Hkv, 0)[None]
    tv = torch.from_numpy(V).double().repeat_interleave(Hq // Hkv, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].numpy()
    np.testing.assert_allclose(O, ref, atol=1e-12)
    s = torch.einsum("hid,hjd->hij", tq[0], tk[0]) / np.sqrt(d)
    s = s.masked_fill(~torch.tril(torch.ones(S, S, dtype=torch.bool)), float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), atol=1e-12)


def test_brute_force_random_masks_gqa_and_scale():
    rng = np.random.default_rng(11)
    Hq, Hkv, S, d = 6, 2, 50, 8
    Q, K, V = rand_qkv(rng, Hq, Hkv, S, d, scale=2.0)
    art = random_art(rng, Hq, S, L=12)
    for scale in (None, 0.37):
        O, lse = oracle.attend_prefill(Q, K, V, art, scale)
        Ob, lb = brute(Q, K, V, art, scale)
        np.testing.assert_allclose(O, Ob, atol=1e-12)
        np.testing.assert_allclose(lse, lb, atol=1e-12)
    # GQA equals multi-head attention with the K/V heads repeated
    O2, _ = oracle.attend_prefill(Q, np.repeat(K, 3, 0), np.repeat(V, 3, 0), art)
    O1, _ = oracle.attend_prefill(Q, K, V, art)
    assert np.array_equal(O1, O2)
    # ... and the grouping is contiguous: head h reads KV head h // G (a transposed grouping fails)
    Kp = K.copy()
    Kp[1] += 1.0
    O3, _ = oracle.attend_prefill(Q, Kp, V, art)
    assert np.array_equal(O3[:3], O1[:3]) and not np.allclose(O3[3:], O1[3:])


def test_empty_rows_single_key_and_convexity():
    rng = np.random.default_rng(12)
    Hq, S, d = 2, 40, 8
    Q, K, V = rand_qkv(rng, Hq, Hq, S, d, scale=3.0)
    # head 0: only the diagonal r = 3  -> rows 0..2 empty, rows >= 3 keep exactly key i-3
    # head 1: random
    dg = np.zeros((Hq, S), np.uint8)
    vt = np.zeros((Hq, S), np.uint8)
    dg[0, 3] = 1
    dg[1] = rng.random(S) < 0.3
    art = oracle.from_patterns(dg, vt)
    O, lse = oracle.attend_prefill(Q, K, V, art)
    assert np.all(O[0, :3] == 0) and np.all(np.isneginf(lse[0, :3])) and not np.isnan(O).any()
    assert np.array_equal(O[0, 3:], V[0, :S - 3].astype(np.float64))      # that V row exactly
    np.testing.assert_allclose(lse[0, 3:], np.einsum("id,id->i", Q[0, 3:].astype(np.float64),
                                                     K[0, :S - 3].astype(np.float64)) / np.sqrt(d), atol=1e-12)
    for i in range(S):
        kept = oracle.kept_list(art, 1, i)
        if len(kept) == 0:
            assert np.all(O[1, i] == 0)
            continue
        lo, hi = V[1, kept].min(0), V[1, kept].max(0)
        assert np.all(O[1, i] >= lo - 1e-12) and np.all(O[1, i] <= hi + 1e-12)


def test_list_form_identities():
    rng = np.random.default_rng(13)
    d, T = 16, 300
    q = rng.standard_normal((1, d)).astype(np.float32) * 2
    Kc = rng.standard_normal((1, T, d)).astype(np.float32)
    Vc = rng.standard_normal((1, T, d)).astype(np.float32)
    idx = np.sort(rng.choice(T, 70, replace=False)).astype(np.int32)
    O, lse = oracle.attend_lists(q, Kc, Vc, [0], [0, 70], idx)
    # permuting the kept keys changes nothing but rounding
    perm = rng.permutation(70)
    Op, lp = oracle.attend_lists(q, Kc, Vc, [0], [0, 70], idx[perm])
    np.testing.assert_allclose(Op, O, atol=1e-13)
    # adding a constant to every logit (append a constant feature) changes nothing but lse
    q2 = np.concatenate([q, np.full((1, 1), 4.0, np.float32)], 1)
    K2 = np.concatenate([Kc, np.full((1, T, 1), 0.5, np.float32)], 2)
    V2 = np.concatenate([Vc, np.zeros((1, T, 1), np.float32)], 2)
    sc = 1.0 / np.sqrt(d)
    O2, l2 = oracle.attend_lists(q2, K2, V2, [0], [0, 70], idx, scale=sc)
    np.testing.assert_allclose(O2[:, :d], O, atol=1e-12)
    np.testing.assert_allclose(l2 - lse, 2.0 * sc, atol=1e-12)
    # split the list in two and merge by log-sum-exp
    Oa, la = oracle.attend_lists(q, Kc, Vc, [0], [0, 30], idx[:30])
    Ob, lb = oracle.attend_lists(q, Kc, Vc, [0], [0, 40], idx[30:])
    m = np.maximum(la, lb)
    wa, wb = np.exp(la - m), np.exp(lb - m)
    np.testing.assert_allclose((wa * Oa + wb * Ob) / (wa + wb), O, atol=1e-12)
    np.testing.assert_allclose(m + np.log(wa + wb), lse, atol=1e-12)
    # several items, different cache blocks, one empty list
    q3 = rng.standard_normal((3, d)).astype(np.float32)
    K3 = rng.standard_normal((2, T, d)).astype(np.float32)
    V3 = rng.standard_normal((2, T, d)).astype(np.float32)
    O3, l3 = oracle.attend_lists(q3, K3, V3, [1, 0, 1], [0, 5, 5, 9], np.array([1, 2, 3, 4, 5, 7, 8, 9, 10], np.int32))
    assert np.all(O3[1] == 0) and np.isneginf(l3[1])
    s = (K3[1, [1, 2, 3, 4, 5]].astype(np.float64) @ q3[0].astype(np.float64)) / np.sqrt(d)
    w = np.exp(s - s.max())
    np.testing.assert_allclose(O3[0], (w / w.sum()) @ V3[1, [1, 2, 3, 4, 5]].astype(np.float64), atol=1e-12)


def test_decode_row_equals_prefill_row():
    rng = np.random.default_rng(14)
    Hq, Hkv, S, d = 4, 2, 90, 8
    Q, K, V = rand_qkv(rng, Hq, Hkv, S, d)
    art = random_art(rng, Hq, S, L=20)
    O, lse = oracle.attend_prefill(Q, K, V, art)
    p = S - 1
    lists = [oracle.kept_list(art, h, p) for h in range(Hq)]
    ptr = np.concatenate([[0], np.cumsum([len(x) for x in lists])])
    Od, ld = oracle.attend_lists(Q[:, p], K, V, [h // 2 for h in range(Hq)], ptr, np.concatenate(lists))
    np.testing.assert_allclose(Od, O[:, p], atol=1e-13)
    np.testing.assert_allclose(ld, lse[:, p], atol=1e-13)


# ---------------------------------------------------------------------------------------------
# kept lists merged per KV head (grouped-query decode)
def test_group_lists_worked_example():
    # two KV heads of two query heads each, written out by hand
    lists = [np.array([0, 1, 5, 9], np.int32), np.array([1, 2, 9], np.int32),
             np.array([], np.int32), np.array([3, 4], np.int32)]
    ptr, idx, member = oracle.group_lists(lists, 2)
    assert ptr.tolist() == [0, 5, 7]
    # KV head 0: kept by both {1, 9}; by head 0 alone {0, 5}; by head 1 alone {2}. KV head 1: head 1 alone.
    assert idx.tolist() == [1, 9, 0, 5, 2, 3, 4]
    assert member.tolist() == [3, 3, 1, 1, 2, 2, 2]


def test_group_lists_expand_back_to_the_lists_of_the_heads():
    rng = np.random.default_rng(7)
    for group in (1, 2, 3, 4, 8):
        n_kv = 3
        lists = [np.sort(rng.choice(300, size=int(rng.integers(0, 120)), replace=False)).astype(np.int32)
                 for _ in range(n_kv * group)]
        lists[1 % len(lists)] = lists[0].copy()  # two heads with the same list
        ptr, idx, member = oracle.group_lists(lists, group)
        for kv in range(n_kv):
            seg, mem = idx[ptr[kv]:ptr[kv + 1]], member[ptr[kv]:ptr[kv + 1]]
            assert len(np.unique(seg)) == len(seg)  # every key once
            assert (mem != 0).all() and (mem >> group == 0).all()
            for x in range(group):
                assert np.array_equal(np.sort(seg[(mem >> x) & 1 == 1]), lists[kv * group + x])
            # the runs: shared keys first, then one run per head, each ascending
            n_heads = np.array([bin(int(m)).count("1") for m in mem])
            run = np.where(n_heads >= 2, 0, 1 + np.log2(np.maximum(mem, 1)).astype(int))
            assert (np.diff(run) >= 0).all()
            for r in range(group + 1):
                assert (np.diff(seg[run == r]) > 0).all()


# ---------------------------------------------------------------------------------------------
# Position-independent decode plans (oracle.pattern_plan): pinned by expanding them back into the rows of the
# mask they stand for (Sec. 4.3), which the plain kept_list defines, and by a hand-worked example.
def test_pattern_plan_worked_example():
    P = 12
    d = np.zeros((2, P), np.uint8)
    v = np.zeros((2, P), np.uint8)
    d[0, [0, 1, 5]] = 1          # head 0: diagonals 0, 1, 5
    d[1, [0, 2]] = 1             # head 1: diagonals 0, 2
    v[0, [0, 7]] = 1             # head 0: columns 0, 7
    v[1, [0, 3]] = 1             # head 1: columns 0, 3
    ptr, val, mem, table = oracle.pattern_plan(d, v, 2)
    # diagonals: shared {0}; head 0 alone {1, 5}; head 1 alone {2}. columns: shared {0}; head 0 alone {7}; head 1 alone {3}
    assert list(ptr) == [0, 7]
    assert list(val) == [-1, -6, -2, -3, 0, 7, 3]          # (head 0's own diagonals 5, 1: descending offsets)
    assert list(mem) == [3, 1, 1, 2, 3, 1, 2]
    assert list(table[0]) == [3, 1, 2, 0, 0, 1, 0, 0, 0, 0, 0, 0]
    plan = (ptr, val, mem, table)
    # position 8: head 0 keeps 8, 7 (diagonals 0, 1), 3 (diagonal 5), columns 0 and 7 (7 is also its diagonal 1: once)
    assert list(oracle.plan_row(plan, 0, 0, 8)) == [0, 3, 7, 8]
    # head 1 keeps 8, 6 (diagonals 0, 2), columns 0 and 3
    assert list(oracle.plan_row(plan, 0, 1, 8)) == [0, 3, 6, 8]
    # position 1: diagonal 5 and column 7 do not exist yet; head 1's diagonal 2 neither
    assert list(oracle.plan_row(plan, 0, 0, 1)) == [0, 1]
    assert list(oracle.plan_row(plan, 0, 1, 1)) == [0, 1]


@pytest.mark.parametrize("seed,G", [(1, 1), (2, 2), (3, 4), (4, 8)])
def test_pattern_plan_expands_to_the_rows_of_the_mask(seed, G):
    rng = np.random.default_rng(seed)
    Hq, P = 2 * G, 300
    d = (rng.random((Hq, P)) < 0.1).astype(np.uint8)
    v = (rng.random((Hq, P)) < 0.1).astype(np.uint8)
    d[:, :5] = 1                                   # a window every head has: many keys that are column and diagonal at once
    v[:, :3] = 1
    if Hq > 2:
        d[2], v[2] = 0, 0                          # a head that keeps nothing
    art = oracle.from_patterns(d, v)
    plan = oracle.pattern_plan(d, v, G)
    ptr, val, mem, table = plan
    for g in range(Hq // G):
        seg = slice(int(ptr[g]), int(ptr[g + 1]))
        assert len(set(val[seg].tolist())) == ptr[g + 1] - ptr[g]            # every pattern once
        assert (mem[seg] != 0).all() and (mem[seg] < (1 << G)).all()
    for p in (0, 1, 4, 63, 64, 150, P - 1, P + 40, 2 * P + 7):
        S = max(P, p + 1)
        big = oracle.from_patterns(np.pad(d, ((0, 0), (0, S - P))), np.pad(v, ((0, 0), (0, S - P))))
        for h in range(Hq):
            want = oracle.kept_list(big, h, p)
            got = oracle.plan_row(plan, h // G, h % G, p)
            assert np.array_equal(got, want), (h, p)
    # columns at or beyond the problem length are left out of a plan built for it
    short = oracle.pattern_plan(d, v, G, S=100)
    assert (short[1][short[1] >= 0] < 100).all() and np.array_equal(short[3], table)
    del art
