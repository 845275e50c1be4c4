"""KV eviction on the GPU (dam_kv_evict_plan, dam_kv_compact, dam_kv_remap_lists) against the oracle:
plan and slots bit for bit, compacted rows byte for byte, and decode from the compacted cache equal
to decode from the full cache (same rows, same order of accumulation: identical bits)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_11104_amd import binding as B
from paper_2506_11104_amd import workloads as wl

pytestmark = pytest.mark.gpu


def flags(seed, Hq, P, wide=False):
    rng = np.random.default_rng(seed)
    d = np.zeros((Hq, P), np.uint8)
    v = np.zeros((Hq, P), np.uint8)
    for h in range(Hq):
        d[h, :int(rng.integers(1, 200 if wide else 30))] = 1
        if rng.random() < 0.5:
            a = int(rng.integers(200, 300))
            d[h, a:a + int(rng.integers(1, 20))] = 1
        v[h, :int(rng.integers(1, 9))] = 1
        v[h, rng.choice(P, size=12, replace=False)] = 1
    return d, v


def check_plan(plan, want):
    assert np.array_equal(plan.window.cpu().numpy(), want.window)
    assert np.array_equal(plan.col_ptr.cpu().numpy(), want.col_ptr)
    assert plan.n_cols == len(want.cols)
    assert np.array_equal(plan.cols.cpu().numpy()[:plan.n_cols], want.cols)
    assert np.array_equal(plan.rows.cpu().numpy(), want.window + np.diff(want.col_ptr))


@pytest.mark.parametrize("Hq,Hkv,P,pos", [(8, 2, 1000, 700), (4, 4, 333, 332), (6, 3, 2000, 5), (2, 1, 64, 63)])
def test_plan_matches_oracle(Hq, Hkv, P, pos):
    d, v = flags(3, Hq, P, wide=True)
    if Hq == 4:
        d[1] = 0                                    # a KV head without any diagonal
        v[2] = 0                                    # and one without columns
    plan = B.kv_evict_plan(torch.from_numpy(d).cuda(), torch.from_numpy(v).cuda(), Hkv, pos)
    torch.cuda.synchronize()
    check_plan(plan, oracle.eviction_plan(d, v, Hkv, pos))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_compact_remap_and_decode_are_identical_to_the_full_cache(dtype):
    Bn, Hq, Hkv, d_head, T, steps = 3, 8, 2, 128, 3000, 3
    cap = T + steps
    d, v = flags(4, Hq, cap, wide=True)
    art = oracle.from_patterns(d, v)
    g = torch.Generator().manual_seed(5)
    kc = torch.randn((Bn, Hkv, cap, d_head), generator=g).to(dtype).cuda()
    vc = torch.randn((Bn, Hkv, cap, d_head), generator=g).to(dtype).cuda()
    qs = torch.randn((steps, Bn, Hq, d_head), generator=g).to(dtype).cuda()
    d_dev, v_dev = torch.from_numpy(d).cuda(), torch.from_numpy(v).cuda()
    G = Hq // Hkv
    pos = T - 1
    plan = B.kv_evict_plan(d_dev, v_dev, Hkv, pos, batch=Bn)
    torch.cuda.synchronize()
    want = oracle.eviction_plan(d, v, Hkv, pos)
    check_plan(plan, want)
    ccap = int(plan.rows.max().item())
    assert ccap < cap // 4                                             # the point of the exercise
    kcmp = torch.full((Bn, Hkv, ccap, d_head), 7.0, dtype=dtype, device="cuda")
    vcmp = torch.full((Bn, Hkv, ccap, d_head), 7.0, dtype=dtype, device="cuda")
    B.kv_compact(plan, kc, vc, kcmp, vcmp)
    torch.cuda.synchronize()
    for gk in range(Hkv):
        W, ncol = int(want.window[gk]), int(want.col_ptr[gk + 1] - want.col_ptr[gk])
        live = sorted(set(int(c) for c in want.cols[want.col_ptr[gk]:want.col_ptr[gk + 1]]) | set(range(max(0, pos - W + 1), pos + 1)))
        slots = torch.tensor([oracle.eviction_slot(want, gk, j) for j in live], device="cuda")
        keys = torch.tensor(live, device="cuda")
        assert torch.equal(kcmp[:, gk, slots], kc[:, gk, keys]) and torch.equal(vcmp[:, gk, slots], vc[:, gk, keys])
        assert (kcmp[:, gk, ncol + W:] == 7.0).all()                   # rows past the head's need are untouched
    for step in range(steps):
        p = pos + step
        if step > 0:
            # the new key's K / V rows go to its ring slot (the caller's append), and nothing else moves
            for gk in range(Hkv):
                s = oracle.eviction_slot(want, gk, p)
                kcmp[:, gk, s] = kc[:, gk, p]
                vcmp[:, gk, s] = vc[:, gk, p]
        lists = [oracle.kept_list(art, h, p) for h in range(Hq)]
        lens = np.array([len(x) for x in lists])
        ptr = torch.from_numpy(np.concatenate([[0], np.cumsum(np.tile(lens, Bn))]).astype(np.int32)).cuda()
        idx = torch.from_numpy(np.tile(np.concatenate(lists), Bn).astype(np.int32)).cuda()
        plan.params.pos = p
        slot = B.kv_remap_lists(plan, ptr, idx, Bn)
        torch.cuda.synchronize()
        want_slot = np.tile(np.concatenate([[oracle.eviction_slot(want, h // G, int(j)) for j in lists[h]] for h in range(Hq)]), Bn)
        assert np.array_equal(slot.cpu().numpy(), want_slot)
        full, lse_f = B.dam_sparse_attn_decode(qs[step], kc, vc, ptr, idx, int(lens.max()), want_lse=True)
        comp, lse_c = B.dam_sparse_attn_decode(qs[step], kcmp, vcmp, ptr, slot, int(lens.max()), want_lse=True)
        torch.cuda.synchronize()
        assert torch.equal(full, comp) and torch.equal(lse_f, lse_c), f"position {p}"


def test_c5_plan_at_full_size():
    w = wl.WORKLOADS["c5"]
    d, v = wl.patterns_c5(w)
    pos = w.seq - 1
    plan = B.kv_evict_plan(torch.from_numpy(d).cuda(), torch.from_numpy(v).cuda(), w.hkv, pos, batch=w.batch)
    torch.cuda.synchronize()
    check_plan(plan, oracle.eviction_plan(d, v, w.hkv, pos))
    assert int(plan.rows.max().item()) < w.seq // 4


def test_grouped_decode_from_the_compacted_cache_is_identical_to_the_full_cache():
    """Merged lists per KV head (dam_mask_build with DAM_MASK_GROUP_LISTS), remapped into the compacted cache
    with the lists taken per KV head: the grouped decode gives the same bits from either cache, and the oracle's
    attention over each head's own list within the bf16 bar."""
    Bn, Hq, Hkv, d_head, T = 2, 8, 2, 128, 3000
    cap = T + 1
    G = Hq // Hkv
    d, v = flags(6, Hq, cap, wide=True)
    art = oracle.from_patterns(d, v)
    g = torch.Generator().manual_seed(7)
    kc = torch.randn((Bn, Hkv, cap, d_head), generator=g).to(torch.bfloat16).cuda()
    vc = torch.randn((Bn, Hkv, cap, d_head), generator=g).to(torch.bfloat16).cuda()
    q = torch.randn((Bn, Hq, d_head), generator=g).to(torch.bfloat16).cuda()
    d_dev, v_dev = torch.from_numpy(d).cuda(), torch.from_numpy(v).cuda()
    pos = T - 1
    plan = B.kv_evict_plan(d_dev, v_dev, Hkv, pos, batch=Bn)
    ccap = int(plan.rows.max().item())
    kcmp = torch.zeros((Bn, Hkv, ccap, d_head), dtype=torch.bfloat16, device="cuda")
    vcmp = torch.zeros_like(kcmp)
    B.kv_compact(plan, kc, vc, kcmp, vcmp)
    m = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=Hq, L=0, S=cap, diag_in=d_dev, vert_in=v_dev, blocks=False,
                     rows=(pos, pos + 1), group=G)
    slot = B.kv_remap_lists(plan, m.kept_ptr, m.kept_idx, 1, per_kv_head=True)
    torch.cuda.synchronize()
    want = oracle.eviction_plan(d, v, Hkv, pos)
    ptr = m.kept_ptr.cpu().numpy()
    idx = m.kept_idx.cpu().numpy()
    want_slot = np.concatenate([[oracle.eviction_slot(want, gk, int(j)) for j in idx[ptr[gk]:ptr[gk + 1]]] for gk in range(Hkv)])
    assert np.array_equal(slot.cpu().numpy(), want_slot)
    longest = int(np.diff(ptr).max())
    full, lse_f = B.dam_sparse_attn_decode_grouped(q, kc, vc, m.kept_ptr, m.kept_idx, m.kept_member, longest, want_lse=True,
                                                   shared_lists=True)
    comp, lse_c = B.dam_sparse_attn_decode_grouped(q, kcmp, vcmp, m.kept_ptr, slot, m.kept_member, longest, want_lse=True,
                                                   shared_lists=True)
    torch.cuda.synchronize()
    assert torch.equal(full, comp) and torch.equal(lse_f, lse_c)
    lists = [oracle.kept_list(art, h, pos) for h in range(Hq)]
    lens = np.array([len(x) for x in lists])
    kv_of = np.array([b * Hkv + h // G for b in range(Bn) for h in range(Hq)], np.int32)
    O, _ = oracle.attend_lists(q.float().cpu().numpy().reshape(Bn * Hq, d_head), kc.float().cpu().numpy().reshape(Bn * Hkv, cap, d_head),
                               vc.float().cpu().numpy().reshape(Bn * Hkv, cap, d_head), kv_of,
                               np.concatenate([[0], np.cumsum(np.tile(lens, Bn))]).astype(np.int64),
                               np.tile(np.concatenate(lists), Bn).astype(np.int32))
    assert np.abs(comp.float().cpu().numpy().reshape(Bn * Hq, d_head) - O).max() <= 2e-2


def test_compaction_into_an_interleaved_cache():
    """The compacted caches may share one buffer with the K and V row of a key side by side ([rows][2][d]): the
    entry points take the two pointers and one set of strides. Rows are byte for byte those of the separate
    layout, and decode from it gives the same bits."""
    Bn, Hq, Hkv, d_head, T = 2, 4, 2, 128, 2000
    d, v = flags(8, Hq, T, wide=True)
    g = torch.Generator().manual_seed(10)
    kc = torch.randn((Bn, Hkv, T, d_head), generator=g).to(torch.bfloat16).cuda()
    vc = torch.randn((Bn, Hkv, T, d_head), generator=g).to(torch.bfloat16).cuda()
    q = torch.randn((Bn, Hq, d_head), generator=g).to(torch.bfloat16).cuda()
    d_dev, v_dev = torch.from_numpy(d).cuda(), torch.from_numpy(v).cuda()
    pos = T - 1
    plan = B.kv_evict_plan(d_dev, v_dev, Hkv, pos, batch=Bn)
    ccap = int(plan.rows.max().item())
    k_sep = torch.zeros((Bn, Hkv, ccap, d_head), dtype=torch.bfloat16, device="cuda")
    v_sep = torch.zeros_like(k_sep)
    B.kv_compact(plan, kc, vc, k_sep, v_sep)
    both = torch.zeros((Bn, Hkv, ccap, 2, d_head), dtype=torch.bfloat16, device="cuda")
    k_il, v_il = both[:, :, :, 0], both[:, :, :, 1]
    B.kv_compact(plan, kc, vc, k_il, v_il)
    torch.cuda.synchronize()
    assert torch.equal(k_il, k_sep) and torch.equal(v_il, v_sep)
    m = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=Hq, L=0, S=T, diag_in=d_dev, vert_in=v_dev, blocks=False, rows=(pos, pos + 1))
    slot = B.kv_remap_lists(plan, m.kept_ptr, m.kept_idx, 1)
    longest = int((m.kept_ptr[1:] - m.kept_ptr[:-1]).max().item())
    a = B.dam_sparse_attn_decode(q, k_sep, v_sep, m.kept_ptr, slot, longest, shared_lists=True)
    b = B.dam_sparse_attn_decode(q, k_il, v_il, m.kept_ptr, slot, longest, shared_lists=True)
    c = B.dam_sparse_attn_decode(q, kc, vc, m.kept_ptr, m.kept_idx, longest, shared_lists=True)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(a, c)
