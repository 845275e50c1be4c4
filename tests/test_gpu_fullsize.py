"""The largest configurations at full size, in the launch shapes bench.py uses: c3 (32k prefill,
masks from patterns), c4 (128k prefill, masks from a 4096 x 4096 capture map) and c5 (decode at
64k, batch 16). What the oracle cannot recompute whole within a test's time is checked on seeded
samples it computes one by one: query-tile rows of the block index for every head, (head, row)
pairs of the attention output for every head, plus the ragged ends. c3's outputs are compared row
by row in full in test_gpu_prefill.py; c4's block index is compared in full for every head, its
outputs on every row of two heads and 2048 seeded rows of each head.

Progress lines are printed with pytest's capture switched off: the c4 case is quiet for a while."""
import sys
import time

import numpy as np
import pytest
import torch

import oracle
from dam_testlib import dev, pack_rows_u64, u64
from paper_2506_11104_amd import binding as B
from paper_2506_11104_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2
WORKERS = 16
T0 = time.time()


_CAPSYS = None


@pytest.fixture(autouse=True)
def _progress_output(capsys):
    global _CAPSYS
    _CAPSYS = capsys
    yield
    _CAPSYS = None


def say(msg):
    with _CAPSYS.disabled():
        print(f"[fullsize {time.time() - T0:6.1f}s] {msg}", file=sys.stderr, flush=True)


def check_heads_in_full(art, mask, S, heads):
    g_ptr = mask.blk_row_ptr.cpu().numpy().astype(np.int64)
    for h in heads:
        rp, c, k, bits = oracle.block_index(art, S, 128, 128, heads=[h], workers=WORKERS)
        a, b = g_ptr[h, 0], g_ptr[h, -1]
        assert np.array_equal(g_ptr[h] - a, rp[0]), f"blk_row_ptr head {h}"
        assert np.array_equal(mask.blk_col[a:b].cpu().numpy(), c), f"blk_col head {h}"
        assert np.array_equal(mask.blk_kind[a:b].cpu().numpy(), k), f"blk_kind head {h}"
        assert np.array_equal(u64(mask.tile_bits[a:b]), bits), f"tile_bits head {h}"
        if h % 8 == 7:
            say(f"heads up to {h}: identical ({b - a} tiles in head {h})")


def check_rows(Q, K, V, art, out, lse, hs, rs):
    O, LSE = oracle.attend_rows(Q[hs, rs], K, V, art, Q.shape[0], hs, rs)
    hs_t, rs_t = torch.from_numpy(hs.astype(np.int64)).cuda(), torch.from_numpy(rs).cuda()
    got = out[0][hs_t, rs_t].float().cpu().numpy()
    got_lse = lse[0][hs_t, rs_t].cpu().numpy()
    assert not np.isnan(got).any()
    fin = np.isfinite(LSE)
    assert np.array_equal(np.isneginf(got_lse), ~fin)
    err = np.abs(got - O).max()
    assert err <= TOL_BF16, f"max abs err {err}"
    if fin.any():
        assert np.abs(got_lse[fin] - LSE[fin]).max() <= TOL_BF16
    assert (got[~fin] == 0).all()
    return err


def test_c3_mask_whole_block_index_bit_exact():
    """Every tile of every head of the 32k pattern masks: row pointers, columns, kinds, bits."""
    w = wl.WORKLOADS["c3"]
    dflag, vflag = wl.patterns_c3(w)
    art = oracle.from_patterns(dflag, vflag)
    mask = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=w.hq, L=0, S=w.seq, diag_in=torch.from_numpy(dflag).cuda(),
                        vert_in=torch.from_numpy(vflag).cuda())
    torch.cuda.synchronize()
    say(f"c3: {mask.n_tiles} tiles listed")
    row_ptr, col, kind, bits = oracle.block_index(art, w.seq, 128, 128, workers=WORKERS)
    assert np.array_equal(mask.blk_row_ptr.cpu().numpy().astype(np.int64), row_ptr)
    assert np.array_equal(mask.blk_col.cpu().numpy(), col)
    assert np.array_equal(mask.blk_kind.cpu().numpy(), kind)
    assert np.array_equal(u64(mask.tile_bits), bits)
    # the build bench.py times (full tiles carry no bits): everything else identical
    lean = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=w.hq, L=0, S=w.seq, diag_in=torch.from_numpy(dflag).cuda(),
                        vert_in=torch.from_numpy(vflag).cuda(), flags=B.DAM_MASK_SKIP_FULL_TILE_BITS)
    torch.cuda.synchronize()
    partial = (kind & 1) == 0
    assert np.array_equal(lean.blk_row_ptr.cpu().numpy().astype(np.int64), row_ptr)
    assert np.array_equal(lean.blk_col.cpu().numpy(), col) and np.array_equal(lean.blk_kind.cpu().numpy(), kind)
    assert np.array_equal(u64(lean.tile_bits)[partial], bits[partial])
    assert (bits[~partial] == np.uint64(0xFFFFFFFFFFFFFFFF)).all()
    say(f"c3: {int(partial.sum())} partial tiles identical without the bits of the {int((~partial).sum())} full tiles")
    # ... and with the matched columns gathered into tiles of their own, the layout the benchmark step uses
    del mask, lean, bits
    gath = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=w.hq, L=0, S=w.seq, diag_in=torch.from_numpy(dflag).cuda(),
                        vert_in=torch.from_numpy(vflag).cuda(),
                        flags=B.DAM_MASK_SKIP_FULL_TILE_BITS | B.DAM_MASK_GATHER_COLUMNS)
    torch.cuda.synchronize()
    row_ptr, col, kind, bits = oracle.block_index(art, w.seq, 128, 128, workers=WORKERS, gather=True)
    gptr, gidx = oracle.gathered_columns(art, w.seq, 128)
    got_idx, got_cnt = gath.gather_idx.cpu().numpy(), gath.gather_cnt.cpu().numpy()
    for h in range(w.hq):
        seg = gidx[gptr[h]:gptr[h + 1]]
        assert got_cnt[h] == int((seg >= 0).sum()) and np.array_equal(got_idx[h, :len(seg)], seg)
        assert (got_idx[h, len(seg):] == -1).all()
    partial = (kind & 1) == 0
    assert np.array_equal(gath.blk_row_ptr.cpu().numpy().astype(np.int64), row_ptr)
    assert np.array_equal(gath.blk_col.cpu().numpy(), col) and np.array_equal(gath.blk_kind.cpu().numpy(), kind)
    assert np.array_equal(u64(gath.tile_bits)[partial], bits[partial])
    say(f"c3: gathered layout: {len(col)} tiles ({int((col >= w.seq // 128).sum())} of them gathered) identical")


def test_c4_full_size():
    w = wl.WORKLOADS["c4"]
    S, L, H = w.seq, w.pcl, w.hq
    say("c4: generating Q, K, V (about 5 GiB of normals)")
    Q, K, V = wl.qkv_structured(w)
    say("c4: capture map")
    A = wl.capture_map(Q[:, :L], K[:, :L], L, w.hq // w.hkv)
    say("c4: oracle stage one")
    art = oracle.derive(A, None, w.lam, w.eps, w.tau, w.mu)
    say("c4: GPU mask build")
    mask = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=H, L=L, S=S, lam=w.lam, eps=w.eps, tau=w.tau, mu=w.mu,
                        attn_sum=torch.from_numpy(A).cuda())
    torch.cuda.synchronize()
    # stage one, whole: threshold bits, match counts and flags
    assert np.float32(mask.bmin.item()) == np.float32(art.bmin)
    for h in range(H):
        assert np.array_equal(u64(mask.true_bits[h]), pack_rows_u64(art.true_mask[h])), f"true_bits head {h}"
    assert np.array_equal(mask.diag_cnt.cpu().numpy(), art.diag_cnt)
    assert np.array_equal(mask.vert_cnt.cpu().numpy(), art.vert_cnt)
    assert np.array_equal(mask.diag_flag.cpu().numpy(), art.diag_flag)
    assert np.array_equal(mask.vert_flag.cpu().numpy(), art.vert_flag)
    # density over the S x S triangle, from the block index' own bits
    nnz = 0
    for a in range(0, mask.n_tiles, 1 << 17):
        nnz += int(np.unpackbits(u64(mask.tile_bits[a:a + (1 << 17)]).view(np.uint8)).sum(dtype=np.int64))
    dens = nnz / (H * S * (S + 1) / 2)
    say(f"c4: stage one identical; {mask.n_tiles} tiles, density {dens:.4f}")
    assert 0.01 <= dens <= 0.05, dens
    # the same stage one fused with its capture (dam_mask_build_from_qk, no map): true-mask bits may
    # differ from the map-based ones only where the probability is within the fp32 tolerance of the
    # threshold; counts and flags must be exactly what the oracle derives from the GPU's own bits
    fused = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=H, L=L, S=S, lam=w.lam, eps=w.eps, tau=w.tau, mu=w.mu, blocks=False,
                         qk=(dev(np.ascontiguousarray(Q[:, :L]), "bf16"), dev(np.ascontiguousarray(K[:, :L]), "bf16")))
    torch.cuda.synchronize()
    tri = np.tril(np.ones((L, L), bool))
    theta_lo = max(float(A[h][(art.true_mask[h] == 0) & tri].max()) for h in range(H))
    theta_hi = min(float(A[h][art.true_mask[h] == 1].min()) for h in range(H))
    assert theta_lo <= theta_hi
    theta = 0.5 * (theta_lo + theta_hi)
    n_diff = n_near = 0
    f_dc, f_vc = fused.diag_cnt.cpu().numpy(), fused.vert_cnt.cpu().numpy()
    f_df, f_vf = fused.diag_flag.cpu().numpy(), fused.vert_flag.cpu().numpy()
    for h in range(H):
        got = np.ascontiguousarray(np.unpackbits(u64(fused.true_bits[h]).view(np.uint8), axis=-1, bitorder="little")[:, :L])
        diff = got != art.true_mask[h]
        near = np.abs(A[h] - theta) <= 1e-4 * theta
        assert not (diff & ~near).any(), f"fused true mask head {h}: bits differ away from the threshold"
        n_diff += int(diff.sum())
        n_near += int(near.sum())
        dc, vc, df, vf = oracle.match(got[None], w.mu)
        assert np.array_equal(f_dc[h], dc[0]) and np.array_equal(f_vc[h], vc[0]), f"fused counts head {h}"
        assert np.array_equal(f_df[h], df[0]) and np.array_equal(f_vf[h], vf[0]), f"fused flags head {h}"
    say(f"c4: fused capture: {n_diff} of {H * L * (L + 1) // 2} true-mask bits differ, all among the {n_near} entries "
        f"within tolerance of the threshold {theta:.3e}")
    assert n_diff <= 0.05 * n_near + 64
    del A, fused
    # the S-sized outputs: the block index and the tile bits of every head in full, streamed head by head (the oracle
    # regenerates a head's tiles; the whole pool is never held twice)
    check_heads_in_full(art, mask, S, range(H))
    rng = np.random.default_rng(45)
    nQt = S // 128
    say("c4: block index and tile bits of every head identical; prefill")
    q, k, v = dev(Q, "bf16")[None], dev(K, "bf16")[None], dev(V, "bf16")[None]
    out, lse = B.dam_sparse_attn_prefill(q, k, v, mask, want_lse=True)
    torch.cuda.synchronize()
    say("c4: prefill done; oracle rows")
    # every row of two heads, and 2048 seeded rows of every head (the ends and the rows around L among them)
    full_heads = [int(x) for x in rng.choice(H, 2, replace=False)]
    hs = np.concatenate([np.repeat(np.array(full_heads, np.int32), S), np.repeat(np.arange(H, dtype=np.int32), 2048)])
    rnd = rng.integers(0, S, 2048 * H).astype(np.int64)
    rnd[::2048] = S - 1
    rnd[1::2048] = 0
    rnd[2::2048] = L - 1
    rnd[3::2048] = L
    rs = np.concatenate([np.tile(np.arange(S, dtype=np.int64), 2), rnd])
    n = len(hs)
    err = check_rows(Q, K, V, art, out, lse, hs, rs)
    say(f"c4: every row of heads {full_heads} and 2048 rows of every head ({n} rows), max abs err {err:.2e}")
    # the same with the matched columns gathered into tiles of their own (the method's stripes are many here)
    n_plain = mask.n_tiles
    del mask, out, lse
    gath = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=H, L=L, S=S, lam=w.lam, eps=w.eps, tau=w.tau, mu=w.mu,
                        attn_sum=torch.from_numpy(wl.capture_map(Q[:, :L], K[:, :L], L, w.hq // w.hkv)).cuda(),
                        flags=B.DAM_MASK_GATHER_COLUMNS | B.DAM_MASK_SKIP_FULL_TILE_BITS)
    torch.cuda.synchronize()
    jobs = [(h, int(qt)) for h in range(0, H, 4) for qt in (L // 128 - 1, L // 128, nQt - 1, int(rng.integers(0, nQt)))]
    g_ptr = gath.blk_row_ptr.cpu().numpy().astype(np.int64)
    g_col, g_kind = gath.blk_col.cpu().numpy(), gath.blk_kind.cpu().numpy()
    for h, qt in jobs:
        rp, c, k_, bits = oracle.block_index(art, S, 128, 128, heads=[h], qt_range=(qt, qt + 1), workers=1, gather=True)
        a, b = g_ptr[h, qt], g_ptr[h, qt + 1]
        assert b - a == rp[0, 1] and np.array_equal(g_col[a:b], c) and np.array_equal(g_kind[a:b], k_), (h, qt)
        part = (k_ & 1) == 0
        assert np.array_equal(u64(gath.tile_bits[a:b])[part], bits[part]), (h, qt)
    out, lse = B.dam_sparse_attn_prefill(q, k, v, gath, want_lse=True)
    torch.cuda.synchronize()
    err = check_rows(Q, K, V, art, out, lse, hs, rs)
    say(f"c4: gathered layout: {gath.n_tiles} tiles instead of {n_plain}, sampled tile rows identical, "
        f"{n} sampled rows, max abs err {err:.2e}")


def test_c5_full_size_lists_and_decode():
    """Every position of the 64k decode workload (256 consecutive ones): the kept lists built on the GPU equal
    the oracle's rows of the mask, and the decode outputs of every (sequence, head) match, from the lists
    per head, from the merged lists and from the position-independent plan."""
    w = wl.WORKLOADS["c5"]   # all of its 256 steps
    cap = w.seq + w.steps
    dflag, vflag = wl.patterns_c5(w)
    art = oracle.from_patterns(dflag, vflag)
    say("c5: generating caches")
    qs, kc, vc = wl.decode_inputs(w)
    Kf = kc.float().numpy().reshape(w.batch * w.hkv, cap, w.head_dim)
    Vf = vc.float().numpy().reshape(w.batch * w.hkv, cap, w.head_dim)
    kc_d, vc_d = kc.cuda(), vc.cuda()
    G = w.hq // w.hkv
    kv_of = np.array([b * w.hkv + h // G for b in range(w.batch) for h in range(w.hq)], np.int32)
    d_in, v_in = torch.from_numpy(dflag).cuda(), torch.from_numpy(vflag).cuda()
    # the position-independent plan, built once (the form the bench times as a whole decode step)
    plan = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=w.hq, L=0, S=cap, diag_in=d_in, vert_in=v_in, blocks=False, group=G,
                        plan=True)
    torch.cuda.synchronize()
    want_plan = oracle.pattern_plan(dflag, vflag, G, S=cap)
    assert np.array_equal(plan.kept_ptr.cpu().numpy().astype(np.int64), want_plan[0])
    assert np.array_equal(plan.kept_idx.cpu().numpy(), want_plan[1]) and np.array_equal(plan.kept_member.cpu().numpy(), want_plan[2])
    assert np.array_equal(plan.plan_table.cpu().numpy(), want_plan[3])
    plan_longest = int(np.diff(want_plan[0]).max())
    worst = 0.0
    for step in range(w.steps):
        p = w.seq - 1 + step
        mask = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=w.hq, L=0, S=cap, diag_in=d_in, vert_in=v_in, blocks=False,
                            rows=(p, p + 1))
        torch.cuda.synchronize()
        ptr = mask.kept_ptr.cpu().numpy().astype(np.int64)
        idx = mask.kept_idx.cpu().numpy()
        lists = [oracle.kept_list(art, h, p) for h in range(w.hq)]
        for h in range(w.hq):
            assert np.array_equal(idx[ptr[h]:ptr[h + 1]], lists[h]), f"kept list head {h} position {p}"
        # the same per-head lists serve every sequence of the batch
        lens = np.array([len(x) for x in lists])
        ptr_all = np.concatenate([[0], np.cumsum(np.tile(lens, w.batch))]).astype(np.int64)
        idx_all = np.tile(np.concatenate(lists), w.batch).astype(np.int32)
        qf = qs[step].float().numpy().reshape(w.batch * w.hq, w.head_dim)
        O, LSE = oracle.attend_lists(qf, Kf, Vf, kv_of, ptr_all, idx_all)
        out, lse = B.dam_sparse_attn_decode(qs[step].cuda(), kc_d, vc_d, torch.from_numpy(ptr_all.astype(np.int32)).cuda(),
                                            torch.from_numpy(idx_all).cuda(), int(lens.max()), want_lse=True)
        torch.cuda.synchronize()
        got = out.float().cpu().numpy().reshape(w.batch * w.hq, w.head_dim)
        assert not np.isnan(got).any()
        err = np.abs(got - O).max()
        assert err <= TOL_BF16, f"position {p}: max abs err {err}"
        assert np.abs(lse.cpu().numpy().reshape(-1) - LSE).max() <= TOL_BF16
        # the grouped-query form in the launch configuration the bench times: merged lists per KV head, shared by the batch
        mg = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=w.hq, L=0, S=cap, diag_in=d_in, vert_in=v_in, blocks=False,
                          rows=(p, p + 1), group=G)
        torch.cuda.synchronize()
        want = oracle.group_lists(lists, G)
        assert np.array_equal(mg.kept_ptr.cpu().numpy().astype(np.int64), want[0])
        assert np.array_equal(mg.kept_idx.cpu().numpy(), want[1]) and np.array_equal(mg.kept_member.cpu().numpy(), want[2])
        out_g, lse_g = B.dam_sparse_attn_decode_grouped(qs[step].cuda(), kc_d, vc_d, mg.kept_ptr, mg.kept_idx, mg.kept_member,
                                                        int(np.diff(want[0]).max()), want_lse=True, shared_lists=True)
        torch.cuda.synchronize()
        err_g = np.abs(out_g.float().cpu().numpy().reshape(w.batch * w.hq, w.head_dim) - O).max()
        assert err_g <= TOL_BF16, f"position {p}, grouped: max abs err {err_g}"
        assert np.abs(lse_g.cpu().numpy().reshape(-1) - LSE).max() <= TOL_BF16
        out_p, lse_p = B.dam_sparse_attn_decode_patterns(qs[step].cuda(), kc_d, vc_d, plan, p, plan_longest, want_lse=True)
        torch.cuda.synchronize()
        err_p = np.abs(out_p.float().cpu().numpy().reshape(w.batch * w.hq, w.head_dim) - O).max()
        assert err_p <= TOL_BF16, f"position {p}, from the plan: max abs err {err_p}"
        assert np.abs(lse_p.cpu().numpy().reshape(-1) - LSE).max() <= TOL_BF16
        worst = max(worst, err, err_g, err_p)
        if step % 32 == 31:
            say(f"c5: up to position {p}: {int(lens.sum())} kept keys per sequence, max abs err so far {worst:.2e}")
