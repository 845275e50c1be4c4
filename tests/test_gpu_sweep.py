"""Randomized comparison of the GPU path with the oracle on many small configurations (seeded): odd sizes, tile
shapes, thresholds, count matrices, grouped-query shapes and decode positions that the hand-picked cases of the other
files may not hit."""
import numpy as np
import pytest
import torch

import oracle
import test_gpu_mask as TM
import test_gpu_prefill as TP
from paper_2506_11104_amd import binding as B
from paper_2506_11104_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-2


@pytest.mark.parametrize("seed", [1, 2])
def test_random_mask_builds_and_prefills(seed):
    rng = np.random.default_rng(seed)
    for it in range(60):
        H = int(rng.choice([1, 2, 3, 4, 6]))
        L = int(rng.choice([1, 2, 7, 33, 64, 65, 100, 128, 129, 200, 256, 300]))
        S = int(L + rng.choice([0, 1, 50, 127, 128, 300, 1000]))
        tm, tn = int(rng.choice([64, 128, 192, 256])), int(rng.choice([64, 128, 256]))
        lam = float(rng.choice([0.5, 1.0]))
        tau = float(rng.choice([0.0, 0.05, 0.2, 0.5, 1.0]))
        mu = float(rng.choice([0.0, 0.3, 0.6, 0.9, 1.1]))
        with_cnt = bool(rng.random() < 0.3)
        A = np.tril(rng.random((H, L, L), dtype=np.float32) ** rng.choice([1, 3, 6])).astype(np.float32)
        C = None
        if with_cnt:
            C = np.tril(rng.integers(0, 4, (H, L, L))).astype(np.float32)
            A = A * C
        flags = int(rng.choice([0, B.DAM_MASK_SKIP_FULL_TILE_BITS]))
        case = f"case {it}: H {H} L {L} S {S} tile {tm}x{tn} lam {lam} tau {tau} mu {mu} counts {with_cnt}"
        rows = (S - 1, S) if rng.random() < 0.5 else (max(0, S - 5), S)
        try:
            art, _ = TM.run_from_map(A, C, S, tm, tn, lam, 1e-8, tau, mu, rows=rows, dense=True)
            if tm == tn and tm in (64, 128):   # the attention kernels: bf16 at 128 x 128 tiles, fp32 at 64 x 64
                dtype, d = ("bf16", 128) if tm == 128 else ("f32", 64)
                Hkv = H // 2 if H % 2 == 0 else H
                Q = wl.to_storage(rng.standard_normal((H, S, d)).astype(np.float32) * 1.2, dtype)
                K = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), dtype)
                V = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), dtype)
                for fl in ([0, B.DAM_MASK_GATHER_COLUMNS] if dtype == "bf16" else [0]):
                    m2 = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=H, L=L, S=S, tile_m=tm, tile_n=tn, lam=lam, eps=1e-8, tau=tau,
                                      mu=mu, attn_sum=torch.from_numpy(A).cuda(),
                                      attn_cnt=None if C is None else torch.from_numpy(C).cuda(), flags=fl | flags)
                    TP.compare(Q, K, V, art, m2, dtype)
        except AssertionError as e:
            raise AssertionError(f"{case}: {e}") from e


@pytest.mark.parametrize("seed", [1, 2])
def test_random_decode_positions_in_the_three_forms(seed):
    rng = np.random.default_rng(seed)
    for it in range(25):
        G = int(rng.choice([1, 2, 4, 8]))
        Hkv = int(rng.choice([1, 2, 3]))
        Hq = G * Hkv
        T = int(rng.choice([40, 64, 65, 200, 513, 1500, 4000]))
        Bn, dh = int(rng.choice([1, 2, 5])), 128
        d = (rng.random((Hq, T)) < rng.choice([0.0, 0.01, 0.05])).astype(np.uint8)
        v = (rng.random((Hq, T)) < rng.choice([0.0, 0.01, 0.05])).astype(np.uint8)
        for h in range(Hq):
            d[h, :int(rng.integers(0, 60))] = 1
            v[h, :int(rng.integers(0, 5))] = 1
        if Hq > 1 and rng.random() < 0.3:
            d[1], v[1] = 0, 0     # a head that keeps nothing
        art = oracle.from_patterns(d, v)
        d_in, v_in = torch.from_numpy(d).cuda(), torch.from_numpy(v).cuda()
        plan = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=Hq, L=0, S=T, diag_in=d_in, vert_in=v_in, blocks=False, group=G, plan=True)
        torch.cuda.synchronize()
        want = oracle.pattern_plan(d, v, G, S=T)
        assert np.array_equal(plan.kept_ptr.cpu().numpy().astype(np.int64), want[0])
        assert np.array_equal(plan.kept_idx.cpu().numpy(), want[1]) and np.array_equal(plan.kept_member.cpu().numpy(), want[2])
        assert np.array_equal(plan.plan_table.cpu().numpy(), want[3])
        longest = max(1, int(np.diff(want[0]).max()))
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        kc = torch.randn((Bn, Hkv, T, dh), generator=g).to(torch.bfloat16)
        vc = torch.randn((Bn, Hkv, T, dh), generator=g).to(torch.bfloat16)
        q = torch.randn((Bn, Hq, dh), generator=g).to(torch.bfloat16)
        Kf = kc.float().numpy().reshape(Bn * Hkv, T, dh)
        Vf = vc.float().numpy().reshape(Bn * Hkv, T, dh)
        kv_of = np.array([b * Hkv + h // G for b in range(Bn) for h in range(Hq)], np.int32)
        kc_d, vc_d, q_d = kc.cuda(), vc.cuda(), q.cuda()
        for pos in sorted(set(int(x) for x in rng.integers(0, T, 3)) | {T - 1, 0}):
            case = f"case {it}: Hq {Hq} G {G} T {T} B {Bn} position {pos}"
            lists = [oracle.kept_list(art, h, pos) for h in range(Hq)]
            lens = np.array([len(x) for x in lists])
            ptr_all = np.concatenate([[0], np.cumsum(np.tile(lens, Bn))]).astype(np.int64)
            idx_all = np.tile(np.concatenate(lists), Bn).astype(np.int32) if lens.sum() else np.zeros(0, np.int32)
            O, LSE = oracle.attend_lists(q.float().numpy().reshape(Bn * Hq, dh), Kf, Vf, kv_of, ptr_all, idx_all)
            fin = np.isfinite(LSE)

            def check(out, lse, what):
                got = out.float().cpu().numpy().reshape(Bn * Hq, dh)
                gl = lse.cpu().numpy().reshape(-1)
                assert not np.isnan(got).any(), (case, what)
                assert np.abs(got - O).max() <= TOL, (case, what, np.abs(got - O).max())
                assert np.array_equal(np.isneginf(gl), ~fin) and (got[~fin] == 0).all(), (case, what)
                assert (np.abs(gl[fin] - LSE[fin]).max() if fin.any() else 0) <= TOL, (case, what)

            kc_p, vc_p = kc_d.clone(), vc_d.clone()     # rows beyond the position must not matter: poison them
            kc_p[:, :, pos + 1:] = float("nan")
            vc_p[:, :, pos + 1:] = float("nan")
            out, lse = B.dam_sparse_attn_decode_patterns(q_d, kc_p, vc_p, plan, pos, longest, want_lse=True)
            torch.cuda.synchronize()
            check(out, lse, "plan")
            m1 = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=Hq, L=0, S=T, diag_in=d_in, vert_in=v_in, blocks=False, rows=(pos, pos + 1))
            torch.cuda.synchronize()
            ptr = m1.kept_ptr.cpu().numpy()
            idx = m1.kept_idx.cpu().numpy() if m1.kept_idx is not None else np.zeros(0, np.int32)
            for h in range(Hq):
                assert np.array_equal(idx[ptr[h]:ptr[h + 1]], lists[h]), (case, h)
            idx_dev = torch.from_numpy(idx_all).cuda() if idx_all.size else torch.zeros(1, dtype=torch.int32, device="cuda")
            out, lse = B.dam_sparse_attn_decode(q_d, kc_d, vc_d, torch.from_numpy(ptr_all.astype(np.int32)).cuda(), idx_dev,
                                                max(1, int(lens.max())), want_lse=True)
            torch.cuda.synchronize()
            check(out, lse, "list per head")
            mg = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=Hq, L=0, S=T, diag_in=d_in, vert_in=v_in, blocks=False,
                              rows=(pos, pos + 1), group=G)
            torch.cuda.synchronize()
            wg = oracle.group_lists(lists, G)
            assert np.array_equal(mg.kept_ptr.cpu().numpy().astype(np.int64), wg[0]), case
            if wg[1].size:
                assert np.array_equal(mg.kept_idx.cpu().numpy(), wg[1]) and np.array_equal(mg.kept_member.cpu().numpy(), wg[2]), case
                out, lse = B.dam_sparse_attn_decode_grouped(q_d, kc_d, vc_d, mg.kept_ptr, mg.kept_idx, mg.kept_member,
                                                            max(1, int(np.diff(wg[0]).max())), want_lse=True, shared_lists=True)
                torch.cuda.synchronize()
                check(out, lse, "merged lists")
