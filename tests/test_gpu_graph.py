"""The entry points under HIP graph capture: they allocate nothing, never synchronise and record no
memset, so a caller can capture a whole step (mask build + prefill, or list build + decode) and replay
it. Every replay is checked against the eager result; the replays are separated by eager work and
synchronisations of the program's own."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2506_11104_amd import binding as B

pytestmark = pytest.mark.gpu


def patterns(rng, H, S):
    d = (rng.random((H, S)) < 0.01).astype(np.uint8)
    v = (rng.random((H, S)) < 0.01).astype(np.uint8)
    for h in range(H):
        d[h, :60 + 40 * h] = 1
        v[h, :4] = 1
    return d, v


def test_mask_build_and_prefill_replayed_from_a_graph():
    rng = np.random.default_rng(71)
    Hq, Hkv, S, d = 4, 2, 1000, 128
    dflag, vflag = patterns(rng, Hq, S)
    d_in, v_in = torch.from_numpy(dflag).cuda(), torch.from_numpy(vflag).cuda()
    flags = B.DAM_MASK_SKIP_FULL_TILE_BITS | B.DAM_MASK_GATHER_COLUMNS
    # sizes from an eager build; the captured step then writes into buffers of its own
    m0 = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=Hq, L=0, S=S, diag_in=d_in, vert_in=v_in, flags=flags)
    p = B.MaskParams(B.DAM_FROM_PATTERNS, Hq, 0, S, 128, 128, 0, 0, 0.5, 1e-8, 0.3, 0.8, float("nan"), flags)
    ws_m = B.mask_workspace(p, "cuda")
    m = B.Mask(H=Hq, L=0, S=S, tile_m=128, tile_n=128)
    m.blk_row_ptr = torch.zeros_like(m0.blk_row_ptr)
    m.blk_col, m.blk_kind, m.tile_bits = torch.zeros_like(m0.blk_col), torch.zeros_like(m0.blk_kind), torch.zeros_like(m0.tile_bits)
    m.gather_idx, m.gather_cnt, m.gather_rows, m.n_tiles = torch.zeros_like(m0.gather_idx), torch.zeros_like(m0.gather_cnt), m0.gather_rows, m0.n_tiles
    total = torch.zeros(1, dtype=torch.int64, device="cuda")
    o = B.MaskOut()
    o.blk_row_ptr, o.blk_col, o.blk_kind, o.tile_bits = (m.blk_row_ptr.data_ptr(), m.blk_col.data_ptr(), m.blk_kind.data_ptr(),
                                                         m.tile_bits.data_ptr())
    o.blk_capacity, o.blk_total = m.n_tiles, total.data_ptr()
    o.gather_idx, o.gather_cnt = m.gather_idx.data_ptr(), m.gather_cnt.data_ptr()
    g = torch.Generator().manual_seed(3)
    q = torch.randn((1, Hq, S, d), generator=g).to(torch.bfloat16).cuda()
    k = torch.randn((1, Hkv, S, d), generator=g).to(torch.bfloat16).cuda()
    v = torch.randn((1, Hkv, S, d), generator=g).to(torch.bfloat16).cuda()
    out = torch.empty_like(q)
    ws_a = B.prefill_workspace(B.attn_params(q, k, v, out, 128, 128, gather_rows=m.gather_rows), "cuda")

    def step():
        B.dam_mask_build(p, None, None, d_in, v_in, o, ws_m)
        B.dam_sparse_attn_prefill(q, k, v, m, out=out, ws=ws_a)

    step()  # eager: loads the code objects, and gives the reference
    torch.cuda.synchronize()
    want = out.clone()
    assert torch.equal(m.blk_col, m0.blk_col) and torch.equal(m.blk_kind, m0.blk_kind)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        # new inputs for the replay, and eager work of the same library in between
        q.copy_(torch.randn((1, Hq, S, d), generator=g).to(torch.bfloat16))
        m.blk_col.zero_()
        m.tile_bits.zero_()
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        assert torch.equal(m.blk_col, m0.blk_col), f"replay {rep}: block index"
        out.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(got, out), f"replay {rep}: attention output differs from the eager call"
    assert not torch.equal(out, want)  # the inputs did change


def test_list_build_and_grouped_decode_replayed_from_a_graph():
    rng = np.random.default_rng(72)
    Bn, Hq, Hkv, d, cap = 3, 8, 2, 128, 6000
    G = Hq // Hkv
    dflag, vflag = patterns(rng, Hq, cap)
    d_in, v_in = torch.from_numpy(dflag).cuda(), torch.from_numpy(vflag).cuda()
    pos = cap - 2
    p = B.MaskParams(B.DAM_FROM_PATTERNS, Hq, 0, cap, 128, 128, pos, pos + 1, 0.5, 1e-8, 0.3, 0.8, float("nan"),
                     B.DAM_MASK_GROUP_LISTS, 0, G)
    ws_m = B.mask_workspace(p, "cuda")
    n_max = Hq * (pos + 1)
    ptr = torch.zeros(Hkv + 1, dtype=torch.int32, device="cuda")
    idx = torch.zeros(n_max, dtype=torch.int32, device="cuda")
    mem = torch.zeros(n_max, dtype=torch.uint8, device="cuda")
    total = torch.zeros(1, dtype=torch.int64, device="cuda")
    o = B.MaskOut()
    o.kept_ptr, o.kept_idx, o.kept_member, o.kept_capacity, o.kept_total = ptr.data_ptr(), idx.data_ptr(), mem.data_ptr(), n_max, total.data_ptr()
    g = torch.Generator().manual_seed(4)
    q = torch.randn((Bn, Hq, d), generator=g).to(torch.bfloat16).cuda()
    kc = torch.randn((Bn, Hkv, cap, d), generator=g).to(torch.bfloat16).cuda()
    vc = torch.randn((Bn, Hkv, cap, d), generator=g).to(torch.bfloat16).cuda()
    out = torch.empty_like(q)
    ws_d = B.decode_grouped_workspace(B.decode_params(q, kc, out, shared_lists=True), pos + 1, "cuda")

    def step():
        B.dam_mask_build(p, None, None, d_in, v_in, o, ws_m)
        B.dam_sparse_attn_decode_grouped(q, kc, vc, ptr, idx, mem, pos + 1, out=out, ws=ws_d, shared_lists=True)

    step()
    torch.cuda.synchronize()
    art = oracle.from_patterns(dflag, vflag)
    want_lists = oracle.group_lists([oracle.kept_list(art, h, pos) for h in range(Hq)], G)
    n = int(want_lists[0][-1])
    assert np.array_equal(idx.cpu().numpy()[:n], want_lists[1])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        q.copy_(torch.randn((Bn, Hq, d), generator=g).to(torch.bfloat16))
        idx.zero_()
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        assert np.array_equal(idx.cpu().numpy()[:n], want_lists[1]), f"replay {rep}: lists"
        out.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(got, out), f"replay {rep}: decode output differs from the eager call"
