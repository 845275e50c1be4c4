"""dam_sparse_attn_prefill on the GPU against the oracle (fp64 masked softmax attention).
Tolerances: max-abs 1e-4 for the fp32 kernel, 2e-2 for bf16 inputs/outputs."""
import numpy as np
import pytest
import torch

import oracle
from dam_testlib import dev
from paper_2506_11104_amd import binding as B
from paper_2506_11104_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def gpu_mask_from_art(art, S, tm, tn, flags=0):
    """Mask buffers for the kernels from an oracle-side artefact's *inputs* (flags / true mask are
    inputs of the FROM_PATTERNS mode; the S-sized outputs are built by the GPU)."""
    from dam_testlib import pack_rows_u64
    tb = None
    if art.true_mask is not None:
        tb = torch.from_numpy(pack_rows_u64(art.true_mask).view(np.int64)).cuda()
    d = np.zeros((art.H, S), np.uint8)
    v = np.zeros((art.H, S), np.uint8)
    n = min(S, art.P)
    d[:, :n], v[:, :n] = art.diag_flag[:, :n], art.vert_flag[:, :n]
    return B.build_mask(mode=B.DAM_FROM_PATTERNS, H=art.H, L=art.L, S=S, tile_m=tm, tile_n=tn,
                        diag_in=torch.from_numpy(d).cuda(), vert_in=torch.from_numpy(v).cuda(), true_bits=tb, flags=flags)


def compare(Q, K, V, art, mask, dtype, batch=1, heads_rows=None, flags=0, scale=0.0):
    Hq, S, d = Q.shape
    q, k, v = dev(Q, dtype)[None], dev(K, dtype)[None], dev(V, dtype)[None]
    if batch > 1:   # the mask is shared over the batch: entry b gets the inputs rolled by b heads
        q = torch.cat([q.roll(b, 1) for b in range(batch)], 0).contiguous()
        k = k.expand(batch, -1, -1, -1).contiguous()
        v = v.expand(batch, -1, -1, -1).contiguous()
    out, lse = B.dam_sparse_attn_prefill(q, k, v, mask, want_lse=True, flags=flags, scale=scale)
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()
    lse = lse.cpu().numpy()
    assert not np.isnan(out).any()
    if heads_rows is None:
        O, LSE = oracle.attend_prefill(Q, K, V, art, scale=scale or None)
        err = np.abs(out[0] - O).max()
        fin = np.isfinite(LSE)
        assert np.array_equal(np.isneginf(lse[0]), ~fin)
        lerr = np.abs(lse[0][fin] - LSE[fin]).max() if fin.any() else 0.0
        assert (out[0][~fin] == 0).all()
    else:
        hs, rs = heads_rows
        O, LSE = oracle.attend_rows(Q[hs, rs], K, V, art, Hq, hs, rs, scale=scale or None)
        err = np.abs(out[0][hs, rs] - O).max()
        fin = np.isfinite(LSE)
        lerr = np.abs(lse[0][hs, rs][fin] - LSE[fin]).max() if fin.any() else 0.0
    assert err <= TOL[dtype], f"max abs err {err}"
    assert lerr <= TOL[dtype], f"lse err {lerr}"
    return err


@pytest.mark.parametrize("tau,mu", [(0.257, 0.8), (0.3, 0.8), (0.0, 0.8), (0.257, 1.5)])
@pytest.mark.parametrize("tile", [64, 128])
def test_c1_fp32(tau, mu, tile):
    w = wl.WORKLOADS["c1"]
    Q, K, V = wl.qkv_iid(w, std=1 / 8)
    A = wl.capture_map(Q, K, w.pcl, 1)
    art = oracle.derive(A, None, w.lam, w.eps, tau, mu)
    mask = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=w.hq, L=w.pcl, S=w.seq, tile_m=tile, tile_n=tile, lam=w.lam,
                        eps=w.eps, tau=tau, mu=mu, attn_sum=torch.from_numpy(A).cuda())
    compare(Q, K, V, art, mask, "f32")


def random_patterns(rng, H, S, L=0):
    d = (rng.random((H, S)) < 0.01).astype(np.uint8)
    v = (rng.random((H, S)) < 0.01).astype(np.uint8)
    for h in range(H):
        d[h, :int(rng.integers(1, 200))] = 1
        v[h, :int(rng.integers(1, 9))] = 1
    if H > 2:
        d[2], v[2] = 0, 0
        d[2, 300] = 1                      # rows < 300 of head 2 are empty
    tm = None
    if L:
        tm = (rng.random((H, L, L)) < 0.3).astype(np.uint8) * np.tril(np.ones((L, L), np.uint8))
    return oracle.from_patterns(d, v, tm)


@pytest.mark.parametrize("dtype,d,S,tile", [("bf16", 128, 1000, 128), ("bf16", 128, 384, 128), ("f32", 128, 700, 128),
                                            ("f32", 64, 333, 64)])
def test_mid_size_ragged_gqa_batch(dtype, d, S, tile):
    rng = np.random.default_rng(31)
    Hq, Hkv = 4, 2
    Q = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32) * 1.5, dtype)
    K = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), dtype)
    V = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), dtype)
    art = random_patterns(rng, Hq, S, L=90)
    mask = gpu_mask_from_art(art, S, tile, tile)
    compare(Q, K, V, art, mask, dtype)
    # batch of 3 sharing the mask: check entry 2 (inputs rolled by two heads) against the oracle
    q = torch.cat([dev(Q, dtype)[None].roll(b, 1) for b in range(3)], 0).contiguous()
    k = dev(K, dtype)[None].expand(3, -1, -1, -1).contiguous()
    v = dev(V, dtype)[None].expand(3, -1, -1, -1).contiguous()
    out = B.dam_sparse_attn_prefill(q, k, v, mask)
    torch.cuda.synchronize()
    O2, _ = oracle.attend_prefill(np.roll(Q, 2, 0), K, V, art)
    assert np.abs(out[2].float().cpu().numpy() - O2).max() <= TOL[dtype]


def test_dense_causal_bf16_matches_oracle_and_is_all_full_tiles():
    rng = np.random.default_rng(32)
    Hq, Hkv, S, d = 2, 1, 512, 128
    Q = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32), "bf16")
    K = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), "bf16")
    V = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), "bf16")
    art = oracle.from_patterns(np.ones((Hq, S), np.uint8), np.zeros((Hq, S), np.uint8))
    mask = gpu_mask_from_art(art, S, 128, 128)
    assert int((mask.blk_kind & 1).sum().item()) == Hq * 6          # 4*3/2 strictly-below-diagonal tiles per head
    compare(Q, K, V, art, mask, "bf16")


@pytest.mark.parametrize("dtype,d,tile", [("bf16", 128, 128), ("f32", 64, 64)])
def test_full_tiles_are_never_read(dtype, d, tile):
    """With DAM_MASK_SKIP_FULL_TILE_BITS the pool slots of full tiles are unwritten: both kernels must
    take such tiles from blk_kind alone. The slots are filled with a pattern that would wreck the result."""
    rng = np.random.default_rng(35)
    Hq, Hkv, S = 2, 1, 900
    Q = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32), dtype)
    K = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), dtype)
    V = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), dtype)
    dflag = np.zeros((Hq, S), np.uint8)
    vflag = np.zeros((Hq, S), np.uint8)
    dflag[0, :500] = 1
    dflag[1, :333] = 1
    vflag[1, :3] = 1
    art = oracle.from_patterns(dflag, vflag)
    mask = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=Hq, L=0, S=S, tile_m=tile, tile_n=tile,
                        diag_in=torch.from_numpy(dflag).cuda(), vert_in=torch.from_numpy(vflag).cuda(),
                        flags=B.DAM_MASK_SKIP_FULL_TILE_BITS)
    full = (mask.blk_kind & 1).bool()
    assert int(full.sum()) >= 6
    mask.tile_bits[full] = 0x0F0F0F0F00000000
    compare(Q, K, V, art, mask, dtype)


@pytest.mark.parametrize("dtype,d,S,tile,L", [("bf16", 128, 1000, 128, 90), ("bf16", 128, 1300, 128, 0), ("f32", 64, 500, 64, 70),
                                              ("f32", 128, 700, 128, 0)])
def test_gathered_column_tiles_give_the_same_attention(dtype, d, S, tile, L):
    """The block index with the matched columns gathered into tiles of their own describes the same
    mask: outputs against the oracle, GQA, batch of two, many columns (several gathered tiles)."""
    rng = np.random.default_rng(36)
    Hq, Hkv = 4, 2
    Q = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32) * 1.5, dtype)
    K = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), dtype)
    V = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), dtype)
    art = random_patterns(rng, Hq, S, L=L)
    art.vert_flag[1, rng.choice(S, size=300, replace=False)] = 1       # three gathered tiles for head 1
    art.vert_flag[3] = 0                                                # none for head 3
    mask = gpu_mask_from_art(art, S, tile, tile, flags=B.DAM_MASK_GATHER_COLUMNS | B.DAM_MASK_SKIP_FULL_TILE_BITS)
    nKt = (S + tile - 1) // tile
    assert int((mask.blk_col >= nKt).sum()) > 0 and mask.gather_rows >= 300
    mask.tile_bits[(mask.blk_kind & 1).bool()] = 0x0F0F0F0F00000000    # unwritten slots of full tiles
    compare(Q, K, V, art, mask, dtype, batch=2)


def test_large_logits_do_not_overflow():
    # a masked-out key with a huge logit must not disturb the kept ones (mask before the max)
    rng = np.random.default_rng(33)
    Hq, S, d = 1, 256, 128
    Q = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32), "bf16")
    K = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32), "bf16")
    V = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32), "bf16")
    K[0, 5] = Q[0].mean(0) * 400.0
    K[0, 5] = wl.to_storage(K[0, 5], "bf16")
    dflag = np.zeros((1, S), np.uint8)
    dflag[0, :3] = 1                       # window of 3: key 5 is masked for rows >= 8
    art = oracle.from_patterns(dflag, np.zeros((1, S), np.uint8))
    mask = gpu_mask_from_art(art, S, 128, 128)
    compare(Q, K, V, art, mask, "bf16")


def test_c2_full_size():
    w = wl.WORKLOADS["c2"]
    Q, K, V = wl.qkv_structured(w)
    A = wl.capture_map(Q, K, w.pcl, w.hq // w.hkv)
    art = oracle.derive(A, None, w.lam, w.eps, w.tau, w.mu)
    mask = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=w.hq, L=w.pcl, S=w.seq, lam=w.lam, eps=w.eps, tau=w.tau, mu=w.mu,
                        attn_sum=torch.from_numpy(A).cuda())
    compare(Q, K, V, art, mask, "bf16")


def test_c3_full_size_every_row_both_layouts():
    """The benchmark workload in the launch shape bench.py times: every one of the 32 x 32768 output rows and
    log-sum-exps against the oracle, for the gathered-column layout (the one the benchmark step uses) and for
    the plain one (both describe the same mask, so the oracle runs once)."""
    w = wl.WORKLOADS["c3"]
    Q, K, V = wl.qkv_iid(w)
    dflag, vflag = wl.patterns_c3(w)
    art = oracle.from_patterns(dflag, vflag)
    O, LSE = oracle.attend_prefill(Q, K, V, art)
    fin = np.isfinite(LSE)
    q, k, v = dev(Q, "bf16")[None], dev(K, "bf16")[None], dev(V, "bf16")[None]
    for flags in (B.DAM_MASK_SKIP_FULL_TILE_BITS | B.DAM_MASK_GATHER_COLUMNS, B.DAM_MASK_SKIP_FULL_TILE_BITS):
        # as bench.py builds it: full tiles carry no bits
        mask = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=w.hq, L=0, S=w.seq, diag_in=torch.from_numpy(dflag).cuda(),
                            vert_in=torch.from_numpy(vflag).cuda(), flags=flags)
        mask.tile_bits[(mask.blk_kind & 1).bool()] = 0
        out, lse = B.dam_sparse_attn_prefill(q, k, v, mask, want_lse=True)
        torch.cuda.synchronize()
        got, got_lse = out[0].float().cpu().numpy(), lse[0].cpu().numpy()
        assert not np.isnan(got).any()
        assert np.array_equal(np.isneginf(got_lse), ~fin)
        err = max(float(np.abs(got[h] - O[h]).max()) for h in range(w.hq))      # (per head: no 1 GiB temporary)
        assert err <= TOL["bf16"], f"flags {flags}: max abs err {err}"
        assert np.abs(got_lse[fin] - LSE[fin]).max() <= TOL["bf16"]
        assert (got[~fin] == 0).all()
        del mask, out, lse


@pytest.mark.parametrize("S,flags", [(128 * 300, 0), (128 * 131 - 37, B.DAM_MASK_GATHER_COLUMNS)])
def test_query_tiles_with_more_listed_tiles_than_one_list_segment(S, flags):
    """The bf16 kernel expands the listed tiles of a query tile 128 at a time. Head 0 is dense causal (up to
    S / 128 tiles per query tile), head 1 keeps every fourth diagonal block and scattered columns (partial
    tiles in every segment); rows around the segment boundaries and the last rows are checked."""
    rng = np.random.default_rng(35)
    Hq, Hkv, d = 2, 1, 128
    Q = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32), "bf16")
    K = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), "bf16")
    V = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), "bf16")
    dflag = np.ones((Hq, S), np.uint8)
    dflag[1] = (np.arange(S) // 96) % 4 == 0
    vflag = np.zeros((Hq, S), np.uint8)
    vflag[1, rng.choice(S, 200, replace=False)] = 1
    art = oracle.from_patterns(dflag, vflag)
    mask = gpu_mask_from_art(art, S, 128, 128, flags=flags | B.DAM_MASK_SKIP_FULL_TILE_BITS)
    nQt = (S + 127) // 128
    per_row = (mask.blk_row_ptr[:, 1:] - mask.blk_row_ptr[:, :-1]).cpu().numpy()
    assert per_row.max() > 128        # at least two segments in the longest rows (three at S = 38400)
    rows = np.unique(np.concatenate([np.arange(S - 130, S), 128 * 127 + np.arange(0, 260), 128 * 255 + np.arange(0, 260),
                                     rng.integers(0, S, 200)]))
    rows = rows[rows < S]
    hs = np.concatenate([np.zeros(len(rows), np.int32), np.ones(len(rows), np.int32)])
    rs = np.concatenate([rows, rows]).astype(np.int64)
    compare(Q, K, V, art, mask, "bf16", heads_rows=(hs, rs))


@pytest.mark.parametrize("dtype,d,tile,S", [(torch.bfloat16, 128, 128, 700), (torch.bfloat16, 128, 128, 1024), (torch.float32, 64, 64, 333)])
def test_strided_layouts_give_the_same_bits_as_contiguous_ones(dtype, d, tile, S):
    """The entry point takes element strides: Q, K, V and O stored sequence-major ([B][S][H][d], the heads of a
    token side by side) and as slices of wider buffers give the same output bits as contiguous [B][H][S][d]
    tensors (whose parity with the oracle the other tests check). Gathered column tiles included: their copies
    follow the row stride of K and of V."""
    rng = np.random.default_rng(37)
    Bn, Hq, Hkv = 2, 4, 2
    art = random_patterns(rng, Hq, S, L=0)
    art.vert_flag[0, rng.choice(S, size=150, replace=False)] = 1
    mask = gpu_mask_from_art(art, S, tile, tile, flags=B.DAM_MASK_GATHER_COLUMNS if dtype == torch.bfloat16 else 0)
    g = torch.Generator().manual_seed(8)
    q = torch.randn((Bn, Hq, S, d), generator=g).to(dtype).cuda()
    k = torch.randn((Bn, Hkv, S, d), generator=g).to(dtype).cuda()
    v = torch.randn((Bn, Hkv, S, d), generator=g).to(dtype).cuda()
    want, want_lse = B.dam_sparse_attn_prefill(q, k, v, mask, want_lse=True)
    # sequence-major storage, K and V with different row strides (V padded), O into a slice of a wider buffer
    q2 = q.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    k2 = k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    v_wide = torch.zeros((Bn, S, Hkv, 2 * d), dtype=dtype, device="cuda")
    v_wide[..., :d] = v.permute(0, 2, 1, 3)
    v2 = v_wide[..., :d].permute(0, 2, 1, 3)
    o_wide = torch.full((Bn, Hq, S, d + 64), 3.0, dtype=dtype, device="cuda")
    o2 = o_wide[..., :d]
    assert not q2.is_contiguous() and k2.stride() != v2.stride() and not o2.is_contiguous()
    got, got_lse = B.dam_sparse_attn_prefill(q2, k2, v2, mask, out=o2, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(got, want) and torch.equal(got_lse, want_lse)
    assert (o_wide[..., d:] == 3.0).all()          # nothing written outside the slice


@pytest.mark.parametrize("S", [1, 5, 31, 33, 127, 129])
def test_tiny_sequences_bf16(S):
    """Sequences shorter than a key block, a tile, or just past one: the copies of a block that reaches past the
    end are redirected to the last row, the rows past the end are never stored."""
    rng = np.random.default_rng(38 + S)
    Hq, Hkv, d = 2, 1, 128
    Q = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32), "bf16")
    K = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), "bf16")
    V = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), "bf16")
    dflag = np.ones((Hq, S), np.uint8)                       # head 0: dense causal
    dflag[1] = (np.arange(S) % 3 == 0)                       # head 1: every third diagonal
    vflag = np.zeros((Hq, S), np.uint8)
    vflag[1, 0] = 1
    art = oracle.from_patterns(dflag, vflag)
    for flags in (0, B.DAM_MASK_GATHER_COLUMNS):
        mask = gpu_mask_from_art(art, S, 128, 128, flags=flags)
        compare(Q, K, V, art, mask, "bf16")


# ---------------------------------------------------------------------------------------------
# The bf16 kernel's two softmax variants: without a running maximum first (the weights are exp2 of the
# logits themselves), then, for the query tiles in which a row's sum of weights left the safe range, with one.
def _qkv(rng, Hq, Hkv, S, d=128, qs=1.0):
    Q = wl.to_storage(rng.standard_normal((Hq, S, d)).astype(np.float32) * qs, "bf16")
    K = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), "bf16")
    V = wl.to_storage(rng.standard_normal((Hkv, S, d)).astype(np.float32), "bf16")
    return Q, K, V


@pytest.mark.parametrize("S,L,flags", [(1000, 90, 0), (1300, 0, B.DAM_MASK_GATHER_COLUMNS), (384, 0, 0)])
def test_running_reference_variant_alone(S, L, flags):
    """DAM_ATTN_RUNNING_REFERENCE: every work item goes through the variant with the running maximum (ragged
    and exact lengths, gathered tiles, GQA, a batch of two)."""
    rng = np.random.default_rng(71)
    Q, K, V = _qkv(rng, 4, 2, S, qs=1.5)
    art = random_patterns(rng, 4, S, L=L)
    mask = gpu_mask_from_art(art, S, 128, 128, flags=flags | B.DAM_MASK_SKIP_FULL_TILE_BITS)
    compare(Q, K, V, art, mask, "bf16", batch=2, flags=B.DAM_ATTN_RUNNING_REFERENCE)


@pytest.mark.parametrize("scale,what", [(6.0, "overflow"), (40.0, "overflow and underflow"), (0.0, "one head only")])
def test_rows_outside_the_range_of_the_plain_exponential_are_redone(scale, what):
    """Logits far beyond what exp2 without a reference can carry: at scale 6 the logits have a standard deviation of
    about 68 (weights up to 2^300 and down to 2^-300), at scale 40 every row overflows or underflows. The first pass
    flags such rows (sum of weights infinite, NaN, tiny or zero), the second pass recomputes their query tiles, and the
    results match the oracle like any others. "one head only": head 1's queries are multiplied by 64, head 0 and the
    other batch entry stay ordinary, so both passes contribute rows to one output."""
    rng = np.random.default_rng(72)
    S = 700
    Q, K, V = _qkv(rng, 2, 1, S)
    if what == "one head only":
        Q[1] = wl.to_storage(Q[1] * 64.0, "bf16")
    art = random_patterns(rng, 2, S, L=0)
    mask = gpu_mask_from_art(art, S, 128, 128)
    compare(Q, K, V, art, mask, "bf16", batch=2, scale=scale)
    # the same through the flag: both routes give the same bits for the rows the second pass handles
    q, k, v = dev(Q, "bf16")[None], dev(K, "bf16")[None], dev(V, "bf16")[None]
    a = B.dam_sparse_attn_prefill(q, k, v, mask, scale=scale)
    b = B.dam_sparse_attn_prefill(q, k, v, mask, scale=scale, flags=B.DAM_ATTN_RUNNING_REFERENCE)
    torch.cuda.synchronize()
    if what != "one head only":
        assert torch.equal(a, b)
    else:
        assert torch.equal(a[0, 1], b[0, 1]) and not torch.equal(a[0, 0], b[0, 0])


def test_all_logits_far_below_zero_underflow_is_caught():
    """Every kept logit of a row around -200 * log2(e): all weights flush to zero without a reference; the row has
    kept keys, so its zero sum sends the tile to the second pass (an empty row's zero sum does not)."""
    rng = np.random.default_rng(73)
    S, d = 300, 128
    u = rng.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    Q = wl.to_storage(np.tile(u * 48.0, (1, S, 1)) + 0.05 * rng.standard_normal((1, S, d)).astype(np.float32), "bf16")
    K = wl.to_storage(np.tile(-u * 48.0, (1, S, 1)) + 0.05 * rng.standard_normal((1, S, d)).astype(np.float32), "bf16")
    V = wl.to_storage(rng.standard_normal((1, S, d)).astype(np.float32), "bf16")
    dflag = np.zeros((1, S), np.uint8)
    dflag[0, 2:9] = 1                                   # rows 0 and 1 keep nothing: empty rows among failed ones
    art = oracle.from_patterns(dflag, np.zeros((1, S), np.uint8))
    mask = gpu_mask_from_art(art, S, 128, 128)
    compare(Q, K, V, art, mask, "bf16")
