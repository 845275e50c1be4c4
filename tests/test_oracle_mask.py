"""Pins of the oracle's mask derivation against what the paper and the mathematics fix.

None of these re-types the oracle's own formula in the same form: they use closed forms, printed
values, literally materialised pattern matrices, special cases and invariants.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
PAPER = dict(lam=0.5, eps=1e-8, tau=0.3, mu=0.8)   # Sec. 5.1 "DAM Configuration", Sec. 4.2.2


def softmax_map(rng, H, L, sharp=2.0):
    s = rng.standard_normal((H, L, L)) * sharp
    s[:, ~np.tril(np.ones((L, L), bool))] = -np.inf
    e = np.exp(s - s.max(-1, keepdims=True))
    return (e / e.sum(-1, keepdims=True)).astype(np.float32)


def read_golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = v
    return out


# ---------------------------------------------------------------- Sec. 4.2.2, Box-Cox + shift
def test_boxcox_printed_max_value():
    # App. B table prints "Max Value 2.00" for the Box-Cox map: probability 1 with the global
    # minimum at the clamp gives 2 (1 - sqrt(eps)); both eps values the paper names print as 2.00.
    g = read_golden("boxcox_table_appB.txt")
    A = np.zeros((1, 2, 2), np.float32)
    A[0, 0, 0] = 1.0
    A[0, 1, 0] = 0.25
    A[0, 1, 1] = 0.75
    for eps in (1e-8, 1e-10):
        B, bmin = oracle.boxcox(A, None, 0.5, eps)
        bstar = B - bmin
        assert f"{bstar.max():.2f}" == g["max_value"]
        assert abs(float(bstar.max()) - 2.0 * (1.0 - np.sqrt(eps))) < 1e-6
        assert bstar[0, 0, 1] == 0.0          # never-valid pair sits at the global minimum exactly


def test_boxcox_closed_forms():
    rng = np.random.default_rng(1)
    A = softmax_map(rng, 3, 17)
    eps = 1e-8
    X = np.maximum(A.astype(np.float64) * np.tril(np.ones((17, 17))) / (np.tril(np.ones((17, 17))) + eps), eps)
    # lambda = 0.5: B* = 2 (sqrt X - sqrt Xmin)
    B, bmin = oracle.boxcox(A, None, 0.5, eps)
    np.testing.assert_allclose(B - bmin, 2.0 * (np.sqrt(X) - np.sqrt(X.min())), atol=5e-7)
    # lambda = 1: B* = X - Xmin
    B, bmin = oracle.boxcox(A, None, 1.0, eps)
    np.testing.assert_allclose(B - bmin, X - X.min(), atol=2e-7)
    # lambda = 0: ln X - ln Xmin
    B, bmin = oracle.boxcox(A, None, 0.0, eps)
    np.testing.assert_allclose(B - bmin, np.log(X) - np.log(X.min()), rtol=1e-5, atol=1e-5)
    # general lambda, against scipy's Box-Cox
    from scipy.special import boxcox as sp_boxcox
    B, bmin = oracle.boxcox(A, None, 0.3, eps)
    np.testing.assert_allclose(B, sp_boxcox(X, 0.3), rtol=2e-5, atol=2e-5)
    assert bmin == B.min()


def test_boxcox_min_is_global_and_monotone():
    rng = np.random.default_rng(2)
    A = softmax_map(rng, 4, 9)
    B, bmin = oracle.boxcox(A, None, 0.5, 1e-8)
    assert bmin == B.min()
    # with a causal capture and L >= 2 the minimum is the Box-Cox of the clamp itself
    assert abs(float(bmin) - (np.sqrt(1e-8) - 1.0) / 0.5) < 1e-6
    # Box-Cox is increasing: ordering of A on valid pairs is preserved (ties allowed by rounding)
    a = A[0][np.tril_indices(9)]
    b = B[0][np.tril_indices(9)]
    order = np.argsort(a, kind="stable")
    assert np.all(np.diff(b[order]) >= 0)


def test_null_count_ignores_upper_triangle_and_counts_average():
    rng = np.random.default_rng(3)
    L = 12
    A = softmax_map(rng, 2, L)
    junk = A.copy()
    junk[:, ~np.tril(np.ones((L, L), bool))] = 7.0          # never read when C is NULL
    B0, m0 = oracle.boxcox(A, None, 0.5, 1e-8)
    B1, m1 = oracle.boxcox(junk, None, 0.5, 1e-8)
    assert m0 == m1 and np.array_equal(B0, B1)
    # explicit C equal to the implied one gives the same map
    C = np.broadcast_to(np.tril(np.ones((L, L), np.float32)), A.shape).copy()
    B2, m2 = oracle.boxcox(A, C, 0.5, 1e-8)
    assert m0 == m2 and np.array_equal(B0, B2)
    # three identical captures summed, C = 3: the mean is the single capture (up to rounding of 3a/3)
    B3, m3 = oracle.boxcox(3 * A, 3 * C, 0.5, 1e-8)
    np.testing.assert_allclose(B3, B0, atol=1e-6)
    # a pair seen in only one of three captures is divided by 1, not 3
    A4, C4 = (3 * A).copy(), (3 * C).copy()
    A4[0, 5, 2], C4[0, 5, 2] = A[0, 5, 2], 1.0
    B4, _ = oracle.boxcox(A4, C4, 0.5, 1e-8)
    assert abs(B4[0, 5, 2] - B0[0, 5, 2]) < 1e-6


# ---------------------------------------------------------------- Sec. 4.2.3, true mask
def test_true_mask_special_cases_and_threshold_equivalence():
    rng = np.random.default_rng(4)
    L = 40
    A = softmax_map(rng, 3, L, sharp=3.0)
    tri = np.tril(np.ones((L, L), bool))
    B, bmin = oracle.boxcox(A, None, 0.5, 1e-8)
    assert np.array_equal(oracle.true_mask(B, bmin, 0.0).astype(bool), np.broadcast_to(tri, A.shape))
    assert np.array_equal(oracle.true_mask(B, bmin, -1.0).astype(bool), np.broadcast_to(tri, A.shape))
    assert oracle.true_mask(B, bmin, 2.01).sum() == 0          # B* <= 2 (1 - sqrt eps) < 2
    # B* >= tau  <=>  X >= theta = (tau/2 + sqrt(eps))^2, away from the rounding boundary
    for tau in (0.3, 0.1, 0.02):
        m = oracle.true_mask(B, bmin, tau).astype(bool)
        theta = (tau / 2 + np.sqrt(1e-8)) ** 2
        X = A.astype(np.float64)
        sure = np.abs(X - theta) > 1e-5 * theta + 1e-9
        expect = (X >= theta) & tri
        assert np.array_equal(m[sure], expect[sure])
        assert (~sure).sum() < 10
        # rows of a softmax sum to one, so no row keeps more than floor(1/theta) keys
        assert m.sum(-1).max() <= int(1.0 / theta)


def test_true_mask_is_causal_even_with_counts_above_diagonal():
    # C given with "valid" pairs above the diagonal: causality is still enforced.
    L = 6
    A = np.full((1, L, L), 0.5, np.float32)
    C = np.ones((1, L, L), np.float32)
    B, bmin = oracle.boxcox(A, C, 0.5, 1e-8)
    m = oracle.true_mask(B, bmin - 1.0, 0.3)
    assert np.array_equal(m[0].astype(bool), np.tril(np.ones((L, L), bool)))


# ---------------------------------------------------------------- Sec. 4.2.4, pattern matching
def brute_match(m, mu):
    """gamma_k = sum(M * P_k) / sum(P_k) with every P_k materialised as an L x L matrix."""
    L = m.shape[0]
    ii, jj = np.meshgrid(np.arange(L), np.arange(L), indexing="ij")
    gd, gv = np.zeros(L), np.zeros(L)
    for r in range(L):
        P = (jj == ii - r)
        gd[r] = (m * P).sum() / P.sum()
    for c in range(L):
        P = (jj == c) & (ii >= c)
        gv[c] = (m * P).sum() / P.sum()
    return gd, gv


def test_match_against_materialised_patterns():
    rng = np.random.default_rng(5)
    for L in (1, 2, 7, 32):
        m = (rng.random((3, L, L)) < 0.6).astype(np.uint8) * np.tril(np.ones((L, L), np.uint8))
        for mu in (0.5, 0.8):
            dc, vc, df, vf = oracle.match(m, mu)
            for h in range(3):
                gd, gv = brute_match(m[h], mu)
                sizes = L - np.arange(L)
                assert np.array_equal(dc[h], np.rint(gd * sizes).astype(np.int32))
                assert np.array_equal(vc[h], np.rint(gv * sizes).astype(np.int32))
                far_d = np.abs(gd - mu) > 1e-6
                far_v = np.abs(gv - mu) > 1e-6
                assert np.array_equal(df[h][far_d].astype(bool), (gd >= mu)[far_d])
                assert np.array_equal(vf[h][far_v].astype(bool), (gv >= mu)[far_v])


def test_match_hand_built_masks():
    L = 16
    ii, jj = np.meshgrid(np.arange(L), np.arange(L), indexing="ij")
    for r in (0, 3, 15):
        m = (jj == ii - r).astype(np.uint8)[None]
        dc, vc, df, vf = oracle.match(m, 1.0)
        assert dc[0, r] == L - r and df[0, r] == 1
        assert df[0].sum() == 1                                  # no other diagonal matches
        # column c holds exactly one entry of that diagonal (row c + r) when it exists
        assert np.array_equal(vc[0], ((np.arange(L) + r) <= L - 1).astype(np.int32))
        # ... so only a column of size 1 can reach gamma = 1: c = L-1 when r = 0
        assert np.array_equal(np.flatnonzero(vf[0]), np.array([L - 1]) if r == 0 else np.array([], int))
    # a column: matched as that column; diagonal r has one entry of it (row c + r)
    c = 5
    m = ((jj == c) & (ii >= c)).astype(np.uint8)[None]
    dc, vc, df, vf = oracle.match(m, 1.0)
    assert vc[0, c] == L - c and vf[0, c] == 1 and vf[0].sum() == 1
    assert np.array_equal(dc[0], ((np.arange(L) + c) <= L - 1).astype(np.int32))
    # ">= mu" (the equations), not ">": 4 of 5 kept with mu = 0.8 matches
    m = np.zeros((1, 5, 5), np.uint8)
    m[0, 1:, 0] = 1
    _, vc, _, vf = oracle.match(m, 0.8)
    assert vc[0, 0] == 4 and vf[0, 0] == 1
    # mu = 0 matches all 2L patterns, mu > 1 none
    m = np.zeros((1, 8, 8), np.uint8)
    _, _, df, vf = oracle.match(m, 0.0)
    assert df.all() and vf.all()
    _, _, df, vf = oracle.match(np.tril(np.ones((1, 8, 8), np.uint8)), 1.0001)
    assert not df.any() and not vf.any()
    # single hit at (L-1, 0): the one-entry diagonal r = L-1 matches (no minimum support)
    m = np.zeros((1, 8, 8), np.uint8)
    m[0, 7, 0] = 1
    _, _, df, vf = oracle.match(m, 0.8)
    assert np.array_equal(np.flatnonzero(df[0]), [7]) and not vf.any()


# ---------------------------------------------------------------- Sec. 4.3, applying / extending
def make_art(rng, H=3, L=24, tau=0.08, mu=0.6):
    A = softmax_map(rng, H, L, sharp=1.0)
    A[:, :, 0] += 0.2            # a sink column
    A /= A.sum(-1, keepdims=True)
    return oracle.derive(A, None, 0.5, 1e-8, tau, mu)


def test_extension_cases():
    rng = np.random.default_rng(6)
    art = make_art(rng)
    L = art.L
    assert art.vert_flag[:, 0].all()
    for h in range(art.H):
        # Case 1: S <= L is the crop of the true mask
        for S in (1, 5, L):
            assert np.array_equal(oracle.rows(art, h, S, 0, S), art.true_mask[h][:S, :S])
        # Case 2: top-left block unchanged; elsewhere union of matched patterns, causal
        S = 3 * L + 5
        M = oracle.rows(art, h, S, 0, S)
        assert np.array_equal(M[:L, :L], art.true_mask[h])
        ii, jj = np.meshgrid(np.arange(S), np.arange(S), indexing="ij")
        R = np.flatnonzero(art.diag_flag[h])
        Cc = np.flatnonzero(art.vert_flag[h])
        expect = (np.isin(ii - jj, R) | np.isin(jj, Cc)) & (jj <= ii)
        outside = (ii >= L) | (jj >= L)
        assert np.array_equal(M[outside].astype(bool), expect[outside])
        # rows >= L reach columns < L through the vertical patterns (the sink survives)
        assert M[L:, 0].all()
        # a row outside the block keeps at most |R| + |C| keys
        assert M[L:].sum(1).max() <= len(R) + len(Cc)
        # prefix stability: building at S and cropping equals building at S'
        for S2 in (L, L + 1, 2 * L, S - 1):
            assert np.array_equal(M[:S2, :S2], oracle.rows(art, h, S2, 0, S2))
        # single-entry access and kept lists agree with the rows
        for i in (0, L - 1, L, S - 1):
            assert np.array_equal(oracle.kept_list(art, h, i), np.flatnonzero(M[i]))
            for j in (0, i // 2, i):
                assert oracle.kept(art, h, i, j) == M[i, j]


def test_extension_extremes():
    rng = np.random.default_rng(7)
    A = softmax_map(rng, 2, 10)
    S = 37
    tri = np.tril(np.ones((S, S), np.uint8))
    art = oracle.derive(A, None, 0.5, 1e-8, 0.3, 0.0)      # mu = 0: everything matches
    M = oracle.rows(art, 0, S, 0, S)
    outside = np.ones((S, S), bool)
    outside[:10, :10] = False
    # all 2L patterns: every offset < L and every column < L, i.e. dense causal up to S = 2L and an
    # L-wide window plus L sink columns beyond
    ii, jj = np.meshgrid(np.arange(S), np.arange(S), indexing="ij")
    expect = (((ii - jj) < 10) | (jj < 10)) & (jj <= ii)
    assert np.array_equal(M[outside].astype(bool), expect[outside])
    assert np.array_equal(M[:20, :20][outside[:20, :20]], tri[:20, :20][outside[:20, :20]])
    art = oracle.derive(A, None, 0.5, 1e-8, 0.3, 1.5)      # mu > 1: nothing matches
    M = oracle.rows(art, 0, S, 0, S)
    assert M[outside].sum() == 0 and M[10:].sum() == 0
    # patterns only (no true mask): overlap of a diagonal and a column is kept once
    d = np.zeros((1, S), np.uint8)
    v = np.zeros((1, S), np.uint8)
    d[0, 2] = 1
    v[0, 3] = 1
    art = oracle.from_patterns(d, v)
    M = oracle.rows(art, 0, S, 0, S)
    assert M[5, 3] == 1 and M.sum() == (S - 2) + (S - 3) - 1
    assert np.array_equal(oracle.kept_list(art, 0, 5), [3])
    assert np.array_equal(oracle.kept_list(art, 0, 10), [3, 8])


# ---------------------------------------------------------------- block index / tile bits
def expand_tiles(row_ptr, col, kind, bits, S, tm, tn):
    nQt = row_ptr.shape[0] - 1
    nKt = (S + tn - 1) // tn
    dense = np.zeros((nQt * tm, nKt * tn), np.uint8)
    for qt in range(nQt):
        for t in range(row_ptr[qt] - row_ptr[0], row_ptr[qt + 1] - row_ptr[0]):
            words = bits[t]                                  # [tm][tn//64]
            b = ((words[:, :, None] >> np.arange(64, dtype=np.uint64)[None, None, :]) & np.uint64(1))
            dense[qt * tm:(qt + 1) * tm, col[t] * tn:(col[t] + 1) * tn] = b.reshape(tm, tn)
    return dense


@pytest.mark.parametrize("S,tm,tn", [(256, 64, 64), (200, 64, 128), (130, 128, 64), (64, 128, 128)])
def test_block_index_reexpansion(S, tm, tn):
    rng = np.random.default_rng(8)
    art = make_art(rng, H=2, L=48, tau=0.05, mu=0.5)
    row_ptr, col, kind, bits = oracle.block_index(art, S, tm, tn)
    nQt = (S + tm - 1) // tm
    assert row_ptr.shape == (2, nQt + 1) and row_ptr[0, 0] == 0 and row_ptr[1, 0] == row_ptr[0, nQt]
    assert row_ptr[-1, -1] == len(col) == len(kind) == len(bits)
    for h in range(2):
        M = oracle.rows(art, h, S, 0, S)
        lo, hi = row_ptr[h, 0], row_ptr[h, -1]
        dense = expand_tiles(row_ptr[h], col[lo:hi], kind[lo:hi], bits[lo:hi], S, tm, tn)
        assert np.array_equal(dense[:S, :S], M)              # listed tiles reproduce the mask,
        assert dense[S:].sum() == 0 and dense[:, S:].sum() == 0   # unlisted tiles and bits beyond S are 0
        for qt in range(nQt):
            cols = col[row_ptr[h, qt]:row_ptr[h, qt + 1]]
            assert np.all(np.diff(cols) > 0)                 # ascending, no duplicates
        pc = np.array([int(np.unpackbits(bits[t].view(np.uint8)).sum()) for t in range(lo, hi)])
        assert pc.sum() == M.sum() and (pc > 0).all()
        assert np.array_equal(kind[lo:hi] & 1, (pc == tm * tn).astype(np.uint8))
        for t in range(lo, hi):                              # quarter-occupancy bits, from the dense mask
            qt = int(np.searchsorted(row_ptr[h], t, side="right") - 1)
            blk = M[qt * tm:(qt + 1) * tm, col[t] * tn:(col[t] + 1) * tn]
            want = sum((1 << (1 + q)) for q in range(4) if blk[:, q * tn // 4:(q + 1) * tn // 4].any())
            assert (kind[t] & 0x1E) == want and kind[t] < 32


def test_block_index_full_tiles_only_below_diagonal():
    S, t = 512, 64
    d = np.ones((1, S), np.uint8)
    v = np.zeros((1, S), np.uint8)
    art = oracle.from_patterns(d, v)                         # dense causal
    row_ptr, col, kind, bits = oracle.block_index(art, S, t, t)
    n = S // t
    assert len(col) == n * (n + 1) // 2
    for qt in range(n):
        sl = slice(row_ptr[0, qt], row_ptr[0, qt + 1])
        assert np.array_equal(col[sl], np.arange(qt + 1))
        assert np.array_equal(kind[sl] & 1, [1] * qt + [0])  # the diagonal tile is partial
        assert np.all(kind[sl] >> 1 == 15)


# ------------------------------------------------- gathered column tiles (a layout, not a new mask)
@pytest.mark.parametrize("S,tm,tn,L", [(300, 64, 64, 0), (300, 64, 64, 48), (520, 128, 128, 100), (256, 64, 128, 64)])
def test_gathered_block_index_reexpands_to_the_same_mask(S, tm, tn, L):
    """With the matched columns gathered into tiles of their own, scattering the ordinary tiles back by
    position and the gathered tiles back through the column list must give the mask itself, every kept
    entry exactly once."""
    rng = np.random.default_rng(18)
    H = 3
    d = (rng.random((H, S)) < 0.02).astype(np.uint8)
    v = (rng.random((H, S)) < 0.03).astype(np.uint8)
    d[:, :20] = 1
    v[:, :5] = 1
    v[2] = 0                                                  # a head without columns
    tm_ = (rng.random((H, L, L)) < 0.3).astype(np.uint8) * np.tril(np.ones((L, L), np.uint8)) if L else None
    art = oracle.from_patterns(d, v, tm_)
    row_ptr, col, kind, bits = oracle.block_index(art, S, tm, tn, gather=True)
    gptr, gidx = oracle.gathered_columns(art, S, tn)
    nQt, nKt = (S + tm - 1) // tm, (S + tn - 1) // tn
    plain_ptr, plain_col, _, _ = oracle.block_index(art, S, tm, tn)
    for h in range(H):
        M = oracle.rows(art, h, S, 0, S)
        hits = np.zeros((nQt * tm, max(S, nKt * tn)), np.int32)
        cols_h = gidx[gptr[h]:gptr[h + 1]]
        assert len(cols_h) % tn == 0 and np.array_equal(cols_h[cols_h >= 0], np.flatnonzero(v[h]))
        for qt in range(nQt):
            ts = range(row_ptr[h, qt], row_ptr[h, qt + 1])
            assert np.all(np.diff(col[list(ts)]) > 0)
            for t in ts:
                b = np.unpackbits(bits[t].view(np.uint8), bitorder="little").reshape(tm, tn)
                assert b.any()
                assert (kind[t] & 1) == int(b.all())
                assert (kind[t] >> 1) == sum((1 << q) for q in range(4) if b[:, q * tn // 4:(q + 1) * tn // 4].any())
                if col[t] < nKt:
                    hits[qt * tm:(qt + 1) * tm, col[t] * tn:(col[t] + 1) * tn] += b
                else:
                    assert qt * tm >= L                       # gathered tiles only in the pattern region
                    seg = cols_h[(col[t] - nKt) * tn:(col[t] - nKt + 1) * tn]
                    for s_at, c in enumerate(seg):
                        if c >= 0:
                            hits[qt * tm:(qt + 1) * tm, c] += b[:, s_at]
                        else:
                            assert not b[:, s_at].any()
            if qt * tm < L:                                   # tiles touching the true-mask block: the plain listing
                assert np.array_equal(col[row_ptr[h, qt]:row_ptr[h, qt + 1]], plain_col[plain_ptr[h, qt]:plain_ptr[h, qt + 1]])
        assert hits.max() <= 1                                # nothing is counted twice
        assert np.array_equal(hits[:S, :S], M)
        assert hits[S:].sum() == 0 and hits[:, S:].sum() == 0


def test_gathered_tiles_shrink_a_striped_mask():
    # 40 stripe columns scattered over 2000 keys and a short window: plain listing needs one tile per stripe
    # and query tile, the gathered layout one tile per query tile
    S, t = 2048, 128
    d = np.zeros((1, S), np.uint8)
    v = np.zeros((1, S), np.uint8)
    d[0, :64] = 1
    v[0, np.arange(40) * 50] = 1
    art = oracle.from_patterns(d, v)
    plain = oracle.block_index(art, S, t, t)[1]
    gath = oracle.block_index(art, S, t, t, gather=True)[1]
    assert len(gath) < len(plain) // 2
