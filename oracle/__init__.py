"""CPU oracle of the DAM hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``dam_oracle.c`` (plain C, fp32 mask rule, fp64 attention). Only tests,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import this package; the
GPU library and its Python binding never do, and this package imports nothing of theirs.

Paper: arXiv 2506.11104 (Dynamic Attention Mask). Section numbers in the docstrings refer to it.
"""
from __future__ import annotations

import ctypes
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_LIB = None


def _ptr(a: Optional[np.ndarray], ctype):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctype))
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def lib() -> ctypes.CDLL:
    global _LIB
    if _LIB is None:
        # DAM_ORACLE_SANITIZE=1: the AddressSanitizer + UBSan build (the process must have libasan preloaded)
        path = _build.build(force=False, sanitize=os.environ.get("DAM_ORACLE_SANITIZE") == "1")
        _LIB = ctypes.CDLL(path)
        _LIB.dam_oracle_boxcox.restype = ctypes.c_float
        _LIB.dam_oracle_boxcox.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float),
                                           ctypes.c_int32, ctypes.c_int32, ctypes.c_float, ctypes.c_float,
                                           ctypes.POINTER(ctypes.c_float)]
        _LIB.dam_oracle_transform.restype = ctypes.c_float
        _LIB.dam_oracle_transform.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float),
                                              ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                              ctypes.c_float, ctypes.POINTER(ctypes.c_float)]
        _LIB.dam_oracle_true_mask.restype = None
        _LIB.dam_oracle_true_mask.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_int32, ctypes.c_int32,
                                              ctypes.c_float, ctypes.c_float, ctypes.POINTER(ctypes.c_uint8)]
        _LIB.dam_oracle_match.restype = None
        _LIB.dam_oracle_match.argtypes = [ctypes.POINTER(ctypes.c_uint8), ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_float, ctypes.POINTER(ctypes.c_int32),
                                          ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint8),
                                          ctypes.POINTER(ctypes.c_uint8)]
        head = [ctypes.POINTER(ctypes.c_uint8), ctypes.c_int32, ctypes.POINTER(ctypes.c_uint8),
                ctypes.POINTER(ctypes.c_uint8), ctypes.c_int32]
        _LIB.dam_oracle_kept.restype = ctypes.c_int
        _LIB.dam_oracle_kept.argtypes = head + [ctypes.c_int64, ctypes.c_int64]
        _LIB.dam_oracle_rows.restype = None
        _LIB.dam_oracle_rows.argtypes = head + [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                                ctypes.POINTER(ctypes.c_uint8)]
        _LIB.dam_oracle_kept_list.restype = ctypes.c_int64
        _LIB.dam_oracle_kept_list.argtypes = head + [ctypes.c_int64, ctypes.POINTER(ctypes.c_int32),
                                                     ctypes.c_int64]
        _LIB.dam_oracle_block_index.restype = ctypes.c_int64
        _LIB.dam_oracle_block_index.argtypes = head + [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                                       ctypes.c_int64, ctypes.c_int64,
                                                       ctypes.POINTER(ctypes.c_int32),
                                                       ctypes.POINTER(ctypes.c_int32),
                                                       ctypes.POINTER(ctypes.c_uint8),
                                                       ctypes.POINTER(ctypes.c_uint64), ctypes.c_int64]
        _LIB.dam_oracle_block_index_gathered.restype = ctypes.c_int64
        _LIB.dam_oracle_block_index_gathered.argtypes = head + [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                                                ctypes.c_int64, ctypes.c_int64,
                                                                ctypes.POINTER(ctypes.c_int32), ctypes.c_int64,
                                                                ctypes.POINTER(ctypes.c_int32),
                                                                ctypes.POINTER(ctypes.c_int32),
                                                                ctypes.POINTER(ctypes.c_uint8),
                                                                ctypes.POINTER(ctypes.c_uint64), ctypes.c_int64]
        _LIB.dam_oracle_attend_lists.restype = None
        _LIB.dam_oracle_attend_lists.argtypes = [ctypes.POINTER(ctypes.c_float)] * 3 + [
            ctypes.POINTER(ctypes.c_int32), ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64),
            ctypes.POINTER(ctypes.c_int32), ctypes.c_int64, ctypes.c_double, ctypes.POINTER(ctypes.c_double),
            ctypes.POINTER(ctypes.c_double)]
        _LIB.dam_oracle_attend_rows.restype = None
        _LIB.dam_oracle_attend_rows.argtypes = [ctypes.POINTER(ctypes.c_float)] * 3 + [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(ctypes.c_uint8),
            ctypes.c_int32, ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_uint8), ctypes.c_int32,
            ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64), ctypes.c_int64, ctypes.c_double,
            ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        _LIB.dam_oracle_capture.restype = None
        _LIB.dam_oracle_capture.argtypes = [ctypes.POINTER(ctypes.c_float)] * 2 + [
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int64, ctypes.c_double,
            ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
        _LIB.dam_oracle_threads.restype = ctypes.c_int
        _LIB.dam_oracle_threads.argtypes = []
    return _LIB


def threads() -> int:
    """Threads the oracle's parallel loops use."""
    return int(lib().dam_oracle_threads())


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint8)


@dataclass
class MaskArtefact:
    """What is stored per (layer, head) after stage one (Sec. 4.3, "stored matched positions"):
    the L x L true mask and the matched diagonal offsets / columns as flags over 0..P-1."""
    L: int
    P: int
    true_mask: Optional[np.ndarray]   # [H][L][L] u8, None when L == 0
    diag_flag: np.ndarray             # [H][P] u8
    vert_flag: np.ndarray             # [H][P] u8
    diag_cnt: Optional[np.ndarray] = None  # [H][L] i32
    vert_cnt: Optional[np.ndarray] = None
    bmin: Optional[float] = None

    @property
    def H(self) -> int:
        return int(self.diag_flag.shape[0])

    def head_args(self, h: int):
        tm = self.true_mask[h] if self.true_mask is not None else None
        return (_ptr(tm, ctypes.c_uint8), ctypes.c_int32(self.L), _ptr(self.diag_flag[h], ctypes.c_uint8),
                _ptr(self.vert_flag[h], ctypes.c_uint8), ctypes.c_int32(self.P))


def capture(Q, K, L: int, attn_sum: Optional[np.ndarray] = None, attn_cnt: Optional[np.ndarray] = None,
            scale: Optional[float] = None, want_cnt: bool = True):
    """Sec. 4.2.1 / 4.2.2: add the causal attention probabilities of one captured sequence
    (Q [Hq][n][d], K [Hkv][n][d], n <= L) to the statistics A, C [Hq][L][L] (fp32; created as zeros
    when not given). Returns (A, C); C is None when want_cnt is false and none was given."""
    Q, K = _f32(Q), _f32(K)
    Hq, n, d = Q.shape
    Hkv = K.shape[0]
    assert K.shape[1] == n and K.shape[2] == d and Hq % Hkv == 0 and n <= L
    A = np.zeros((Hq, L, L), np.float32) if attn_sum is None else attn_sum
    C = attn_cnt if attn_cnt is not None else (np.zeros((Hq, L, L), np.float32) if want_cnt else None)
    assert A.dtype == np.float32 and A.flags.c_contiguous and A.shape == (Hq, L, L)
    sc = float(scale) if scale else 1.0 / float(np.sqrt(np.float64(d)))
    lib().dam_oracle_capture(_ptr(Q, ctypes.c_float), _ptr(K, ctypes.c_float), Hq, Hkv, n, d, L,
                             ctypes.c_double(sc), _ptr(A, ctypes.c_float), _ptr(C, ctypes.c_float))
    return A, C


def boxcox(attn_sum: np.ndarray, attn_cnt: Optional[np.ndarray], lam: float, eps: float):
    """Sec. 4.2.2: returns (B [H][L][L] f32, bmin). B* = B - bmin is the normalised map."""
    A = _f32(attn_sum)
    H, L, _ = A.shape
    C = _f32(attn_cnt) if attn_cnt is not None else None
    B = np.empty_like(A)
    bmin = lib().dam_oracle_boxcox(_ptr(A, ctypes.c_float), _ptr(C, ctypes.c_float), H, L,
                                   ctypes.c_float(lam), ctypes.c_float(eps), _ptr(B, ctypes.c_float))
    return B, np.float32(bmin)


TRANSFORMS = {"boxcox": 0, "raw_sum": 1, "average": 2, "log": 3, "yeo_johnson": 4, "zscore": 5, "minmax": 6,
              "sqrt": 7, "arcsinh": 8}


def transform(attn_sum: np.ndarray, attn_cnt: Optional[np.ndarray], kind: str, lam: float, eps: float):
    """App. B: one of the nine feature-amplification transforms. Returns (T [H][L][L] f32, tmin);
    T - tmin is the normalised map the threshold of Sec. 4.2.3 is applied to."""
    A = _f32(attn_sum)
    H, L, _ = A.shape
    C = _f32(attn_cnt) if attn_cnt is not None else None
    T = np.empty_like(A)
    tmin = lib().dam_oracle_transform(_ptr(A, ctypes.c_float), _ptr(C, ctypes.c_float), H, L, TRANSFORMS[kind],
                                      ctypes.c_float(lam), ctypes.c_float(eps), _ptr(T, ctypes.c_float))
    return T, np.float32(tmin)


def true_mask(B: np.ndarray, bmin, tau: float) -> np.ndarray:
    """Sec. 4.2.3: m = (B - bmin >= tau) and causal, [H][L][L] u8."""
    B = _f32(B)
    H, L, _ = B.shape
    m = np.empty((H, L, L), dtype=np.uint8)
    lib().dam_oracle_true_mask(_ptr(B, ctypes.c_float), H, L, ctypes.c_float(bmin), ctypes.c_float(tau),
                               _ptr(m, ctypes.c_uint8))
    return m


def match(m: np.ndarray, mu: float):
    """Sec. 4.2.4: (diag_cnt, vert_cnt, diag_flag, vert_flag), each [H][L]."""
    m = _u8(m)
    H, L, _ = m.shape
    dc = np.empty((H, L), np.int32)
    vc = np.empty((H, L), np.int32)
    df = np.empty((H, L), np.uint8)
    vf = np.empty((H, L), np.uint8)
    lib().dam_oracle_match(_ptr(m, ctypes.c_uint8), H, L, ctypes.c_float(mu), _ptr(dc, ctypes.c_int32),
                           _ptr(vc, ctypes.c_int32), _ptr(df, ctypes.c_uint8), _ptr(vf, ctypes.c_uint8))
    return dc, vc, df, vf


def derive(attn_sum, attn_cnt, lam: float, eps: float, tau: float, mu: float,
           bmin_override: Optional[float] = None, kind: str = "boxcox") -> MaskArtefact:
    """Stage one end to end (Sec. 4.2.2 - 4.2.4): statistics at length L -> stored artefact.
    kind selects the transform (App. B); the default is the method's Box-Cox."""
    B, bmin = boxcox(attn_sum, attn_cnt, lam, eps) if kind == "boxcox" else transform(attn_sum, attn_cnt, kind, lam, eps)
    if bmin_override is not None:
        bmin = np.float32(bmin_override)
    m = true_mask(B, bmin, tau)
    dc, vc, df, vf = match(m, mu)
    L = m.shape[1]
    return MaskArtefact(L=L, P=L, true_mask=m, diag_flag=df, vert_flag=vf, diag_cnt=dc, vert_cnt=vc,
                        bmin=float(bmin))


def from_patterns(diag_flag, vert_flag, true_mask_: Optional[np.ndarray] = None) -> MaskArtefact:
    """Artefact from given matched sets (flags over 0..P-1) and an optional true mask."""
    df, vf = _u8(diag_flag), _u8(vert_flag)
    tm = _u8(true_mask_) if true_mask_ is not None else None
    return MaskArtefact(L=0 if tm is None else tm.shape[1], P=df.shape[1], true_mask=tm, diag_flag=df,
                        vert_flag=vf)


def kept(art: MaskArtefact, h: int, i: int, j: int) -> int:
    """Sec. 4.3: entry (i, j) of head h's mask."""
    return int(lib().dam_oracle_kept(*art.head_args(h), i, j))


def rows(art: MaskArtefact, h: int, S: int, i0: int, i1: int) -> np.ndarray:
    """Rows [i0, i1) of head h's S x S mask, [i1-i0][S] u8."""
    out = np.empty((i1 - i0, S), np.uint8)
    lib().dam_oracle_rows(*art.head_args(h), S, i0, i1, _ptr(out, ctypes.c_uint8))
    return out


def kept_list(art: MaskArtefact, h: int, i: int) -> np.ndarray:
    """Kept keys of row i of head h, ascending (i32)."""
    idx = np.empty(i + 1, np.int32)
    n = lib().dam_oracle_kept_list(*art.head_args(h), i, _ptr(idx, ctypes.c_int32), i + 1)
    return idx[:n].copy()


def gathered_columns(art: MaskArtefact, S: int, tile_n: int):
    """The matched columns below S of every head, ascending (the keys the gathered tiles hold):
    (ptr [H + 1] i64, idx i32), each head's stretch padded with -1 to a multiple of tile_n."""
    ptr = [0]
    out = []
    for h in range(art.H):
        cols = [c for c in range(min(S, art.P)) if art.vert_flag[h, c]]
        pad = (-len(cols)) % tile_n
        out.extend(cols + [-1] * pad)
        ptr.append(len(out))
    return np.array(ptr, np.int64), np.array(out, np.int32)


def block_index(art: MaskArtefact, S: int, tile_m: int, tile_n: int, heads: Optional[Sequence[int]] = None,
                want_bits: bool = True, workers: int = 8, qt_range: Optional[Tuple[int, int]] = None,
                gather: bool = False):
    """Block index of the given heads (default all): returns
    (row_ptr [n_heads][nQt+1] i64 with offsets global over the given heads in order,
     col i32 [n_tiles], kind u8 [n_tiles], tile_bits u64 [n_tiles][tile_m][tile_n//64] or None).
    qt_range = (q0, q1) restricts every head to its query-tile rows q0 .. q1-1 (row_ptr then has
    q1 - q0 + 1 entries per head)."""
    heads = list(range(art.H)) if heads is None else list(heads)
    qa, qb = (0, (S + tile_m - 1) // tile_m) if qt_range is None else qt_range
    nQt = qb - qa
    wpr = tile_n // 64
    chunk = max(1, nQt // 64)
    jobs = [(h, q0, min(qb, q0 + chunk)) for h in heads for q0 in range(qa, qb, chunk)]
    gcols = {}
    if gather:   # "gather = True": the layout with the matched columns in tiles of their own (see the C source)
        for h in heads:
            gcols[h] = np.array([c for c in range(min(S, art.P)) if art.vert_flag[h, c]], np.int32)

    def call(h, q0, q1, cnt, col, kind, bits, cap):
        args = art.head_args(h)
        if gather:
            return lib().dam_oracle_block_index_gathered(*args, S, tile_m, tile_n, q0, q1, _ptr(gcols[h], ctypes.c_int32),
                                                         len(gcols[h]), _ptr(cnt, ctypes.c_int32),
                                                         _ptr(col, ctypes.c_int32), _ptr(kind, ctypes.c_uint8),
                                                         _ptr(bits, ctypes.c_uint64), cap)
        return lib().dam_oracle_block_index(*args, S, tile_m, tile_n, q0, q1, _ptr(cnt, ctypes.c_int32),
                                            _ptr(col, ctypes.c_int32), _ptr(kind, ctypes.c_uint8),
                                            _ptr(bits, ctypes.c_uint64), cap)

    nKt = (S + tile_n - 1) // tile_n
    n_gt = {h: (len(gcols[h]) + tile_n - 1) // tile_n for h in heads} if gather else {}

    def run(job):
        # one call with room for every tile the chunk could list (its causal tiles, plus the gathered ones)
        h, q0, q1 = job
        cnt = np.zeros(q1 - q0, np.int32)
        cap = sum(min(nKt, ((qt + 1) * tile_m + tile_n - 1) // tile_n) + n_gt.get(h, 0) for qt in range(q0, q1))
        col = np.empty(cap, np.int32)
        kind = np.empty(cap, np.uint8)
        bits = np.empty((cap, tile_m, wpr), np.uint64) if want_bits else None
        n = call(h, q0, q1, cnt, col, kind, bits, cap)
        assert n <= cap
        return cnt, col[:n].copy(), kind[:n].copy(), bits[:n].copy() if want_bits else None

    with ThreadPoolExecutor(max_workers=workers) as ex:
        res = list(ex.map(run, jobs))
    cnts = np.concatenate([r[0] for r in res]).reshape(len(heads), nQt)
    row_ptr = np.zeros((len(heads), nQt + 1), np.int64)
    flat = np.concatenate([[0], np.cumsum(cnts.reshape(-1), dtype=np.int64)])
    for a in range(len(heads)):
        row_ptr[a] = flat[a * nQt:(a + 1) * nQt + 1]
    col = np.concatenate([r[1] for r in res]) if res else np.empty(0, np.int32)
    kind = np.concatenate([r[2] for r in res]) if res else np.empty(0, np.uint8)
    bits = np.concatenate([r[3] for r in res]) if want_bits else None
    return row_ptr, col, kind, bits


def attend_rows(q_rows, K, V, art: MaskArtefact, Hq: int, heads, rows_, scale: Optional[float] = None):
    """Sec. 3 / 4.3: masked attention of rows (heads[a], rows_[a]). q_rows [n][d] f32 (the query
    vectors of those rows), K, V [Hkv][S][d] f32. Returns (O [n][d] f64, lse [n] f64)."""
    q_rows, K, V = _f32(q_rows), _f32(K), _f32(V)
    Hkv, S, d = K.shape
    n = q_rows.shape[0]
    heads = np.ascontiguousarray(heads, np.int32)
    rows_ = np.ascontiguousarray(rows_, np.int64)
    assert art.H == Hq and heads.shape[0] == n and rows_.shape[0] == n
    sc = float(scale) if scale else 1.0 / float(np.sqrt(np.float64(d)))
    out = np.empty((n, d), np.float64)
    lse = np.empty(n, np.float64)
    tm = art.true_mask if art.true_mask is not None else None
    lib().dam_oracle_attend_rows(_ptr(q_rows, ctypes.c_float), _ptr(K, ctypes.c_float), _ptr(V, ctypes.c_float),
                                 Hq, Hkv, S, d, _ptr(tm, ctypes.c_uint8), art.L,
                                 _ptr(art.diag_flag, ctypes.c_uint8), _ptr(art.vert_flag, ctypes.c_uint8), art.P,
                                 _ptr(heads, ctypes.c_int32), _ptr(rows_, ctypes.c_int64), n,
                                 ctypes.c_double(sc), _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double))
    return out, lse


def attend_prefill(Q, K, V, art: MaskArtefact, scale: Optional[float] = None):
    """All rows of one batch entry: Q [Hq][S][d], K, V [Hkv][S][d] -> (O [Hq][S][d] f64, lse [Hq][S])."""
    Q = _f32(Q)
    Hq, S, d = Q.shape
    heads = np.repeat(np.arange(Hq, dtype=np.int32), S)
    rws = np.tile(np.arange(S, dtype=np.int64), Hq)
    out, lse = attend_rows(Q.reshape(Hq * S, d), K, V, art, Hq, heads, rws, scale)
    return out.reshape(Hq, S, d), lse.reshape(Hq, S)


def attend_lists(q, kcache, vcache, kv_of, kept_ptr, kept_idx, scale: Optional[float] = None):
    """Decode form: q [n][d] f32; caches [n_blocks][T][d] f32; kv_of [n] i32 (cache block per item);
    CSR lists. Returns (O [n][d] f64, lse [n] f64)."""
    q, kcache, vcache = _f32(q), _f32(kcache), _f32(vcache)
    n, d = q.shape
    T = kcache.shape[1]
    kv_of = np.ascontiguousarray(kv_of, np.int32)
    kept_ptr = np.ascontiguousarray(kept_ptr, np.int64)
    kept_idx = np.ascontiguousarray(kept_idx, np.int32)
    sc = float(scale) if scale else 1.0 / float(np.sqrt(np.float64(d)))
    out = np.empty((n, d), np.float64)
    lse = np.empty(n, np.float64)
    lib().dam_oracle_attend_lists(_ptr(q, ctypes.c_float), _ptr(kcache, ctypes.c_float), _ptr(vcache, ctypes.c_float),
                                  _ptr(kv_of, ctypes.c_int32), T, d, _ptr(kept_ptr, ctypes.c_int64),
                                  _ptr(kept_idx, ctypes.c_int32), n, ctypes.c_double(sc),
                                  _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double))
    return out, lse


def group_lists(lists: Sequence[np.ndarray], group: int):
    """Kept lists of one decode row merged per KV head (grouped-query attention: `group` consecutive
    query heads read the K / V rows of one KV head; the mask row of each head is that of Sec. 4.3).
    lists: one ascending key array per query head. Returns (ptr [n_kv + 1] i64, idx i32, member u8):
    the list of a KV head holds every key some head of its group keeps exactly once, as group + 1 runs,
    each ascending: keys kept by two or more of the heads, then keys kept by head 0 of the group only,
    by head 1 only, ...; bit x of member[e] says that head x of the group keeps key idx[e]."""
    assert len(lists) % group == 0 and 1 <= group <= 8
    ptr, idx, member = [0], [], []
    for kv in range(len(lists) // group):
        who = {}
        for x in range(group):
            for j in lists[kv * group + x]:
                who[int(j)] = who.get(int(j), 0) | (1 << x)
        runs = [sorted(j for j, m in who.items() if bin(m).count("1") >= 2)]
        for x in range(group):
            runs.append(sorted(j for j, m in who.items() if m == 1 << x))
        for run in runs:
            idx.extend(run)
            member.extend(who[j] for j in run)
        ptr.append(len(idx))
    return np.array(ptr, np.int64), np.array(idx, np.int32), np.array(member, np.uint8)


def pattern_plan(diag_flag, vert_flag, group: int, S: Optional[int] = None):
    """Merged decode lists that do not depend on the position, for rows of the pattern region (Sec. 4.3: row p
    keeps key j <= p iff p - j is a matched diagonal or j is a matched column). diag_flag, vert_flag: [Hq][P] flags;
    `group` consecutive query heads share a KV head; S: length of the problem (columns >= S do not exist; default P).
    Per KV head the plan lists first every diagonal offset r matched by some head of the group, then every such
    column c, each part in group + 1 runs: patterns of two or more heads, then those of head 0 alone, of head 1
    alone, ... Each run is ascending in the key it stands for at any position: diagonals by descending offset,
    columns by ascending index. An entry's value is -1 - r for a diagonal (it stands for key p - r at position p)
    and c for a column; bit x of its member byte says that head x of the group has the pattern.
    Returns (ptr [n_kv + 1] i64, val i32, member u8, table u8 [n_kv][P]) with table[g][r] = member bits of
    diagonal r: at position p a column entry c serves the heads in member & ~table[g][p - c], the others meet
    key c through their diagonal p - c already (Sec. 4.2.4: overlapping patterns are a union, a key counts once)."""
    df, vf = _u8(diag_flag), _u8(vert_flag)
    Hq, P = df.shape
    assert Hq % group == 0 and 1 <= group <= 8
    n_cols = P if S is None else min(P, S)
    ptr, val, member = [0], [], []
    table = np.zeros((Hq // group, P), np.uint8)
    for g in range(Hq // group):
        for part, flags, limit in (("diag", df, P), ("col", vf, n_cols)):
            who = {}
            for x in range(group):
                for t in range(limit):
                    if flags[g * group + x, t]:
                        who[t] = who.get(t, 0) | (1 << x)
            if part == "diag":
                for r, m in who.items():
                    table[g, r] = m
            down = part == "diag"          # descending offsets are ascending keys
            runs = [sorted((t for t, m in who.items() if bin(m).count("1") >= 2), reverse=down)]
            for x in range(group):
                runs.append(sorted((t for t, m in who.items() if m == 1 << x), reverse=down))
            for run in runs:
                val.extend((-1 - t) if part == "diag" else t for t in run)
                member.extend(who[t] for t in run)
        ptr.append(len(val))
    return np.array(ptr, np.int64), np.array(val, np.int32), np.array(member, np.uint8), table


def plan_row(plan, g: int, x: int, p: int) -> np.ndarray:
    """The keys head x of KV head g keeps at position p according to a pattern plan: the decoding rule stated
    in pattern_plan, ascending."""
    ptr, val, member, table = plan
    P = table.shape[1]
    keys = []
    for e in range(int(ptr[g]), int(ptr[g + 1])):
        v, m = int(val[e]), int(member[e])
        if v < 0:
            j = p + 1 + v                       # p - r
            if j >= 0 and (m >> x) & 1:
                keys.append(j)
        else:
            if v <= p:
                covered = int(table[g, p - v]) if p - v < P else 0
                if ((m & ~covered) >> x) & 1:
                    keys.append(v)
    return np.array(sorted(keys), np.int32)


# ---------------------------------------------------------------------------------------------
@dataclass
class EvictionPlan:
    """Which cached keys a KV head still needs at position p, and where they live in a compacted
    cache (Sec. 2: local patterns allow evicting the cache beyond the attention span; Sec. 4.3: a row
    i of the pattern region keeps key j iff i - j is a matched diagonal or j a matched column)."""
    window: np.ndarray        # [Hkv] i32: W_g = 1 + largest matched diagonal offset of the group's heads (0: none)
    col_ptr: np.ndarray       # [Hkv + 1] i32 offsets into cols
    cols: np.ndarray          # i32: matched columns <= p of the group's heads (union), ascending per group


def eviction_plan(diag_flag, vert_flag, Hkv: int, p: int) -> EvictionPlan:
    """Pattern-only masks (flags over 0..P-1, rows in the pattern region). For the query heads h of KV
    head g: a key j <= p is attended by some row i >= p of some h  iff  j is a matched column of such
    an h, or  p - j <= r for a matched diagonal r of such an h, i.e. j >= p - r_max(g)."""
    df, vf = _u8(diag_flag), _u8(vert_flag)
    Hq, P = df.shape
    G = Hq // Hkv
    window = np.zeros(Hkv, np.int32)
    ptr = np.zeros(Hkv + 1, np.int32)
    cols = []
    for g in range(Hkv):
        rmax = -1
        live_cols = set()
        for h in range(g * G, (g + 1) * G):
            for r in range(P):
                if df[h, r] and r > rmax:
                    rmax = r
            for c in range(min(P, p + 1)):
                if vf[h, c]:
                    live_cols.add(c)
        window[g] = rmax + 1
        cols.extend(sorted(live_cols))
        ptr[g + 1] = len(cols)
    return EvictionPlan(window=window, col_ptr=ptr, cols=np.array(cols, np.int32))


def eviction_slot(plan: EvictionPlan, g: int, j: int) -> int:
    """Row of key j in KV head g's compacted cache: matched columns first, in ascending order, then a
    ring of W_g rows in which key j sits at position j mod W_g (so a key never moves as p advances).
    -1 for a key that is neither a live column nor representable in the ring (W_g = 0)."""
    a, b = int(plan.col_ptr[g]), int(plan.col_ptr[g + 1])
    seg = plan.cols[a:b]
    k = int(np.searchsorted(seg, j))
    if k < len(seg) and seg[k] == j:
        return k
    W = int(plan.window[g])
    return (b - a) + j % W if W > 0 else -1
