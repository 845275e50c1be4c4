"""ctypes binding of libdam.so (the C ABI declared in include/dam.h).

Argument marshalling only: torch supplies device memory and the current HIP stream, every step of
the path runs in the library's kernels. There is no CPU fallback: if the library has not been
built, loading raises.
"""
from __future__ import annotations

import ctypes
import math
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdam.so")

DAM_OK, DAM_ERR_INVALID_ARG, DAM_ERR_UNSUPPORTED, DAM_ERR_WORKSPACE, DAM_ERR_DEVICE = 0, -1, -2, -3, -5
DAM_F32, DAM_BF16 = 0, 1
DAM_FROM_ATTN_MAP, DAM_FROM_PATTERNS = 0, 1
DAM_MASK_SKIP_FULL_TILE_BITS = 1
DAM_MASK_GATHER_COLUMNS = 2
DAM_MASK_GROUP_LISTS = 4
DAM_MASK_PATTERN_PLAN = 8
DAM_ATTN_RUNNING_REFERENCE = 1
TRANSFORMS = {"boxcox": 0, "raw_sum": 1, "average": 2, "log": 3, "yeo_johnson": 4, "zscore": 5, "minmax": 6,
              "sqrt": 7, "arcsinh": 8}

_STATUS = {0: "DAM_OK", -1: "DAM_ERR_INVALID_ARG", -2: "DAM_ERR_UNSUPPORTED", -3: "DAM_ERR_WORKSPACE",
           -5: "DAM_ERR_DEVICE"}


class DamError(RuntimeError):
    def __init__(self, fn: str, status: int):
        super().__init__(f"{fn} returned {_STATUS.get(status, status)}")
        self.status = status


class MaskParams(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("n_maps", ctypes.c_int32), ("pcl", ctypes.c_int32),
                ("seq", ctypes.c_int32), ("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32),
                ("row_begin", ctypes.c_int32), ("row_end", ctypes.c_int32), ("lam", ctypes.c_float),
                ("eps", ctypes.c_float), ("tau", ctypes.c_float), ("mu", ctypes.c_float),
                ("bmin_override", ctypes.c_float), ("flags", ctypes.c_int32),
                ("transform", ctypes.c_int32), ("group", ctypes.c_int32)]


class MaskOut(ctypes.Structure):
    _fields_ = [("true_bits", ctypes.c_void_p), ("diag_cnt", ctypes.c_void_p), ("vert_cnt", ctypes.c_void_p),
                ("diag_flag", ctypes.c_void_p), ("vert_flag", ctypes.c_void_p), ("bmin", ctypes.c_void_p),
                ("blk_row_ptr", ctypes.c_void_p), ("blk_col", ctypes.c_void_p), ("blk_kind", ctypes.c_void_p),
                ("tile_bits", ctypes.c_void_p), ("blk_capacity", ctypes.c_int64), ("blk_total", ctypes.c_void_p),
                ("dense_bits", ctypes.c_void_p), ("kept_ptr", ctypes.c_void_p), ("kept_idx", ctypes.c_void_p),
                ("kept_capacity", ctypes.c_int64), ("kept_total", ctypes.c_void_p), ("gather_idx", ctypes.c_void_p),
                ("gather_cnt", ctypes.c_void_p), ("kept_member", ctypes.c_void_p), ("plan_table", ctypes.c_void_p)]


class AttnParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("hq", ctypes.c_int32), ("hkv", ctypes.c_int32), ("seq", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3), ("v_stride", ctypes.c_int64 * 3),
                ("o_stride", ctypes.c_int64 * 3), ("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32),
                ("gather_rows", ctypes.c_int32), ("flags", ctypes.c_int32)]


class MaskView(ctypes.Structure):
    _fields_ = [("blk_row_ptr", ctypes.c_void_p), ("blk_col", ctypes.c_void_p), ("blk_kind", ctypes.c_void_p),
                ("tile_bits", ctypes.c_void_p), ("gather_idx", ctypes.c_void_p), ("gather_cnt", ctypes.c_void_p),
                ("gather_stride", ctypes.c_int32)]


class DecodeParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("hq", ctypes.c_int32), ("hkv", ctypes.c_int32),
                ("kv_capacity", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("scale", ctypes.c_float), ("q_stride", ctypes.c_int64 * 2), ("kv_stride", ctypes.c_int64 * 3),
                ("o_stride", ctypes.c_int64 * 2), ("shared_lists", ctypes.c_int32)]


class CaptureParams(ctypes.Structure):
    _fields_ = [("hq", ctypes.c_int32), ("hkv", ctypes.c_int32), ("len", ctypes.c_int32), ("pcl", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("q_stride", ctypes.c_int64 * 2), ("k_stride", ctypes.c_int64 * 2)]


class EvictParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("hq", ctypes.c_int32), ("hkv", ctypes.c_int32), ("n_flags", ctypes.c_int32),
                ("pos", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("kv_capacity", ctypes.c_int32), ("compact_capacity", ctypes.c_int32),
                ("kv_stride", ctypes.c_int64 * 3), ("compact_stride", ctypes.c_int64 * 3)]


EXPORTS = ["dam_gather_stride", "dam_kv_evict_workspace", "dam_kv_evict_plan", "dam_kv_compact", "dam_kv_remap_lists", "dam_mask_build_workspace", "dam_mask_build", "dam_capture_workspace", "dam_capture_accumulate",
           "dam_mask_build_from_qk_workspace", "dam_mask_build_from_qk", "dam_sparse_attn_prefill_workspace",
           "dam_sparse_attn_prefill", "dam_sparse_attn_decode_workspace", "dam_sparse_attn_decode",
           "dam_sparse_attn_decode_grouped_workspace", "dam_sparse_attn_decode_grouped",
           "dam_sparse_attn_decode_patterns", "dam_sparse_attn_decode_grouped_static_limit", "dam_sparse_attn_decode_grouped_static", "dam_probe_mfma",
           "dam_probe_stream_read", "dam_version"]

_lib = None


def lib() -> ctypes.CDLL:
    """Load libdam.so; raises if it has not been built (python -m paper_2506_11104_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python paper_2506_11104_amd/build.py` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int64
        L.dam_mask_build_workspace.restype = sz
        L.dam_mask_build_workspace.argtypes = [ctypes.POINTER(MaskParams)]
        L.dam_mask_build.restype = ctypes.c_int
        L.dam_mask_build.argtypes = [ctypes.POINTER(MaskParams), vp, vp, vp, vp, ctypes.POINTER(MaskOut), vp, sz, vp]
        L.dam_capture_workspace.restype = sz
        L.dam_capture_workspace.argtypes = [ctypes.POINTER(CaptureParams)]
        L.dam_capture_accumulate.restype = ctypes.c_int
        L.dam_capture_accumulate.argtypes = [ctypes.POINTER(CaptureParams), vp, vp, vp, vp, vp, sz, vp]
        L.dam_mask_build_from_qk_workspace.restype = sz
        L.dam_mask_build_from_qk_workspace.argtypes = [ctypes.POINTER(MaskParams), ctypes.POINTER(CaptureParams)]
        L.dam_mask_build_from_qk.restype = ctypes.c_int
        L.dam_mask_build_from_qk.argtypes = [ctypes.POINTER(MaskParams), ctypes.POINTER(CaptureParams), vp, vp,
                                             ctypes.POINTER(MaskOut), vp, sz, vp]
        L.dam_sparse_attn_prefill_workspace.restype = sz
        L.dam_sparse_attn_prefill_workspace.argtypes = [ctypes.POINTER(AttnParams)]
        L.dam_sparse_attn_prefill.restype = ctypes.c_int
        L.dam_sparse_attn_prefill.argtypes = [ctypes.POINTER(AttnParams), vp, vp, vp, ctypes.POINTER(MaskView), vp, vp,
                                              vp, sz, vp]
        L.dam_sparse_attn_decode_workspace.restype = sz
        L.dam_sparse_attn_decode_workspace.argtypes = [ctypes.POINTER(DecodeParams), i64]
        L.dam_sparse_attn_decode.restype = ctypes.c_int
        L.dam_sparse_attn_decode.argtypes = [ctypes.POINTER(DecodeParams), vp, vp, vp, vp, vp, i64, vp, vp, vp, sz, vp]
        L.dam_sparse_attn_decode_grouped_workspace.restype = sz
        L.dam_sparse_attn_decode_grouped_workspace.argtypes = [ctypes.POINTER(DecodeParams), i64]
        L.dam_sparse_attn_decode_grouped.restype = ctypes.c_int
        L.dam_sparse_attn_decode_grouped.argtypes = [ctypes.POINTER(DecodeParams), vp, vp, vp, vp, vp, vp, i64, vp, vp,
                                                     vp, sz, vp]
        L.dam_sparse_attn_decode_patterns.restype = ctypes.c_int
        L.dam_sparse_attn_decode_patterns.argtypes = [ctypes.POINTER(DecodeParams), vp, vp, vp, vp, vp, vp, vp,
                                                      ctypes.c_int32, ctypes.c_int32, i64, vp, vp, vp, sz, vp]
        L.dam_sparse_attn_decode_grouped_static_limit.restype = sz
        L.dam_sparse_attn_decode_grouped_static_limit.argtypes = []
        L.dam_sparse_attn_decode_grouped_static.restype = ctypes.c_int
        L.dam_sparse_attn_decode_grouped_static.argtypes = [ctypes.POINTER(DecodeParams), vp, vp, vp, vp, vp, vp, i64, vp,
                                                            vp, vp]
        L.dam_gather_stride.restype = ctypes.c_int32
        L.dam_gather_stride.argtypes = [ctypes.POINTER(MaskParams)]
        L.dam_kv_evict_workspace.restype = sz
        L.dam_kv_evict_workspace.argtypes = [ctypes.POINTER(EvictParams)]
        L.dam_kv_evict_plan.restype = ctypes.c_int
        L.dam_kv_evict_plan.argtypes = [ctypes.POINTER(EvictParams), vp, vp, vp, vp, vp, i64, vp, vp, vp, sz, vp]
        L.dam_kv_compact.restype = ctypes.c_int
        L.dam_kv_compact.argtypes = [ctypes.POINTER(EvictParams), vp, vp, vp, vp, vp, vp, vp, vp]
        L.dam_kv_remap_lists.restype = ctypes.c_int
        L.dam_kv_remap_lists.argtypes = [ctypes.POINTER(EvictParams), vp, vp, vp, vp, vp, vp, vp]
        L.dam_probe_mfma.restype = ctypes.c_int
        L.dam_probe_mfma.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp]
        L.dam_probe_stream_read.restype = ctypes.c_int
        L.dam_probe_stream_read.argtypes = [vp, sz, vp, ctypes.c_int32, vp]
        L.dam_version.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(fn: str, st: int):
    if st != DAM_OK:
        raise DamError(fn, st)


# ---------------------------------------------------------------------------------------------
@dataclass
class Mask:
    """Device buffers written by dam_mask_build for H heads at problem length S."""
    H: int
    L: int
    S: int
    tile_m: int
    tile_n: int
    true_bits: Optional[torch.Tensor] = None   # [H][L][ceil(L/64)] i64 (bit patterns of u64)
    diag_cnt: Optional[torch.Tensor] = None
    vert_cnt: Optional[torch.Tensor] = None
    diag_flag: Optional[torch.Tensor] = None
    vert_flag: Optional[torch.Tensor] = None
    bmin: Optional[torch.Tensor] = None
    blk_row_ptr: Optional[torch.Tensor] = None  # [H][nQt+1] i32
    blk_col: Optional[torch.Tensor] = None
    blk_kind: Optional[torch.Tensor] = None
    tile_bits: Optional[torch.Tensor] = None    # [n_tiles][tile_m][tile_n/64] i64
    n_tiles: int = 0
    dense_bits: Optional[torch.Tensor] = None
    kept_ptr: Optional[torch.Tensor] = None
    kept_idx: Optional[torch.Tensor] = None
    kept_member: Optional[torch.Tensor] = None  # u8 beside kept_idx (DAM_MASK_GROUP_LISTS)
    plan_table: Optional[torch.Tensor] = None   # u8 [H / group][P] (DAM_MASK_PATTERN_PLAN)
    n_kept: int = 0
    gather_idx: Optional[torch.Tensor] = None   # [H][gather_stride] i32 (DAM_MASK_GATHER_COLUMNS)
    gather_cnt: Optional[torch.Tensor] = None   # [H] i32
    gather_rows: int = 0                        # largest padded column count of a head: rows of the gathered K / V

    def view(self) -> MaskView:
        return MaskView(_p(self.blk_row_ptr), _p(self.blk_col), _p(self.blk_kind), _p(self.tile_bits),
                        _p(self.gather_idx), _p(self.gather_cnt),
                        0 if self.gather_idx is None else self.gather_idx.shape[1])


def mask_workspace(params: MaskParams, device) -> torch.Tensor:
    n = lib().dam_mask_build_workspace(ctypes.byref(params))
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def dam_mask_build(params: MaskParams, attn_sum, attn_cnt, diag_in, vert_in, out: MaskOut, ws: torch.Tensor) -> None:
    """Raw call: enqueues on torch's current stream; raises DamError on a non-zero status."""
    st = lib().dam_mask_build(ctypes.byref(params), _p(attn_sum), _p(attn_cnt), _p(diag_in), _p(vert_in),
                              ctypes.byref(out), _p(ws), ws.numel(), _stream())
    _check("dam_mask_build", st)


def capture_params(q: torch.Tensor, k: torch.Tensor, L: int, scale: float = 0.0) -> CaptureParams:
    """q [Hq][n][d], k [Hkv][n][d] (d contiguous): one captured sequence of n <= L tokens."""
    Hq, n, d = q.shape
    assert k.shape[1] == n and k.shape[2] == d and q.stride(2) == 1 and k.stride(2) == 1
    p = CaptureParams()
    p.hq, p.hkv, p.len, p.pcl, p.head_dim, p.dtype, p.scale = Hq, k.shape[0], n, L, d, _dtype_code(q), scale
    p.q_stride = (ctypes.c_int64 * 2)(*q.stride()[:2])
    p.k_stride = (ctypes.c_int64 * 2)(*k.stride()[:2])
    return p


def capture_workspace(p: CaptureParams, device) -> torch.Tensor:
    n = lib().dam_capture_workspace(ctypes.byref(p))
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def dam_capture_accumulate(q, k, attn_sum, attn_cnt=None, scale: float = 0.0, ws=None) -> None:
    """attn_sum (and attn_cnt) [Hq][L][L] f32 += the causal attention probabilities (the valid pairs)
    of the captured sequence q [Hq][n][d], k [Hkv][n][d]."""
    p = capture_params(q, k, attn_sum.shape[1], scale)
    if ws is None:
        ws = capture_workspace(p, q.device)
    st = lib().dam_capture_accumulate(ctypes.byref(p), _p(q), _p(k), _p(attn_sum), _p(attn_cnt), _p(ws), ws.numel(),
                                      _stream())
    _check("dam_capture_accumulate", st)


def mask_from_qk_workspace(params: MaskParams, cp: CaptureParams, device) -> torch.Tensor:
    n = lib().dam_mask_build_from_qk_workspace(ctypes.byref(params), ctypes.byref(cp))
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def dam_mask_build_from_qk(params: MaskParams, cp: CaptureParams, q, k, out: MaskOut, ws: torch.Tensor) -> None:
    st = lib().dam_mask_build_from_qk(ctypes.byref(params), ctypes.byref(cp), _p(q), _p(k), ctypes.byref(out), _p(ws),
                                      ws.numel(), _stream())
    _check("dam_mask_build_from_qk", st)


def build_mask(*, mode: int, H: int, L: int, S: int, tile_m: int = 128, tile_n: int = 128, lam: float = 0.5,
               eps: float = 1e-8, tau: float = 0.3, mu: float = 0.8, bmin_override: float = float("nan"),
               attn_sum: Optional[torch.Tensor] = None, attn_cnt: Optional[torch.Tensor] = None,
               diag_in: Optional[torch.Tensor] = None, vert_in: Optional[torch.Tensor] = None,
               true_bits: Optional[torch.Tensor] = None, blocks: bool = True, tile_bits: bool = True,
               dense: bool = False, rows: Optional[Tuple[int, int]] = None, device="cuda",
               qk: Optional[Tuple[torch.Tensor, torch.Tensor]] = None, scale: float = 0.0, flags: int = 0, transform: int = 0,
               group: int = 0, plan: bool = False) -> Mask:
    """Convenience wrapper: allocates the outputs, sizes the tile pool / kept lists with a first
    call (blk_col == NULL), then fills them with a second. Only allocation and marshalling.
    qk = (q [H][L][d], k [Hkv][L][d]) selects dam_mask_build_from_qk (one captured sequence, no map).
    group > 0 sets DAM_MASK_GROUP_LISTS: rows must name one row; kept_ptr has H / group + 1 entries.
    plan = True (with group > 0) sets DAM_MASK_PATTERN_PLAN: position-independent lists and plan_table, no rows."""
    if group > 0:
        flags |= DAM_MASK_GROUP_LISTS
    if plan:
        assert group > 0 and not rows
        flags |= DAM_MASK_PATTERN_PLAN
    dev = torch.device(device)
    p = MaskParams(mode, H, L, S, tile_m, tile_n, rows[0] if rows else 0, rows[1] if rows else 0, lam, eps, tau, mu,
                   bmin_override, flags, transform, group)
    if qk is not None:
        cp = capture_params(qk[0], qk[1], L, scale)
        ws = mask_from_qk_workspace(p, cp, dev)

        def call(o):
            dam_mask_build_from_qk(p, cp, qk[0], qk[1], o, ws)
    else:
        ws = mask_workspace(p, dev)

        def call(o):
            dam_mask_build(p, attn_sum, attn_cnt, diag_in, vert_in, o, ws)
    m = Mask(H=H, L=L, S=S, tile_m=tile_m, tile_n=tile_n)
    nQt = (S + tile_m - 1) // tile_m
    if mode == DAM_FROM_ATTN_MAP:
        m.true_bits = torch.empty((H, L, (L + 63) // 64), dtype=torch.int64, device=dev)
        m.diag_cnt = torch.empty((H, L), dtype=torch.int32, device=dev)
        m.vert_cnt = torch.empty((H, L), dtype=torch.int32, device=dev)
        m.diag_flag = torch.empty((H, L), dtype=torch.uint8, device=dev)
        m.vert_flag = torch.empty((H, L), dtype=torch.uint8, device=dev)
        m.bmin = torch.empty(1, dtype=torch.float32, device=dev)
    else:
        m.true_bits = true_bits
        m.diag_flag, m.vert_flag = diag_in, vert_in
    totals = torch.zeros(2, dtype=torch.int64, device=dev)
    o = MaskOut()
    o.true_bits = _p(m.true_bits)
    if mode == DAM_FROM_ATTN_MAP:
        o.diag_cnt, o.vert_cnt, o.diag_flag, o.vert_flag, o.bmin = (_p(m.diag_cnt), _p(m.vert_cnt), _p(m.diag_flag),
                                                                    _p(m.vert_flag), _p(m.bmin))
    if flags & DAM_MASK_GATHER_COLUMNS:
        m.gather_idx = torch.empty((H, lib().dam_gather_stride(ctypes.byref(p))), dtype=torch.int32, device=dev)
        m.gather_cnt = torch.empty(H, dtype=torch.int32, device=dev)
        o.gather_idx, o.gather_cnt = _p(m.gather_idx), _p(m.gather_cnt)
    if blocks:
        m.blk_row_ptr = torch.empty((H, nQt + 1), dtype=torch.int32, device=dev)
        o.blk_row_ptr, o.blk_total = _p(m.blk_row_ptr), totals[0:1].data_ptr()
    if rows or plan:
        n_lists = H // group if group > 0 else H * (rows[1] - rows[0])
        m.kept_ptr = torch.empty(n_lists + 1, dtype=torch.int32, device=dev)
        o.kept_ptr, o.kept_total = _p(m.kept_ptr), totals[1:2].data_ptr()
    if plan:
        m.plan_table = torch.empty((H // group, L if mode == DAM_FROM_ATTN_MAP else S), dtype=torch.uint8, device=dev)
        o.plan_table = _p(m.plan_table)
    if dense:
        m.dense_bits = torch.empty((H, S, (S + 63) // 64), dtype=torch.int64, device=dev)
        o.dense_bits = _p(m.dense_bits)
    call(o)
    if m.gather_cnt is not None:
        m.gather_rows = (int(m.gather_cnt.max().item()) + tile_n - 1) // tile_n * tile_n
    if blocks or rows or plan:
        n_tiles, n_kept = (int(x) for x in totals.cpu())
        again = False
        if blocks and n_tiles > 0:
            m.n_tiles = n_tiles
            m.blk_col = torch.empty(n_tiles, dtype=torch.int32, device=dev)
            m.blk_kind = torch.empty(n_tiles, dtype=torch.uint8, device=dev)
            o.blk_col, o.blk_kind, o.blk_capacity = _p(m.blk_col), _p(m.blk_kind), n_tiles
            if tile_bits:
                m.tile_bits = torch.empty((n_tiles, tile_m, tile_n // 64), dtype=torch.int64, device=dev)
                o.tile_bits = _p(m.tile_bits)
            again = True
        elif blocks:
            m.blk_col = torch.empty(1, dtype=torch.int32, device=dev)
            m.blk_kind = torch.empty(1, dtype=torch.uint8, device=dev)
            m.tile_bits = torch.empty((1, tile_m, tile_n // 64), dtype=torch.int64, device=dev)
        if (rows or plan) and n_kept > 0:
            m.n_kept = n_kept
            m.kept_idx = torch.empty(n_kept, dtype=torch.int32, device=dev)
            o.kept_idx, o.kept_capacity = _p(m.kept_idx), n_kept
            if group > 0:
                m.kept_member = torch.empty(n_kept, dtype=torch.uint8, device=dev)
                o.kept_member = _p(m.kept_member)
            again = True
        if again:
            o.dense_bits = None
            call(o)
    return m


# ---------------------------------------------------------------------------------------------
def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DAM_F32
    if t.dtype == torch.bfloat16:
        return DAM_BF16
    raise DamError("dtype", DAM_ERR_UNSUPPORTED)


def attn_params(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, o: torch.Tensor, tile_m: int, tile_n: int,
                scale: float = 0.0, gather_rows: int = 0, flags: int = 0) -> AttnParams:
    B, Hq, S, d = q.shape
    p = AttnParams()
    p.batch, p.hq, p.hkv, p.seq, p.head_dim = B, Hq, k.shape[1], S, d
    p.dtype, p.scale, p.tile_m, p.tile_n, p.gather_rows, p.flags = _dtype_code(q), scale, tile_m, tile_n, gather_rows, flags
    for name, t in (("q_stride", q), ("k_stride", k), ("v_stride", v), ("o_stride", o)):
        assert t.stride(3) == 1
        setattr(p, name, (ctypes.c_int64 * 3)(*t.stride()[:3]))
    return p


def prefill_workspace(p: AttnParams, device) -> torch.Tensor:
    n = lib().dam_sparse_attn_prefill_workspace(ctypes.byref(p))
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def dam_sparse_attn_prefill(q, k, v, mask: Mask, out=None, lse=None, scale: float = 0.0, ws=None,
                            want_lse: bool = False, flags: int = 0):
    """q [B][Hq][S][d], k, v [B][Hkv][S][d] (d contiguous) -> out like q (and lse [B][Hq][S] f32)."""
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    p = attn_params(q, k, v, out, mask.tile_m, mask.tile_n, scale, mask.gather_rows, flags)
    if ws is None:
        ws = prefill_workspace(p, q.device)
    mv = mask.view()
    st = lib().dam_sparse_attn_prefill(ctypes.byref(p), _p(q), _p(k), _p(v), ctypes.byref(mv), _p(out), _p(lse),
                                       _p(ws), ws.numel(), _stream())
    _check("dam_sparse_attn_prefill", st)
    return (out, lse) if (want_lse or lse is not None) else out


def decode_params(q: torch.Tensor, kc: torch.Tensor, out: torch.Tensor, scale: float = 0.0,
                  shared_lists: bool = False) -> DecodeParams:
    B, Hq, d = q.shape
    p = DecodeParams()
    p.batch, p.hq, p.hkv, p.kv_capacity, p.head_dim = B, Hq, kc.shape[1], kc.shape[2], d
    p.dtype, p.scale = _dtype_code(q), scale
    p.q_stride = (ctypes.c_int64 * 2)(*q.stride()[:2])
    p.kv_stride = (ctypes.c_int64 * 3)(*kc.stride()[:3])
    p.o_stride = (ctypes.c_int64 * 2)(*out.stride()[:2])
    p.shared_lists = 1 if shared_lists else 0
    return p


def decode_workspace(p: DecodeParams, max_kept: int, device) -> torch.Tensor:
    n = lib().dam_sparse_attn_decode_workspace(ctypes.byref(p), max_kept)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def dam_sparse_attn_decode(q, kcache, vcache, kept_ptr, kept_idx, max_kept: int, out=None, lse=None,
                           scale: float = 0.0, ws=None, want_lse: bool = False, shared_lists: bool = False):
    """q [B][Hq][d]; caches [B][Hkv][cap][d] with identical strides; CSR kept lists per (b, hq), or per
    head for the whole batch with shared_lists."""
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    assert kcache.stride() == vcache.stride()
    p = decode_params(q, kcache, out, scale, shared_lists)
    if ws is None:
        ws = decode_workspace(p, max_kept, q.device)
    st = lib().dam_sparse_attn_decode(ctypes.byref(p), _p(q), _p(kcache), _p(vcache), _p(kept_ptr), _p(kept_idx),
                                      max_kept, _p(out), _p(lse), _p(ws), ws.numel(), _stream())
    _check("dam_sparse_attn_decode", st)
    return (out, lse) if (want_lse or lse is not None) else out


def decode_grouped_workspace(p: DecodeParams, max_kept: int, device) -> torch.Tensor:
    n = lib().dam_sparse_attn_decode_grouped_workspace(ctypes.byref(p), max_kept)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)


def dam_sparse_attn_decode_grouped(q, kcache, vcache, kept_ptr, kept_idx, kept_member, max_kept: int, out=None,
                                   lse=None, scale: float = 0.0, ws=None, want_lse: bool = False,
                                   shared_lists: bool = False):
    """As dam_sparse_attn_decode, with one merged list per (b, KV head) (per KV head with shared_lists) and
    a byte of member bits per entry (dam_mask_build with DAM_MASK_GROUP_LISTS)."""
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    assert kcache.stride() == vcache.stride()
    p = decode_params(q, kcache, out, scale, shared_lists)
    if ws is None:
        ws = decode_grouped_workspace(p, max_kept, q.device)
    st = lib().dam_sparse_attn_decode_grouped(ctypes.byref(p), _p(q), _p(kcache), _p(vcache), _p(kept_ptr),
                                              _p(kept_idx), _p(kept_member), max_kept, _p(out), _p(lse), _p(ws),
                                              ws.numel(), _stream())
    _check("dam_sparse_attn_decode_grouped", st)
    return (out, lse) if (want_lse or lse is not None) else out


def dam_sparse_attn_decode_patterns(q, kcache, vcache, plan: "Mask", pos: int, max_entries: int, out=None, lse=None,
                                    scale: float = 0.0, ws=None, want_lse: bool = False):
    """Grouped decode at position pos from a position-independent plan (build_mask(..., group=G, plan=True))."""
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    assert kcache.stride() == vcache.stride()
    p = decode_params(q, kcache, out, scale, True)
    if ws is None:
        ws = decode_grouped_workspace(p, max_entries, q.device)
    st = lib().dam_sparse_attn_decode_patterns(ctypes.byref(p), _p(q), _p(kcache), _p(vcache), _p(plan.kept_ptr),
                                               _p(plan.kept_idx), _p(plan.kept_member), _p(plan.plan_table),
                                               plan.plan_table.shape[1], pos, max_entries, _p(out), _p(lse), _p(ws),
                                               ws.numel(), _stream())
    _check("dam_sparse_attn_decode_patterns", st)
    return (out, lse) if (want_lse or lse is not None) else out


def dam_sparse_attn_decode_grouped_static(q, kcache, vcache, kept_ptr, kept_idx, kept_member, max_kept: int, out,
                                          lse=None, scale: float = 0.0, shared_lists: bool = False) -> None:
    """dam_sparse_attn_decode_grouped without a workspace: the library's fixed scratch array holds the partial
    results. The caller passes every buffer (out, lse): this wrapper allocates nothing either."""
    assert kcache.stride() == vcache.stride()
    p = decode_params(q, kcache, out, scale, shared_lists)
    st = lib().dam_sparse_attn_decode_grouped_static(ctypes.byref(p), _p(q), _p(kcache), _p(vcache), _p(kept_ptr),
                                                     _p(kept_idx), _p(kept_member), max_kept, _p(out), _p(lse), _stream())
    _check("dam_sparse_attn_decode_grouped_static", st)


# ---------------------------------------------------------------------------------------------
@dataclass
class EvictionPlan:
    """Device buffers written by dam_kv_evict_plan."""
    params: EvictParams
    window: torch.Tensor      # [hkv] i32
    col_ptr: torch.Tensor     # [hkv + 1] i32
    cols: torch.Tensor        # [n_cols] i32 (at least one element is allocated)
    rows: torch.Tensor        # [hkv] i32: rows the compacted cache of each KV head needs
    n_cols: int


def kv_evict_plan(diag_flag: torch.Tensor, vert_flag: torch.Tensor, hkv: int, pos: int, batch: int = 1) -> EvictionPlan:
    """Two calls: size the column list, then fill it. diag_flag, vert_flag u8 [hq][P] on the device."""
    hq, P = diag_flag.shape
    dev = diag_flag.device
    p = EvictParams()
    p.batch, p.hq, p.hkv, p.n_flags, p.pos = batch, hq, hkv, P, pos
    n = lib().dam_kv_evict_workspace(ctypes.byref(p))
    ws = torch.empty(max(n, 256), dtype=torch.uint8, device=dev)
    window = torch.empty(hkv, dtype=torch.int32, device=dev)
    col_ptr = torch.empty(hkv + 1, dtype=torch.int32, device=dev)
    rows = torch.empty(hkv, dtype=torch.int32, device=dev)
    total = torch.zeros(1, dtype=torch.int64, device=dev)

    def call(cols, cap):
        st = lib().dam_kv_evict_plan(ctypes.byref(p), _p(diag_flag), _p(vert_flag), _p(window), _p(col_ptr), _p(cols), cap,
                                     _p(rows), _p(total), _p(ws), ws.numel(), _stream())
        _check("dam_kv_evict_plan", st)

    call(None, 0)
    n_cols = int(total.item())
    cols = torch.empty(max(n_cols, 1), dtype=torch.int32, device=dev)
    if n_cols:
        call(cols, n_cols)
    return EvictionPlan(p, window, col_ptr, cols, rows, n_cols)


def kv_compact(plan: EvictionPlan, kcache: torch.Tensor, vcache: torch.Tensor, kcompact: torch.Tensor,
               vcompact: torch.Tensor) -> None:
    """caches [B][Hkv][cap][d], compacted caches [B][Hkv][ccap][d] (d contiguous, K and V alike)."""
    assert kcache.stride() == vcache.stride() and kcompact.stride() == vcompact.stride()
    p = plan.params
    p.batch, p.head_dim, p.dtype = kcache.shape[0], kcache.shape[3], _dtype_code(kcache)
    p.kv_capacity, p.compact_capacity = kcache.shape[2], kcompact.shape[2]
    p.kv_stride = (ctypes.c_int64 * 3)(*kcache.stride()[:3])
    p.compact_stride = (ctypes.c_int64 * 3)(*kcompact.stride()[:3])
    st = lib().dam_kv_compact(ctypes.byref(p), _p(plan.window), _p(plan.col_ptr), _p(plan.cols), _p(kcache), _p(vcache),
                              _p(kcompact), _p(vcompact), _stream())
    _check("dam_kv_compact", st)


def kv_remap_lists(plan: EvictionPlan, kept_ptr: torch.Tensor, kept_idx: torch.Tensor, batch: int,
                   out: Optional[torch.Tensor] = None, per_kv_head: bool = False) -> torch.Tensor:
    """per_kv_head: the lists are the merged ones of the grouped-query decode, one per (sequence, KV head)."""
    if out is None:
        out = torch.empty_like(kept_idx)
    p = plan.params
    if per_kv_head:
        p = EvictParams.from_buffer_copy(plan.params)
        p.hq = p.hkv
    p.batch = batch
    st = lib().dam_kv_remap_lists(ctypes.byref(p), _p(plan.window), _p(plan.col_ptr), _p(plan.cols), _p(kept_ptr),
                                  _p(kept_idx), _p(out), _stream())
    _check("dam_kv_remap_lists", st)
    return out


# ---------------------------------------------------------------------------------------------
def probe_mfma(operands: torch.Tensor, sink: torch.Tensor, workgroups: int, iters: int) -> float:
    """Enqueues the matrix-instruction probe; returns the flop it launches."""
    assert operands.numel() * operands.element_size() >= 8192
    st = lib().dam_probe_mfma(_p(operands), _p(sink), workgroups, iters, _stream())
    _check("dam_probe_mfma", st)
    return workgroups * 4.0 * iters * 16 * 32768


def probe_stream_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int) -> int:
    """Enqueues the streaming-read probe over the whole tensor; returns the bytes it reads."""
    nbytes = src.numel() * src.element_size()
    st = lib().dam_probe_stream_read(_p(src), nbytes, _p(sink), workgroups, _stream())
    _check("dam_probe_stream_read", st)
    return nbytes
