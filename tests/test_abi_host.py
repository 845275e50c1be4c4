"""Host-side checks that need no GPU: the library loads, exports every function the header
declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2506_11104_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "dam.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dam_[a-z_]+)\s*\(", src)))


def test_status_codes_of_the_header_and_the_binding_agree():
    """Every status the header's enum names, with its value, is what the binding holds; -4 names nothing (a capacity
    overflow is reported through the device totals and the clamped offsets, never through the return value)."""
    src = open(os.path.join(ROOT, "include", "dam.h")).read()
    enum = src[src.index("typedef enum {\n  DAM_OK"):src.index("} dam_status;")]
    enum = re.sub(r"/\*.*?\*/", "", enum, flags=re.S)
    codes = {n: int(v) for n, v in re.findall(r"(DAM_[A-Z_]+)\s*=\s*(-?\d+)", enum)}
    assert codes == {"DAM_OK": 0, "DAM_ERR_INVALID_ARG": -1, "DAM_ERR_UNSUPPORTED": -2, "DAM_ERR_WORKSPACE": -3,
                     "DAM_ERR_DEVICE": -5}
    for n, v in codes.items():
        assert getattr(B, n) == v
    assert -4 not in B._STATUS and not hasattr(B, "DAM_ERR_CAPACITY")


def test_every_declared_symbol_is_exported():
    L = B.lib()
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None
    assert L.dam_version() >= 1


def mask_params(**kw):
    d = dict(mode=B.DAM_FROM_ATTN_MAP, n_maps=2, pcl=64, seq=256, tile_m=64, tile_n=64, row_begin=0, row_end=0, lam=0.5,
             eps=1e-8, tau=0.3, mu=0.8, bmin_override=float("nan"), flags=0, transform=0)
    d.update(kw)
    return B.MaskParams(*d.values())


def call_mask(p, attn=4096, diag=None, vert=None, out=None, ws=4096, ws_bytes=1 << 30):
    o = out or B.MaskOut()
    if out is None:
        o.true_bits = 4096
    return B.lib().dam_mask_build(ctypes.byref(p), attn, None, diag, vert, ctypes.byref(o), ws, ws_bytes, None)


def test_mask_build_argument_errors():
    L = B.lib()
    assert L.dam_mask_build(None, None, None, None, None, None, None, 0, None) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(), attn=None) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(n_maps=0)) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(pcl=0)) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(tile_n=96)) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(tile_m=512)) == B.DAM_ERR_UNSUPPORTED
    assert call_mask(mask_params(eps=0.0)) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(lam=0.3)) == B.DAM_ERR_UNSUPPORTED      # bit-exactness is unpinned for powf
    assert call_mask(mask_params(lam=0.0)) == B.DAM_ERR_UNSUPPORTED
    assert call_mask(mask_params(), ws_bytes=16) == B.DAM_ERR_WORKSPACE
    assert call_mask(mask_params(), ws=None) == B.DAM_ERR_WORKSPACE
    assert call_mask(mask_params(mode=7)) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(transform=9)) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(transform=-1)) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(flags=2)) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(mode=B.DAM_FROM_PATTERNS, pcl=0), attn=None) == B.DAM_ERR_INVALID_ARG  # no flags
    o = B.MaskOut()
    o.true_bits, o.blk_col = 4096, 4096                                   # block output without row_ptr / total
    assert call_mask(mask_params(), out=o) == B.DAM_ERR_INVALID_ARG
    o = B.MaskOut()
    o.true_bits, o.kept_ptr, o.kept_total = 4096, 4096, 4096
    assert call_mask(mask_params(row_begin=5, row_end=3), out=o) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(row_begin=0, row_end=257), out=o) == B.DAM_ERR_INVALID_ARG
    # merged lists for grouped-query decoding: group size, one row only, member bytes beside the indices
    GL = B.DAM_MASK_GROUP_LISTS
    assert call_mask(mask_params(flags=GL, group=0, row_begin=3, row_end=4), out=o) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(flags=GL, group=9, row_begin=3, row_end=4), out=o) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(flags=GL, group=2, row_begin=3, row_end=5), out=o) == B.DAM_ERR_UNSUPPORTED
    assert call_mask(mask_params(flags=GL, group=2, n_maps=3, row_begin=3, row_end=4), out=o) == B.DAM_ERR_INVALID_ARG
    o.kept_idx, o.kept_capacity = 4096, 10
    assert call_mask(mask_params(flags=GL, group=2, n_maps=4, row_begin=3, row_end=4), out=o) == B.DAM_ERR_INVALID_ARG
    assert call_mask(mask_params(flags=8)) == B.DAM_ERR_INVALID_ARG
    assert L.dam_mask_build_workspace(ctypes.byref(mask_params())) > 0
    assert L.dam_mask_build_workspace(ctypes.byref(mask_params(seq=0))) == 0


def attn_params(**kw):
    p = B.AttnParams()
    p.batch, p.hq, p.hkv, p.seq, p.head_dim, p.dtype, p.scale, p.tile_m, p.tile_n = 1, 4, 2, 256, 128, B.DAM_BF16, 0.0, 128, 128
    for n in ("q_stride", "k_stride", "v_stride", "o_stride"):
        setattr(p, n, (ctypes.c_int64 * 3)(4 * 256 * 128, 256 * 128, 128))
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def call_prefill(p, q=4096, mv=None, ws=4096, ws_bytes=1 << 40):
    mv = mv or B.MaskView(4096, 4096, 4096, 4096)
    return B.lib().dam_sparse_attn_prefill(ctypes.byref(p), q, 4096, 4096, ctypes.byref(mv), 4096, None, ws, ws_bytes, None)


def test_prefill_argument_errors():
    assert call_prefill(attn_params(), q=None) == B.DAM_ERR_INVALID_ARG
    assert call_prefill(attn_params(hq=3)) == B.DAM_ERR_INVALID_ARG                  # hq % hkv != 0
    assert call_prefill(attn_params(head_dim=96)) == B.DAM_ERR_UNSUPPORTED
    assert call_prefill(attn_params(tile_m=64)) == B.DAM_ERR_UNSUPPORTED             # bf16 kernel: 128 x 128 only
    assert call_prefill(attn_params(dtype=5)) == B.DAM_ERR_UNSUPPORTED
    assert call_prefill(attn_params(scale=-1.0)) == B.DAM_ERR_INVALID_ARG
    assert call_prefill(attn_params(), mv=B.MaskView(4096, None, 4096, 4096)) == B.DAM_ERR_INVALID_ARG
    assert call_prefill(attn_params(q_stride=(ctypes.c_int64 * 3)(0, 0, 130))) == B.DAM_ERR_INVALID_ARG  # unaligned rows
    # a zero tile size with gathered tiles present: rejected, not divided by
    gath = B.MaskView(4096, 4096, 4096, 4096, 4096, 4096, 128)
    assert call_prefill(attn_params(tile_n=0, gather_rows=128), mv=gath) == B.DAM_ERR_INVALID_ARG
    assert call_prefill(attn_params(tile_m=0, tile_n=0, gather_rows=128), mv=gath) == B.DAM_ERR_INVALID_ARG
    assert call_prefill(attn_params(gather_rows=100), mv=gath) == B.DAM_ERR_INVALID_ARG   # not a multiple of tile_n
    assert call_prefill(attn_params(gather_rows=128)) == B.DAM_ERR_INVALID_ARG             # rows without an index
    need = B.lib().dam_sparse_attn_prefill_workspace(ctypes.byref(attn_params()))
    if need:
        assert call_prefill(attn_params(), ws_bytes=need - 1) == B.DAM_ERR_WORKSPACE


def test_decode_argument_errors():
    L = B.lib()
    p = B.DecodeParams()
    p.batch, p.hq, p.hkv, p.kv_capacity, p.head_dim, p.dtype, p.scale = 2, 4, 2, 1024, 128, B.DAM_BF16, 0.0
    p.q_stride = (ctypes.c_int64 * 2)(512, 128)
    p.kv_stride = (ctypes.c_int64 * 3)(2 * 1024 * 128, 1024 * 128, 128)
    p.o_stride = (ctypes.c_int64 * 2)(512, 128)

    def call(pp, q=4096, idx=4096, max_kept=100, ws=4096, ws_bytes=1 << 30):
        return L.dam_sparse_attn_decode(ctypes.byref(pp), q, 4096, 4096, 4096, idx, max_kept, 4096, None, ws, ws_bytes, None)

    assert call(p, q=None) == B.DAM_ERR_INVALID_ARG
    assert call(p, idx=None) == B.DAM_ERR_INVALID_ARG
    assert call(p, max_kept=-1) == B.DAM_ERR_INVALID_ARG
    assert call(p, ws_bytes=8) == B.DAM_ERR_WORKSPACE
    p.head_dim = 80
    assert call(p) == B.DAM_ERR_UNSUPPORTED
    p.head_dim, p.hq = 128, 5
    assert call(p) == B.DAM_ERR_INVALID_ARG
    p.hq = 4
    assert L.dam_sparse_attn_decode_workspace(ctypes.byref(p), 4000) > 0

    def grouped(pp, member=4096, max_kept=100, ws_bytes=1 << 30):
        return L.dam_sparse_attn_decode_grouped(ctypes.byref(pp), 4096, 4096, 4096, 4096, 4096, member, max_kept, 4096, None,
                                                4096, ws_bytes, None)

    assert grouped(p, member=None) == B.DAM_ERR_INVALID_ARG
    assert grouped(p, ws_bytes=8) == B.DAM_ERR_WORKSPACE
    p.hq, p.hkv = 18, 2
    assert grouped(p) == B.DAM_ERR_UNSUPPORTED          # nine heads per KV head: the member bits are a byte
    p.hq, p.hkv = 4, 2
    assert L.dam_sparse_attn_decode_grouped_workspace(ctypes.byref(p), 4000) > 0


def capture_params(**kw):
    p = B.CaptureParams()
    p.hq, p.hkv, p.len, p.pcl, p.head_dim, p.dtype, p.scale = 2, 1, 64, 64, 128, B.DAM_BF16, 0.0
    p.q_stride = (ctypes.c_int64 * 2)(64 * 128, 128)
    p.k_stride = (ctypes.c_int64 * 2)(64 * 128, 128)
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_capture_argument_errors():
    L = B.lib()

    def call(cp, q=4096, a=4096, ws=4096, ws_bytes=1 << 30):
        return L.dam_capture_accumulate(ctypes.byref(cp), q, 4096, a, None, ws, ws_bytes, None)

    assert call(capture_params(), q=None) == B.DAM_ERR_INVALID_ARG
    assert call(capture_params(), a=None) == B.DAM_ERR_INVALID_ARG
    assert call(capture_params(hq=3, hkv=2)) == B.DAM_ERR_INVALID_ARG
    assert call(capture_params(len=65)) == B.DAM_ERR_INVALID_ARG           # longer than the statistics
    assert call(capture_params(len=0)) == B.DAM_ERR_INVALID_ARG
    assert call(capture_params(head_dim=100)) == B.DAM_ERR_UNSUPPORTED
    assert call(capture_params(dtype=3)) == B.DAM_ERR_UNSUPPORTED
    assert call(capture_params(len=64, pcl=16384)) == B.DAM_ERR_UNSUPPORTED
    assert call(capture_params(q_stride=(ctypes.c_int64 * 2)(64 * 128, 132))) == B.DAM_ERR_INVALID_ARG
    assert call(capture_params(k_stride=(ctypes.c_int64 * 2)(64 << 24, 1 << 24))) == B.DAM_ERR_UNSUPPORTED  # 32-bit row offsets
    assert call(capture_params(), ws_bytes=8) == B.DAM_ERR_WORKSPACE
    assert L.dam_capture_workspace(ctypes.byref(capture_params())) >= 2 * 64 * 4

    def fused(mp, cp, q=4096, ws=4096, ws_bytes=1 << 30):
        o = B.MaskOut()
        o.true_bits = 4096
        return L.dam_mask_build_from_qk(ctypes.byref(mp), ctypes.byref(cp), q, 4096, ctypes.byref(o), ws, ws_bytes, None)

    assert fused(mask_params(), capture_params(), q=None) == B.DAM_ERR_INVALID_ARG
    assert fused(mask_params(mode=B.DAM_FROM_PATTERNS), capture_params()) == B.DAM_ERR_INVALID_ARG
    assert fused(mask_params(n_maps=3), capture_params()) == B.DAM_ERR_INVALID_ARG        # n_maps != hq
    assert fused(mask_params(pcl=128), capture_params()) == B.DAM_ERR_INVALID_ARG         # pcl mismatch
    assert fused(mask_params(), capture_params(len=32)) == B.DAM_ERR_INVALID_ARG          # one full-length capture
    assert fused(mask_params(lam=0.3), capture_params()) == B.DAM_ERR_UNSUPPORTED
    assert fused(mask_params(transform=B.TRANSFORMS["sqrt"]), capture_params()) == B.DAM_ERR_UNSUPPORTED
    assert fused(mask_params(), capture_params(), ws_bytes=64) == B.DAM_ERR_WORKSPACE
    both = L.dam_mask_build_from_qk_workspace(ctypes.byref(mask_params()), ctypes.byref(capture_params()))
    assert both > L.dam_mask_build_workspace(ctypes.byref(mask_params()))


def test_eviction_argument_errors():
    L = B.lib()
    p = B.EvictParams()
    p.batch, p.hq, p.hkv, p.n_flags, p.pos, p.head_dim, p.dtype, p.kv_capacity, p.compact_capacity = 2, 4, 2, 512, 300, 128, B.DAM_BF16, 512, 64
    p.kv_stride = (ctypes.c_int64 * 3)(2 * 512 * 128, 512 * 128, 128)
    p.compact_stride = (ctypes.c_int64 * 3)(2 * 64 * 128, 64 * 128, 128)

    def plan(pp, flags=4096, ws=4096, ws_bytes=1 << 20, cols=None, cap=0):
        return L.dam_kv_evict_plan(ctypes.byref(pp), flags, 4096, 4096, 4096, cols, cap, None, 4096, ws, ws_bytes, None)

    assert plan(p, flags=None) == B.DAM_ERR_INVALID_ARG
    assert plan(p, ws_bytes=1) == B.DAM_ERR_WORKSPACE
    assert plan(p, cap=5) == B.DAM_ERR_INVALID_ARG                     # a capacity without a column buffer
    p.hq = 5
    assert plan(p) == B.DAM_ERR_INVALID_ARG
    p.hq = 4
    assert L.dam_kv_compact(ctypes.byref(p), 4096, 4096, 4096, 4096, 4096, 4096, None, None) == B.DAM_ERR_INVALID_ARG
    p.head_dim = 100                                                   # 200-byte rows
    assert L.dam_kv_compact(ctypes.byref(p), 4096, 4096, 4096, 4096, 4096, 4096, 4096, None) == B.DAM_ERR_UNSUPPORTED
    p.head_dim, p.pos = 128, 512                                       # newest key beyond the cache
    assert L.dam_kv_compact(ctypes.byref(p), 4096, 4096, 4096, 4096, 4096, 4096, 4096, None) == B.DAM_ERR_INVALID_ARG
    p.pos = 300
    assert L.dam_kv_remap_lists(ctypes.byref(p), 4096, 4096, 4096, None, 4096, 4096, None) == B.DAM_ERR_INVALID_ARG
    assert L.dam_kv_evict_workspace(ctypes.byref(p)) > 0


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libdam.so"))
    with pytest.raises(RuntimeError, match="missing"):
        B.lib()
