"""dam_sparse_attn_decode_grouped_static (the entry point that allocates nothing: its scratch is a fixed array
inside the library) against dam_sparse_attn_decode_grouped on the same inputs: two calls in a row, the second on a
smaller problem, each bit-identical to the workspace form; a call beyond the array's size is refused. Collected
last on purpose."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2506_11104_amd import binding as B

pytestmark = pytest.mark.gpu


def problem(seed, Bn, Hq, Hkv, T, lens, dtype=torch.bfloat16, d=128):
    rng = np.random.default_rng(seed)
    G = Hq // Hkv
    lists = [np.sort(rng.choice(T, size=int(n), replace=False)).astype(np.int32) for n in lens]
    gptr, gidx, gmem = oracle.group_lists(lists, G)                      # (set operations only: inputs of the call)
    g = torch.Generator().manual_seed(seed)
    kc = torch.randn((Bn, Hkv, T, d), generator=g).to(dtype).cuda()
    vc = torch.randn((Bn, Hkv, T, d), generator=g).to(dtype).cuda()
    q = torch.randn((Bn, Hq, d), generator=g).to(dtype).cuda()
    return (q, kc, vc, torch.from_numpy(gptr.astype(np.int32)).cuda(), torch.from_numpy(gidx).cuda(),
            torch.from_numpy(gmem).cuda(), int(np.diff(gptr).max()))


def both(q, kc, vc, ptr, idx, mem, longest):
    want, want_lse = B.dam_sparse_attn_decode_grouped(q, kc, vc, ptr, idx, mem, longest, want_lse=True, shared_lists=True)
    out = torch.full_like(q, 7.0)
    lse = torch.full(q.shape[:2], 7.0, dtype=torch.float32, device="cuda")
    B.dam_sparse_attn_decode_grouped_static(q, kc, vc, ptr, idx, mem, longest, out, lse=lse, shared_lists=True)
    torch.cuda.synchronize()
    assert torch.equal(out, want) and torch.equal(lse, want_lse)
    assert not torch.isnan(out.float()).any()


def test_static_scratch_decode_matches_the_workspace_form_twice_in_a_row():
    assert B.lib().dam_sparse_attn_decode_grouped_static_limit() == 8 << 20
    # first a problem that is split many ways (long lists, few pairs: the matrix-core kernel with many splits) ...
    big = problem(91, 2, 8, 2, 9000, [4000, 3500, 0, 4100, 2500, 3000, 3999, 1])
    both(*big)
    # ... then a smaller one right behind it (fewer splits, shorter lists, another group size): the array still holds
    # the first call's partial results, none of which may leak into this one
    small = problem(92, 1, 4, 2, 700, [300, 0, 17, 650])
    both(*small)
    both(*big)
    # fp32 and head_dim 64 take the plain-ALU kernels through the same array
    f32 = problem(93, 2, 4, 2, 1200, [500, 900, 30, 0], dtype=torch.float32, d=64)
    both(*f32)


def test_static_scratch_decode_refuses_what_does_not_fit():
    q, kc, vc, ptr, idx, mem, longest = problem(94, 1, 4, 2, 700, [300, 0, 17, 650])
    # the same call declared for a batch whose partial results exceed the array: refused before anything is launched
    p = B.decode_params(q, kc, torch.empty_like(q), shared_lists=True)
    p.batch = 4096
    need = B.lib().dam_sparse_attn_decode_grouped_workspace(ctypes.byref(p), 1 << 20)
    assert need > B.lib().dam_sparse_attn_decode_grouped_static_limit()
    out = torch.full_like(q, 7.0)
    st = B.lib().dam_sparse_attn_decode_grouped_static(ctypes.byref(p), q.data_ptr(), kc.data_ptr(), vc.data_ptr(),
                                                       ptr.data_ptr(), idx.data_ptr(), mem.data_ptr(), 1 << 20,
                                                       out.data_ptr(), None, None)
    torch.cuda.synchronize()
    assert st == B.DAM_ERR_WORKSPACE and (out == 7.0).all()
