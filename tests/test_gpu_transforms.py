"""dam_mask_build with the alternative transforms of App. B against the oracle. raw sum, average,
min-max and square root are exact fp32 sequences: every output bit for bit. log, Yeo-Johnson,
arcsinh and z-score go through library functions / fp64 sums: their true-mask bits may differ only
where the shifted transformed value lies within a few fp32 ulp of tau, and everything after the true
mask must be exactly what the oracle derives from the device's own bits."""
import numpy as np
import pytest
import torch

import oracle
from dam_testlib import pack_rows_u64, u64
from paper_2506_11104_amd import binding as B
from test_gpu_mask import check_against_oracle, synth_map

pytestmark = pytest.mark.gpu

EXACT = ["raw_sum", "average", "minmax", "sqrt"]
BANDED = ["log", "yeo_johnson", "arcsinh", "zscore"]
# tau per transform, chosen inside the range of the shifted map of the test input
TAU = {"raw_sum": 0.05, "average": 0.05, "minmax": 0.05, "sqrt": 0.2, "log": 15.0, "yeo_johnson": 0.04, "arcsinh": 0.05,
       "zscore": 0.5}


def inputs(with_counts):
    rng = np.random.default_rng(41)
    H, L = 3, 200
    A = synth_map(rng, H, L)
    C = None
    if with_counts:
        C = np.zeros((H, L, L), np.float32)
        A2 = np.zeros((H, L, L), np.float32)
        for n in (L, 120):
            C[:, :n, :n] += np.tril(np.ones((n, n), np.float32))
            A2[:, :n, :n] += A[:, :n, :n]
        A = A2
    return A, C


def build(A, C, kind, lam, tau, S):
    H, L, _ = A.shape
    return B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=H, L=L, S=S, tile_m=128, tile_n=128, lam=lam, eps=1e-8, tau=tau, mu=0.7,
                        attn_sum=torch.from_numpy(A).cuda(), attn_cnt=None if C is None else torch.from_numpy(C).cuda(),
                        dense=True, rows=(S - 3, S), transform=B.TRANSFORMS[kind])


@pytest.mark.parametrize("with_counts", [False, True])
@pytest.mark.parametrize("kind", EXACT)
def test_exact_transforms_bit_for_bit(kind, with_counts):
    A, C = inputs(with_counts)
    tau = TAU[kind] * (2.0 if (with_counts and kind == "raw_sum") else 1.0)
    art = oracle.derive(A, C, 0.5, 1e-8, tau, 0.7, kind=kind)
    assert 0.005 < art.true_mask.mean() < 0.45                 # the threshold cuts through the map
    mask = build(A, C, kind, 0.5, tau, 500)
    torch.cuda.synchronize()
    assert np.float32(mask.bmin.item()) == np.float32(art.bmin)
    assert np.array_equal(u64(mask.true_bits), pack_rows_u64(art.true_mask))
    assert np.array_equal(mask.diag_cnt.cpu().numpy(), art.diag_cnt) and np.array_equal(mask.vert_cnt.cpu().numpy(), art.vert_cnt)
    assert np.array_equal(mask.diag_flag.cpu().numpy(), art.diag_flag) and np.array_equal(mask.vert_flag.cpu().numpy(), art.vert_flag)
    check_against_oracle(art, 500, 128, 128, mask, rows=(497, 500))


@pytest.mark.parametrize("with_counts", [False, True])
@pytest.mark.parametrize("kind,lam", [("log", 0.5), ("yeo_johnson", 0.7), ("yeo_johnson", 0.0), ("arcsinh", 0.5), ("zscore", 0.5)])
def test_library_transforms_within_a_band_of_the_threshold(kind, lam, with_counts):
    A, C = inputs(with_counts)
    tau = TAU[kind]
    T, tmin = oracle.transform(A, C, kind, lam, 1e-8)
    art = oracle.derive(A, C, lam, 1e-8, tau, 0.7, kind=kind)
    assert 0.005 < art.true_mask.mean() < 0.45
    mask = build(A, C, kind, lam, tau, 500)
    torch.cuda.synchronize()
    L = A.shape[1]
    got = np.ascontiguousarray(np.unpackbits(u64(mask.true_bits).view(np.uint8), axis=-1, bitorder="little")[..., :L])
    diff = got != art.true_mask
    shifted = T.astype(np.float64) - float(tmin)
    scale = max(1.0, float(np.abs(T).max()), abs(float(tmin)))
    near = np.abs(shifted - tau) <= 16 * 1.2e-7 * scale          # 16 ulp of the largest magnitude involved
    assert not (diff & ~near).any(), f"{int((diff & ~near).sum())} bits differ away from the threshold"
    assert abs(float(mask.bmin.item()) - float(tmin)) <= 4 * 1.2e-7 * scale
    dc, vc, df, vf = oracle.match(got, 0.7)
    assert np.array_equal(mask.diag_cnt.cpu().numpy(), dc) and np.array_equal(mask.vert_cnt.cpu().numpy(), vc)
    assert np.array_equal(mask.diag_flag.cpu().numpy(), df) and np.array_equal(mask.vert_flag.cpu().numpy(), vf)
    art_gpu = oracle.MaskArtefact(L=L, P=L, true_mask=got, diag_flag=df, vert_flag=vf, diag_cnt=dc, vert_cnt=vc)
    check_against_oracle(art_gpu, 500, 128, 128, mask, rows=(497, 500))
