"""dam_capture_accumulate and dam_mask_build_from_qk on the GPU against the oracle.

The accumulated statistics are fp32 sums of fp32 probabilities: they are compared within a
tolerance derived from the arithmetic (fp32 logits from exact bf16 products, fp32 softmax).
The fused build thresholds those probabilities directly, so its true mask may differ from the
oracle's only at entries whose probability lies within that tolerance of the threshold; every
later output must then be exactly what the oracle derives from the GPU's own true mask."""
import numpy as np
import pytest
import torch

import oracle
from dam_testlib import dev, pack_rows_u64, u64
from paper_2506_11104_amd import binding as B
from paper_2506_11104_amd import workloads as wl
from test_gpu_mask import check_against_oracle

pytestmark = pytest.mark.gpu

# |p_gpu - p| <= ATOL + RTOL * p: the logit of a pair carries an absolute error of a few 1e-5 (fp32
# accumulation of 128 products, scale, subtraction of a log-sum-exp of magnitude up to ~50), which is
# the relative error of its probability; the hardware exp2 / log2 add a few ulp.
RTOL, ATOL = 2e-4, 1e-7
# the fused build: true-mask bits may differ only where |p - theta| <= BAND * theta (purely relative: the
# threshold sits far above the absolute floor)
BAND = 1e-4


def seq_pair(seed, Hq, Hkv, n, d, dtype, std=1.0):
    rng = np.random.default_rng(seed)
    Q = wl.to_storage(rng.standard_normal((Hq, n, d)).astype(np.float32) * np.float32(std), dtype)
    K = wl.to_storage(rng.standard_normal((Hkv, n, d)).astype(np.float32) * np.float32(std), dtype)
    return Q, K


CASES = [  # (Hq, Hkv, d, dtype, L, lengths of the captured sequences)
    (2, 2, 64, "f32", 64, (64,)),            # c1's shape, plain kernel
    (4, 2, 128, "bf16", 320, (320, 150)),    # matrix-core kernels, ragged tiles, two captures
    (2, 1, 128, "bf16", 256, (256, 256)),    # whole tiles
    (3, 3, 64, "bf16", 128, (100, 128)),     # bf16 with another head_dim: plain kernel
    (2, 1, 128, "f32", 96, (96, 1)),         # fp32 inputs at head_dim 128, a one-token capture
]


@pytest.mark.parametrize("Hq,Hkv,d,dtype,L,lens", CASES)
def test_accumulate_matches_oracle(Hq, Hkv, d, dtype, L, lens):
    A = C = None
    a_dev = torch.zeros((Hq, L, L), dtype=torch.float32, device="cuda")
    c_dev = torch.zeros((Hq, L, L), dtype=torch.float32, device="cuda")
    for t, n in enumerate(lens):
        Q, K = seq_pair(100 + t, Hq, Hkv, n, d, dtype, std=1.5)
        A, C = oracle.capture(Q, K, L, attn_sum=A, attn_cnt=C)
        B.dam_capture_accumulate(dev(Q, dtype), dev(K, dtype), a_dev, c_dev)
    torch.cuda.synchronize()
    got_a, got_c = a_dev.cpu().numpy(), c_dev.cpu().numpy()
    assert np.array_equal(got_c, C), "counts"
    err = np.abs(got_a - A)
    bound = len(lens) * ATOL + RTOL * A
    assert (err <= bound).all(), f"max excess {(err - bound).max():.3e}, max err {err.max():.3e}"
    assert not got_a[:, ~np.tril(np.ones((L, L), bool))].any(), "entries above the diagonal"


def test_accumulate_without_counts_and_strided_heads():
    # heads interleaved in memory ([n][H][d] storage viewed as [H][n][d]), no count matrix
    Hq, Hkv, n, d, L = 4, 2, 200, 128, 256
    Q, K = seq_pair(7, Hq, Hkv, n, d, "bf16")
    A, _ = oracle.capture(Q, K, L, want_cnt=False)
    q_dev = dev(np.ascontiguousarray(Q.transpose(1, 0, 2)), "bf16").transpose(0, 1)
    k_dev = dev(np.ascontiguousarray(K.transpose(1, 0, 2)), "bf16").transpose(0, 1)
    a_dev = torch.zeros((Hq, L, L), dtype=torch.float32, device="cuda")
    B.dam_capture_accumulate(q_dev, k_dev, a_dev, None)
    torch.cuda.synchronize()
    err = np.abs(a_dev.cpu().numpy() - A)
    assert (err <= ATOL + RTOL * A).all(), err.max()


def unpack(bits_u64: np.ndarray, L: int) -> np.ndarray:
    return np.ascontiguousarray(np.unpackbits(bits_u64.view(np.uint8), axis=-1, bitorder="little")[..., :L])


def fused_against_oracle(Q, K, w, S, tm, tn, tau, mu, dtype, rows=None):
    Hq, L = Q.shape[0], w.pcl
    A, _ = oracle.capture(Q[:, :L].copy(), K[:, :L].copy(), L, want_cnt=False)
    art = oracle.derive(A, None, w.lam, w.eps, tau, mu)
    mask = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=Hq, L=L, S=S, tile_m=tm, tile_n=tn, lam=w.lam, eps=w.eps, tau=tau,
                        mu=mu, qk=(dev(Q[:, :L].copy(), dtype), dev(K[:, :L].copy(), dtype)), dense=S <= 4096, rows=rows)
    torch.cuda.synchronize()
    got = unpack(u64(mask.true_bits), L)
    want = art.true_mask
    diff = got != want
    # the threshold in terms of the stored probability: between the largest dropped and the smallest kept
    tri = np.tril(np.ones((L, L), bool))[None]
    kept_vals, dropped_vals = A[(want == 1)], A[(want == 0) & tri]
    if kept_vals.size and dropped_vals.size:
        theta = 0.5 * (float(kept_vals.min()) + float(dropped_vals.max()))
        assert dropped_vals.max() <= kept_vals.min()
        near = np.abs(A - theta) <= BAND * theta
        assert not (diff & ~near).any(), f"{int((diff & ~near).sum())} true-mask bits differ away from the threshold"
        assert diff.sum() <= max(8, 0.01 * near.sum() + 8) or near.sum() < 64, (int(diff.sum()), int(near.sum()))
    else:  # everything kept or everything dropped: no boundary, the masks must be identical
        assert not diff.any()
    assert not (got & ~tri).any()
    # everything after the true mask is exact given the GPU's own bits
    dc, vc, df, vf = oracle.match(got, mu)
    assert np.array_equal(mask.diag_cnt.cpu().numpy(), dc) and np.array_equal(mask.vert_cnt.cpu().numpy(), vc)
    assert np.array_equal(mask.diag_flag.cpu().numpy(), df) and np.array_equal(mask.vert_flag.cpu().numpy(), vf)
    assert np.float32(mask.bmin.item()) == np.float32(art.bmin)
    art_gpu = oracle.MaskArtefact(L=L, P=L, true_mask=got, diag_flag=df, vert_flag=vf, diag_cnt=dc, vert_cnt=vc)
    check_against_oracle(art_gpu, S, tm, tn, mask, rows=rows, dense=S <= 4096)
    return int(diff.sum()), art, art_gpu


@pytest.mark.parametrize("tau,mu", [(0.257, 0.8), (0.3, 0.8), (0.0, 0.8), (3.0, 0.8)])
def test_fused_build_c1(tau, mu):
    w = wl.WORKLOADS["c1"]
    Q, K, _ = wl.qkv_iid(w, std=1 / 8)
    fused_against_oracle(Q, K, w, w.seq, 64, 64, tau, mu, "f32", rows=(0, w.seq))


def test_fused_build_c2_shape_scaled():
    # c2's recipe at a quarter of its length (L = 256, S = 1024): stripes and a fading window, GQA
    w = wl.scaled(wl.WORKLOADS["c2"], hq=8, hkv=2, seq=1024, pcl=256)
    Q, K, _ = wl.qkv_structured(w)
    ndiff, art, art_gpu = fused_against_oracle(Q, K, w, w.seq, 128, 128, w.tau, w.mu, "bf16", rows=(1000, 1003))
    assert art.vert_flag.sum() > 0 and art.diag_flag.sum() > 0     # the recipe produces both pattern kinds


@pytest.mark.parametrize("tau", [0.0, -1.0, 3.0])
def test_fused_build_keep_all_and_keep_none_on_the_matrix_core_path(tau):
    w = wl.scaled(wl.WORKLOADS["c2"], hq=4, hkv=2, seq=512, pcl=256)
    Q, K, _ = wl.qkv_structured(w)
    ndiff, art, _ = fused_against_oracle(Q, K, w, w.seq, 128, 128, tau, 0.8, "bf16")
    assert ndiff == 0
    assert art.true_mask.sum() == (0 if tau > 2 else 4 * 256 * 257 // 2)


def test_fused_build_ragged_capture_length():
    # L = 200: not a multiple of the key block, of the 128-key group or of the 64-bit word
    w = wl.scaled(wl.WORKLOADS["c2"], hq=4, hkv=2, seq=500, pcl=200)
    Q, K, _ = wl.qkv_structured(w)
    fused_against_oracle(Q, K, w, w.seq, 128, 128, 0.05, 0.8, "bf16")


@pytest.mark.parametrize("n", [2, 33, 64, 65, 128, 130, 192])   # one, two and three stages of 64 keys, whole and ragged
def test_short_captures_on_the_matrix_core_path(n):
    """Capture lengths around the kernels' stage (64 keys), block (32) and tile (128 rows) sizes: the summed form
    against the oracle, and the fused build of a map of that very length."""
    Hq, Hkv, d = 4, 2, 128
    Q, K = seq_pair(300 + n, Hq, Hkv, n, d, "bf16", std=1.2)
    L = max(n, 4)
    A, C = oracle.capture(Q, K, L)
    a_dev = torch.zeros((Hq, L, L), dtype=torch.float32, device="cuda")
    c_dev = torch.zeros((Hq, L, L), dtype=torch.float32, device="cuda")
    B.dam_capture_accumulate(dev(Q, "bf16"), dev(K, "bf16"), a_dev, c_dev)
    torch.cuda.synchronize()
    assert np.array_equal(c_dev.cpu().numpy(), C)
    err = np.abs(a_dev.cpu().numpy() - A)
    assert (err <= ATOL + RTOL * A).all(), err.max()
    w = wl.scaled(wl.WORKLOADS["c2"], hq=Hq, hkv=Hkv, seq=n, pcl=n)
    fused_against_oracle(Q, K, w, n, 128, 128, 0.05, 0.8, "bf16")
