"""Seeded synthetic inputs shaped like long-context LLM attention layers.

This module only *produces inputs*: Q/K/V tensors, the attention statistics a frozen model would
have captured at the pattern capture length (a plain causal softmax of the first L rows, which is
the model's own attention and not part of the DAM method), and given pattern sets. It holds none of
the DAM arithmetic (no Box-Cox, threshold, matching, extension or sparse attention) and imports
neither the GPU binding nor the CPU oracle; both are fed the same bytes from here.

The five workloads mirror the benchmark configurations of this repository; each generator below states
its recipe. They stand in for what the paper measures on (LongEval / LV-Eval / Multi-News with
LLaMA-3.2 and Vicuna weights, Sec. 5), none of which is available here.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20250611


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str            # "prefill_map" | "prefill_patterns" | "decode"
    batch: int
    hq: int
    hkv: int
    head_dim: int
    seq: int             # S (prefill) or T, the current KV length (decode)
    pcl: int             # L; 0 when patterns are given directly
    dtype: str           # "f32" | "bf16"
    tile_m: int = 128
    tile_n: int = 128
    lam: float = 0.5
    eps: float = 1e-8
    tau: float = 0.3
    mu: float = 0.8
    seed: int = BASE_SEED
    steps: int = 1       # decode steps
    extra: Dict[str, float] = field(default_factory=dict)


# tau of c1/c2/c4 was chosen once, offline, so that the achieved density lands where the
# configuration asks (c1: ragged boundary around row 60; c2: ~10 %; c4: 1-5 %); the achieved density
# is always what gets reported.
WORKLOADS: Dict[str, Workload] = {
    "c1": Workload("c1", "prefill_map", 1, 2, 2, 64, 256, 64, "f32", 64, 64, tau=0.257, seed=BASE_SEED + 0),
    "c2": Workload("c2", "prefill_map", 1, 32, 8, 128, 4096, 1024, "bf16", tau=0.02, seed=BASE_SEED + 1),
    "c3": Workload("c3", "prefill_patterns", 1, 32, 8, 128, 32768, 0, "bf16", seed=BASE_SEED + 2),
    "c4": Workload("c4", "prefill_map", 1, 64, 8, 128, 131072, 4096, "bf16", tau=0.005, seed=BASE_SEED + 3,
                   extra={"win_lo": 300.0, "win_hi": 2500.0}),
    "c5": Workload("c5", "decode", 16, 32, 8, 128, 65536, 0, "bf16", seed=BASE_SEED + 4, steps=256),
}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller or altered copy of a workload (tests use it for tile-spanning mid sizes)."""
    return replace(w, **kw)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array to the storage dtype and return it as fp32 (bf16 values are exactly
    representable in fp32). Round-to-nearest-even on the upper 16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    u = x.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x_f32: np.ndarray) -> np.ndarray:
    """Upper 16 bits of fp32 values that are already bf16-representable (for upload as bf16)."""
    return (np.ascontiguousarray(x_f32, np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _ou_process(rng: np.random.Generator, n: int, dims: int, rho: float) -> np.ndarray:
    """Stationary AR(1) path p_i = rho p_{i-1} + sqrt(1-rho^2) xi_i, unit variance per dim, so that
    E[p_i . p_j] = dims * rho^|i-j| : a positional feature whose inner product decays with distance."""
    xi = rng.standard_normal((n, dims))
    p = np.empty((n, dims))
    p[0] = xi[0]
    c = np.sqrt(1.0 - rho * rho)
    for i in range(1, n):
        p[i] = rho * p[i - 1] + c * xi[i]
    return p


def qkv_structured(w: Workload):
    """c2 / c4 recipe. Q [Hq][S][d], K, V [Hkv][S][d] as fp32 arrays holding storage-rounded values.

    content:   iid N(0,1) in every entry (logits ~ N(0,1) after the 1/sqrt(d) scale);
    stripes:   per KV head 4 spike positions in [0, L) and a unit direction u; K[p] += a u, and each
               query head of the group adds b_h u to all its rows, a * b_h / sqrt(d) in [4, 8]
               (heterogeneous strength) -> vertical stripes at the spike columns;
    band:      per KV head an AR(1) positional feature p (32 dims) added to K's first 32 dims and,
               scaled by a per-query-head gain, to Q's: the logit gains beta_h * rho^|i-j|, i.e. a
               fading local window whose width differs per head (rho per KV head, beta per Q head).
    """
    rng = np.random.default_rng(w.seed)
    Hq, Hkv, S, d, L = w.hq, w.hkv, w.seq, w.head_dim, w.pcl
    G = Hq // Hkv
    pos_dims = 32
    Q = np.empty((Hq, S, d), np.float32)
    K = np.empty((Hkv, S, d), np.float32)
    V = np.empty((Hkv, S, d), np.float32)
    streams = rng.spawn(Hkv)
    for g, r in enumerate(streams):
        K[g] = r.standard_normal((S, d), dtype=np.float32)
        V[g] = r.standard_normal((S, d), dtype=np.float32)
        u = r.standard_normal(d)
        u[:pos_dims] = 0.0
        u /= np.linalg.norm(u)
        spikes = r.choice(L, size=4, replace=False)
        a = 8.0
        K[g, spikes] += (a * u).astype(np.float32)
        rho = 1.0 - 1.0 / r.uniform(w.extra.get("win_lo", 60.0), w.extra.get("win_hi", 400.0))
        p = _ou_process(r, S, pos_dims, rho)
        K[g, :, :pos_dims] += p.astype(np.float32)
        for q in range(G):
            h = g * G + q
            Q[h] = r.standard_normal((S, d), dtype=np.float32)
            strength = r.uniform(4.0, 8.0)            # stripe logit boost
            b = strength * np.sqrt(d) / a
            Q[h] += (b * u).astype(np.float32)
            beta = r.uniform(w.extra.get("beta_lo", 6.0), w.extra.get("beta_hi", 10.0))
            gain = beta * np.sqrt(d) / pos_dims
            Q[h, :, :pos_dims] += (gain * p).astype(np.float32)
    return to_storage(Q, w.dtype), to_storage(K, w.dtype), to_storage(V, w.dtype)


def qkv_iid(w: Workload, std: float = 1.0):
    """c1 / c3 recipe: iid N(0, std^2) entries."""
    rng = np.random.default_rng(w.seed)
    Q = rng.standard_normal((w.hq, w.seq, w.head_dim), dtype=np.float32) * np.float32(std)
    K = rng.standard_normal((w.hkv, w.seq, w.head_dim), dtype=np.float32) * np.float32(std)
    V = rng.standard_normal((w.hkv, w.seq, w.head_dim), dtype=np.float32) * np.float32(std)
    return to_storage(Q, w.dtype), to_storage(K, w.dtype), to_storage(V, w.dtype)


def capture_map(Q: np.ndarray, K: np.ndarray, L: int, hq_per_kv: int) -> np.ndarray:
    """What a frozen model would hand to stage one after ONE captured sequence of length L: its
    causal softmax attention probabilities A [Hq][L][L] (fp64 softmax, stored fp32, zeros above the
    diagonal). The count matrix C of that capture is 1 on j <= i and 0 above."""
    Hq, _, d = Q.shape
    A = np.zeros((Hq, L, L), np.float32)
    tri = np.tril(np.ones((L, L), bool))
    for h in range(Hq):
        q = Q[h, :L].astype(np.float64)
        k = K[h // hq_per_kv, :L].astype(np.float64)
        s = (q @ k.T) / np.sqrt(np.float64(d))
        s[~tri] = -np.inf
        s -= s.max(axis=1, keepdims=True)
        e = np.exp(s)
        A[h] = (e / e.sum(axis=1, keepdims=True)).astype(np.float32)
    return A


def density_of_patterns(diag: np.ndarray, vert: np.ndarray, S: int) -> float:
    """Kept fraction of the causal triangle for a pattern-only mask (union of diagonals/columns)."""
    nd = np.flatnonzero(diag)
    nv = np.flatnonzero(vert)
    tot = float(np.sum(S - nd)) + float(np.sum(S - nv))
    # overlaps: entry (i, c) with i - c in diag, counted once
    if len(nd) and len(nv):
        dset = np.zeros(S, bool)
        dset[nd] = True
        for c in nv:
            tot -= float(np.count_nonzero(dset[: S - c]))
    return tot / (S * (S + 1) / 2.0)


def patterns_c3(w: Workload):
    """c3 recipe: per query head a random mixture of sink columns (first 4..64 keys), a sliding
    window (256..4096 diagonals), 0..32 extra stripe columns anywhere and 0..4 diagonal bands of
    width 16..256, re-drawn until the head's density lies in [2 %, 20 %]. All of it is inside the
    paper's pattern pool (Sec. 4.2.4). Returns (diag_flag, vert_flag) u8 [Hq][S]."""
    S, Hq = w.seq, w.hq
    rng = np.random.default_rng(w.seed + 7919)
    lo, hi = w.extra.get("dens_lo", 0.02), w.extra.get("dens_hi", 0.20)
    win_lo = int(w.extra.get("win_lo", min(256, max(1, S // 128))))
    win_hi = int(w.extra.get("win_hi", min(4096, max(2, S // 8))))
    diag = np.zeros((Hq, S), np.uint8)
    vert = np.zeros((Hq, S), np.uint8)
    for h, r in enumerate(rng.spawn(Hq)):
        while True:
            d = np.zeros(S, np.uint8)
            v = np.zeros(S, np.uint8)
            v[: min(S, int(r.integers(4, 65)))] = 1
            d[: min(S, int(r.integers(win_lo, win_hi + 1)))] = 1
            n_str = int(r.integers(0, 33))
            if n_str:
                v[r.integers(0, S, size=n_str)] = 1
            for _ in range(int(r.integers(0, 5))):
                bw = int(r.integers(16, 257))
                r0 = int(r.integers(0, max(1, S - bw)))
                d[r0:r0 + bw] = 1
            if lo <= density_of_patterns(d, v, S) <= hi:
                break
        diag[h], vert[h] = d, v
    return diag, vert


def patterns_c5(w: Workload):
    """c5 recipe: per query head, sink columns (4..64), a window, and stripe columns sized so that a
    row near position T keeps about 5 % of its keys. Returns (diag_flag, vert_flag) u8 [Hq][P],
    P = T + steps (the lists are taken at positions T-1 .. T+steps-2)."""
    P = w.seq + w.steps
    rng = np.random.default_rng(w.seed + 104729)
    target = w.extra.get("kept_frac", 0.05) * w.seq
    diag = np.zeros((w.hq, P), np.uint8)
    vert = np.zeros((w.hq, P), np.uint8)
    for h, r in enumerate(rng.spawn(w.hq)):
        n_sink = int(r.integers(4, 65))
        share = r.uniform(0.3, 0.8)                      # part of the budget spent on the window
        win = max(1, int(share * target))
        n_str = max(0, int(target) - win - n_sink)
        vert[h, :n_sink] = 1
        diag[h, :win] = 1
        if n_str:
            vert[h, r.choice(np.arange(n_sink, w.seq - win), size=n_str, replace=False)] = 1
    return diag, vert


def decode_inputs(w: Workload, device: Optional[str] = None):
    """c5 tensors, generated with torch's seeded CPU generator (bf16-rounded, returned as torch
    tensors): q [steps][B][Hq][d], K/V caches [B][Hkv][T+steps][d]."""
    import torch
    g = torch.Generator().manual_seed(w.seed)
    cap = w.seq + w.steps
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    q = torch.randn((w.steps, w.batch, w.hq, w.head_dim), generator=g, dtype=torch.float32).to(dt)
    kc = torch.empty((w.batch, w.hkv, cap, w.head_dim), dtype=dt)
    vc = torch.empty((w.batch, w.hkv, cap, w.head_dim), dtype=dt)
    for b in range(w.batch):
        kc[b] = torch.randn((w.hkv, cap, w.head_dim), generator=g, dtype=torch.float32).to(dt)
        vc[b] = torch.randn((w.hkv, cap, w.head_dim), generator=g, dtype=torch.float32).to(dt)
    if device:
        q, kc, vc = q.to(device), kc.to(device), vc.to(device)
    return q, kc, vc
