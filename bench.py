#!/usr/bin/env python3
"""Benchmark of the DAM hot path on one MI355X.

A step is one pass of the hot path over one synthetic batch of the 32k prefill workload (c3):
dam_mask_build (matched patterns -> tile pool + block index at S = 32768) followed by
dam_sparse_attn_prefill over the listed tiles. `value` is effective TFLOP/s on kept entries,
4 * head_dim * nnz / step time, with every input resident in HBM before the timed region.
The same run also reports (extra keys of the one JSON line) the prefill kernel against the bf16
MFMA roofline, the decode workload (c5) and the attention-map mask build (c2 and c4 shapes) against
the HBM roofline, and the CPU oracle timed on a bounded sample of the same prefill workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c2] [--no-decode] [--no-cpu]
"""
import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

# `traffic` in the roofline objects is null: this script does not read hardware counters. The HBM bytes per launch of
# the dominant kernels, from rocprofv3 --pmc runs of this script (--copy-calibration gives the counters' scale), are
# kept with their commands under profiles/.


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=["c3", "c2"])
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-maskmap", action="store_true")
    ap.add_argument("--no-small", action="store_true", help="skip the c1 and c2 lines")
    ap.add_argument("--pause-before-decode", type=float, default=4.0, help="idle seconds before the decode section")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay timings (profiler runs)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain device copies of 1 GiB (a kernel of known traffic, for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command)")
    return ap.parse_args()


def events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def timed_ms(fn, n, warm=3):
    """Mean duration of n back-to-back calls of fn on torch's current stream (HIP events), after `warm` untimed ones."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ev = events(2)
    ev[0].record()
    for _ in range(n):
        fn()
    ev[1].record()
    torch.cuda.synchronize()
    return ev[0].elapsed_time(ev[1]) / n


def graph_replay_ms(fn, n):
    """fn captured once into a HIP graph (the entry points allocate nothing and never synchronise), then the mean
    duration of n replays: what a launch-bound sequence costs without the host's part."""
    import torch
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return timed_ms(g.replay, n)


def bench_prefill(args, w, torch, B, wl):
    """Returns the result dict of the prefill workload (mask build + sparse prefill per step)."""
    dev = "cuda"
    H, S, d = w.hq, w.seq, w.head_dim
    Q, K, V = wl.qkv_iid(w) if w.kind == "prefill_patterns" else wl.qkv_structured(w)
    if w.kind == "prefill_patterns":
        dflag, vflag = wl.patterns_c3(w)
        mode, L = B.DAM_FROM_PATTERNS, 0
        A = None
    else:
        A = torch.from_numpy(wl.capture_map(Q, K, w.pcl, w.hq // w.hkv)).to(dev)
        mode, L = B.DAM_FROM_ATTN_MAP, w.pcl
        dflag = vflag = None
    to_dev = lambda x: torch.from_numpy(x).to(torch.bfloat16)[None].to(dev)
    q, k, v = to_dev(Q), to_dev(K), to_dev(V)
    d_in = torch.from_numpy(dflag).to(dev) if dflag is not None else None
    v_in = torch.from_numpy(vflag).to(dev) if vflag is not None else None

    # sizing call (outside the timed region): how many tiles does the pool need
    # (full tiles carry no bits in the pool: DAM_MASK_SKIP_FULL_TILE_BITS, the attention kernel takes them from blk_kind;
    # the matched columns are listed in tiles of their own: DAM_MASK_GATHER_COLUMNS)
    FLAGS = B.DAM_MASK_SKIP_FULL_TILE_BITS | B.DAM_MASK_GATHER_COLUMNS
    sized = B.build_mask(mode=mode, H=H, L=L, S=S, tile_m=w.tile_m, tile_n=w.tile_n, lam=w.lam, eps=w.eps, tau=w.tau,
                         mu=w.mu, attn_sum=A, diag_in=d_in, vert_in=v_in, flags=FLAGS)
    torch.cuda.synchronize()
    n_tiles = sized.n_tiles
    kinds = sized.blk_kind.cpu().numpy()
    n_full = int((kinds & 1).sum())
    # kept entries: popcount of the partial tiles of the pool (chunked on the device as bytes through a lookup
    # table) plus the area of the full tiles
    lut = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device=dev)
    nnz = n_full * w.tile_m * w.tile_n
    tb = sized.tile_bits[(sized.blk_kind & 1) == 0].view(torch.uint8).reshape(-1)
    for off in range(0, tb.numel(), 1 << 28):
        nnz += int(lut[tb[off:off + (1 << 28)].long()].sum().item())
    del tb
    causal = H * S * (S + 1) // 2

    # preallocated outputs for the timed steps
    p = B.MaskParams(mode, H, L, S, w.tile_m, w.tile_n, 0, 0, w.lam, w.eps, w.tau, w.mu, float("nan"), FLAGS)
    ws_mask = B.mask_workspace(p, dev)
    o = B.MaskOut()
    for name in ("true_bits", "diag_cnt", "vert_cnt", "diag_flag", "vert_flag", "bmin"):
        t = getattr(sized, name)
        if mode == B.DAM_FROM_ATTN_MAP and t is not None:
            setattr(o, name, t.data_ptr())
    total = torch.zeros(1, dtype=torch.int64, device=dev)
    o.blk_row_ptr, o.blk_col, o.blk_kind = sized.blk_row_ptr.data_ptr(), sized.blk_col.data_ptr(), sized.blk_kind.data_ptr()
    o.tile_bits, o.blk_capacity, o.blk_total = sized.tile_bits.data_ptr(), n_tiles, total.data_ptr()
    o.gather_idx, o.gather_cnt = sized.gather_idx.data_ptr(), sized.gather_cnt.data_ptr()
    out = torch.empty_like(q)
    ap_ = B.attn_params(q, k, v, out, w.tile_m, w.tile_n, gather_rows=sized.gather_rows)
    ws_attn = B.prefill_workspace(ap_, dev)

    def step(ev=None):
        if ev:
            ev[0].record()
        B.dam_mask_build(p, A, None, d_in, v_in, o, ws_mask)
        if ev:
            ev[1].record()
        B.dam_sparse_attn_prefill(q, k, v, sized, out=out, ws=ws_attn)
        if ev:
            ev[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [events(3) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # medians over the timed steps (HIP events on the launch stream); the mean of the host's clock over the same steps
    # is kept beside them
    mask_ms = float(np.median([e[0].elapsed_time(e[1]) for e in evs]))
    attn_ms = float(np.median([e[1].elapsed_time(e[2]) for e in evs]))
    step_ms = float(np.median([e[0].elapsed_time(e[2]) for e in evs]))
    step_ms_wall = wall * 1e3 / args.steps
    assert int(total.item()) == n_tiles

    flops_kept = 4.0 * d * nnz
    # the same prefill over the plain layout (every matched column in the ordinary tile it falls into), kernel alone
    plain = B.build_mask(mode=mode, H=H, L=L, S=S, tile_m=w.tile_m, tile_n=w.tile_n, lam=w.lam, eps=w.eps, tau=w.tau,
                         mu=w.mu, attn_sum=A, diag_in=d_in, vert_in=v_in, flags=B.DAM_MASK_SKIP_FULL_TILE_BITS)
    ws_plain = B.prefill_workspace(B.attn_params(q, k, v, out, w.tile_m, w.tile_n), dev)
    plain_ms = timed_ms(lambda: B.dam_sparse_attn_prefill(q, k, v, plain, out=out, ws=ws_plain), 10, warm=2)
    plain_tiles = plain.n_tiles
    n_blocks = int(np.unpackbits((kinds >> 1)[:, None].astype(np.uint8), axis=1).sum())
    plain_blocks = int(np.unpackbits((plain.blk_kind.cpu().numpy() >> 1)[:, None].astype(np.uint8), axis=1).sum())
    del plain

    flops_tiles = 4.0 * d * w.tile_m * w.tile_n * n_tiles
    mask_bytes = (n_tiles - n_full) * (w.tile_m * w.tile_n // 8) + 5 * n_tiles + 4 * H * (sized.blk_row_ptr.shape[1]) + 2 * H * S
    if A is not None:
        mask_bytes += 2 * H * L * (L + 1) + H * L * L // 8
    res = {
        "step_ms": step_ms, "step_ms_mean_host_clock": step_ms_wall, "mask_build_ms": mask_ms, "prefill_ms": attn_ms, "nnz": nnz, "n_tiles": n_tiles,
        "n_full_tiles": n_full, "density": nnz / causal, "tile_fill": nnz / (n_tiles * w.tile_m * w.tile_n),
        "tflops_kept_step": flops_kept / (step_ms * 1e-3) / 1e12,
        "tflops_kept_prefill": flops_kept / (attn_ms * 1e-3) / 1e12,
        "tflops_tiles_prefill": flops_tiles / (attn_ms * 1e-3) / 1e12,
        "mask_build_gbs": mask_bytes / (mask_ms * 1e-3) / 1e9, "mask_build_bytes": mask_bytes,
        "n_blocks": n_blocks, "tflops_blocks_prefill": 4.0 * d * w.tile_m * 32 * n_blocks / (attn_ms * 1e-3) / 1e12,
        "gathered_tiles": int((sized.blk_col >= (S + w.tile_n - 1) // w.tile_n).sum().item()),
        "plain_layout": {"listed_tiles": plain_tiles, "key_blocks_of_32": plain_blocks, "prefill_ms_back_to_back": plain_ms,
                         "tflops_kept_entries": flops_kept / (plain_ms * 1e-3) / 1e12,
                         "tflops_issued_blocks": 4.0 * d * w.tile_m * 32 * plain_blocks / (plain_ms * 1e-3) / 1e12,
                         "frac_issued_blocks": 4.0 * d * w.tile_m * 32 * plain_blocks / (plain_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
    }
    ctx = dict(Q=Q, K=K, V=V, dflag=dflag, vflag=vflag, A=A, sized=sized)
    return res, ctx


def bench_cpu_oracle(args, w, ctx, wl):
    """The oracle (fp64, OpenMP over rows) timed on a bounded random sample of rows of the same
    workload; reported in the metric's unit (TFLOP/s on kept entries)."""
    import oracle
    if ctx["dflag"] is not None:
        art = oracle.from_patterns(ctx["dflag"], ctx["vflag"])
    else:
        art = oracle.derive(ctx["A"].cpu().numpy(), None, w.lam, w.eps, w.tau, w.mu)
    rng = np.random.default_rng(1234)

    def run(n):
        hs = rng.integers(0, w.hq, n).astype(np.int32)
        rs = rng.integers(0, w.seq, n).astype(np.int64)
        t0 = time.perf_counter()
        _, _ = oracle.attend_rows(ctx["Q"][hs, rs], ctx["K"], ctx["V"], art, w.hq, hs, rs)
        dt = time.perf_counter() - t0
        m = min(n, 4096)
        kept = sum(len(oracle.kept_list(art, int(h), int(r))) for h, r in zip(hs[:m], rs[:m])) / m * n
        return dt, kept

    run(512)                                   # thread start-up, page faults
    dt, kept = run(16384)
    n = int(min(2_000_000, max(16384, 16384 * args.cpu_seconds / max(dt, 1e-3))))
    dt, kept = run(n)
    return {"value": 4.0 * w.head_dim * kept / dt / 1e12, "unit": "TFLOP/s (kept entries)", "cores": oracle.threads(),
            "kind": "oracle", "sample": f"{n} random (head,row) pairs of {w.name}, {dt:.1f} s, fp64, kept entries "
                                        f"estimated from 4096 of them"}


def bench_decode(args, torch, B, wl):
    """c5: a decode step = the kept lists of the new row (dam_mask_build, list form) + attention over them. The main
    numbers are for the grouped-query form (one merged list per KV head, shared by the batch, every cached row read
    once per group: the algorithmic bytes are exactly the rows it lists); the form with a list per head follows, and
    the KV eviction at the first position."""
    w = wl.WORKLOADS["c5"]
    dev = "cuda"
    steps = args.decode_steps
    cap = w.seq + steps
    G = w.hq // w.hkv
    g = torch.Generator(device=dev).manual_seed(w.seed)
    kc = torch.randn((w.batch, w.hkv, cap, w.head_dim), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    vc = torch.randn((w.batch, w.hkv, cap, w.head_dim), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    qs = torch.randn((steps, w.batch, w.hq, w.head_dim), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    dflag, vflag = wl.patterns_c5(wl.scaled(w, steps=steps))
    # every sequence of the batch sits at the same position, and a mask belongs to its head, not to an input:
    # the lists are shared by the batch (dam_decode_params.shared_lists)
    d_in = torch.from_numpy(dflag).to(dev)
    v_in = torch.from_numpy(vflag).to(dev)
    max_kept = int((dflag.sum(1) + vflag.sum(1)).max())          # bound of one head's list
    max_group = min(G * max_kept, cap)                           # bound of a merged list
    total = torch.zeros(1, dtype=torch.int64, device=dev)
    out = torch.empty((w.batch, w.hq, w.head_dim), dtype=torch.bfloat16, device=dev)
    dp = B.decode_params(qs[0], kc, out, shared_lists=True)
    row_bytes = w.batch * w.head_dim * 2 * 2                     # a listed row: K and V, every sequence of the batch

    def params(pos, grouped):
        # rows of the mask do not depend on the problem length it is built for (the extension only
        # continues patterns), so the lists are taken from the length-`cap` mask the flags are sized for
        return B.MaskParams(B.DAM_FROM_PATTERNS, w.hq, 0, cap, 128, 128, pos, pos + 1, 0.5, 1e-8, 0.3, 0.8, float("nan"),
                            B.DAM_MASK_GROUP_LISTS if grouped else 0, 0, G if grouped else 0)

    def form(grouped, n_steps):
        n_lists = w.hkv if grouped else w.hq
        bound = max_group if grouped else max_kept
        ptr = torch.empty(n_lists + 1, dtype=torch.int32, device=dev)
        idx = torch.empty(n_lists * bound, dtype=torch.int32, device=dev)
        mem = torch.empty(n_lists * bound, dtype=torch.uint8, device=dev) if grouped else None
        o = B.MaskOut()
        o.kept_ptr, o.kept_idx, o.kept_capacity, o.kept_total = ptr.data_ptr(), idx.data_ptr(), idx.numel(), total.data_ptr()
        if grouped:
            o.kept_member = mem.data_ptr()
        ws_mask = B.mask_workspace(params(cap - 1, grouped), dev)
        ws_dec = B.decode_grouped_workspace(dp, bound, dev) if grouped else B.decode_workspace(dp, bound, dev)

        def step(s, ev=None):
            pos = w.seq - 1 + s
            if ev:
                ev[0].record()
            B.dam_mask_build(params(pos, grouped), None, None, d_in, v_in, o, ws_mask)
            if ev:
                ev[1].record()
            if grouped:
                B.dam_sparse_attn_decode_grouped(qs[s], kc, vc, ptr, idx, mem, bound, out=out, ws=ws_dec, shared_lists=True)
            else:
                B.dam_sparse_attn_decode(qs[s], kc, vc, ptr, idx, bound, out=out, ws=ws_dec, shared_lists=True)
            if ev:
                ev[2].record()

        for s in range(3):
            step(s)
        torch.cuda.synchronize()
        evs = [events(3) for _ in range(n_steps)]
        t0 = time.perf_counter()
        for s in range(n_steps):
            step(s, evs[s])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        entries_last = int(total.item())
        step(0)
        torch.cuda.synchronize()
        entries = 0.5 * (entries_last + int(total.item()))       # list entries per step, mean of first and last position
        res = {"steps": n_steps, "us_per_step": wall * 1e6 / n_steps,
               "list_build_us": float(np.mean([e[0].elapsed_time(e[1]) for e in evs])) * 1e3,
               "decode_us": float(np.mean([e[1].elapsed_time(e[2]) for e in evs])) * 1e3, "list_entries": entries}
        # the attention call alone, 50 in a row between two events (no event between the calls)
        B.dam_mask_build(params(w.seq - 1, grouped), None, None, d_in, v_in, o, ws_mask)
        if grouped:
            res["decode_us_back_to_back"] = timed_ms(lambda: B.dam_sparse_attn_decode_grouped(
                qs[0], kc, vc, ptr, idx, mem, bound, out=out, ws=ws_dec, shared_lists=True), 50) * 1e3
        else:
            res["decode_us_back_to_back"] = timed_ms(lambda: B.dam_sparse_attn_decode(
                qs[0], kc, vc, ptr, idx, bound, out=out, ws=ws_dec, shared_lists=True), 50) * 1e3
        if not args.no_graph:
            res["us_per_step_graph_replay"] = graph_replay_ms(lambda: step(0), 50) * 1e3
        return res, (ptr, idx, bound)

    def overlapped(n_steps):
        """The grouped form with the list build of step s + 1 on a second stream (default priority) while step s
        attends: a head's mask rows do not depend on the step's output, so only the lists' buffers (two sets) and
        two events per step tie the streams together."""
        side = torch.cuda.Stream()
        bufs = []
        for _ in range(2):
            ptr = torch.empty(w.hkv + 1, dtype=torch.int32, device=dev)
            idx = torch.empty(w.hkv * max_group, dtype=torch.int32, device=dev)
            mem = torch.empty(w.hkv * max_group, dtype=torch.uint8, device=dev)
            o = B.MaskOut()
            o.kept_ptr, o.kept_idx, o.kept_capacity, o.kept_total = ptr.data_ptr(), idx.data_ptr(), idx.numel(), total.data_ptr()
            o.kept_member = mem.data_ptr()
            bufs.append((ptr, idx, mem, o))
        ws_mask = B.mask_workspace(params(cap - 1, True), dev)
        ws_dec = B.decode_grouped_workspace(dp, max_group, dev)
        main_stream = torch.cuda.current_stream()

        def run(n):
            built = [torch.cuda.Event() for _ in range(n)]
            done = [torch.cuda.Event() for _ in range(n)]

            def build(s):
                with torch.cuda.stream(side):
                    if s >= 2:
                        side.wait_event(done[s - 2])          # the buffers of step s - 2 are free again
                    B.dam_mask_build(params(w.seq - 1 + s, True), None, None, d_in, v_in, bufs[s % 2][3], ws_mask)
                    built[s].record(side)

            build(0)
            for s in range(n):
                if s + 1 < n:
                    build(s + 1)
                main_stream.wait_event(built[s])
                ptr, idx, mem, _ = bufs[s % 2]
                B.dam_sparse_attn_decode_grouped(qs[s], kc, vc, ptr, idx, mem, max_group, out=out, ws=ws_dec, shared_lists=True)
                done[s].record(main_stream)

        side.wait_stream(main_stream)
        run(3)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(n_steps)
        t_host = time.perf_counter() - t0                        # the host's part: if it is the larger one, it is the bound
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / n_steps, t_host * 1e6 / n_steps

    def plan_form(n_steps):
        """The same rows from a position-independent plan of the pattern masks (built once, outside the loop): a step
        is one dam_sparse_attn_decode_patterns call, no list is built."""
        plan = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=w.hq, L=0, S=cap, diag_in=d_in, vert_in=v_in, blocks=False, group=G,
                            plan=True)
        torch.cuda.synchronize()
        longest = int(np.diff(plan.kept_ptr.cpu().numpy()).max())
        ws_p = B.decode_grouped_workspace(dp, longest, dev)

        def step(s):
            B.dam_sparse_attn_decode_patterns(qs[s], kc, vc, plan, w.seq - 1 + s, longest, out=out, ws=ws_p)

        for s in range(3):
            step(s)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(n_steps):          # (no events inside the loop: a pair per step costs 4-5 us of its ~95)
            step(s)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        res = {"steps": n_steps, "us_per_step": wall * 1e6 / n_steps,
               "plan_entries": int(plan.n_kept), "longest_list": longest,
               "decode_us_back_to_back": timed_ms(lambda: step(0), 50) * 1e3}
        if not args.no_graph:
            res["us_per_step_graph_replay"] = graph_replay_ms(lambda: step(0), 50) * 1e3
        return res

    main, (g_ptr, g_idx, g_bound) = form(True, steps)
    planned = plan_form(steps)
    main["us_per_step_list_build_on_a_second_stream"], main["host_us_per_step_of_that_loop"] = overlapped(steps)
    # the merged lists of the first position, kept for the decode from the compacted cache below
    mg = B.build_mask(mode=B.DAM_FROM_PATTERNS, H=w.hq, L=0, S=cap, diag_in=d_in, vert_in=v_in, blocks=False,
                      rows=(w.seq - 1, w.seq), group=G)
    ub = main["list_entries"] * row_bytes                         # the union of the heads' kept rows: what must move
    per_head, (kept_ptr, kept_idx, _) = form(False, min(steps, 64))
    sb = per_head["list_entries"] * row_bytes                     # what moves without sharing between the heads of a group
    per_head["gbs_union"] = ub / (per_head["decode_us"] * 1e-6) / 1e9
    per_head["frac_of_hbm_peak"] = per_head["gbs_union"] / PEAK_HBM_GBS

    # KV eviction at the first timed position: plan, gather into the compacted cache, remap the lists, decode from it
    pos0 = w.seq - 1
    plan = B.kv_evict_plan(d_in, v_in, w.hkv, pos0, batch=w.batch)
    plan_us = timed_ms(lambda: B.kv_evict_plan(d_in, v_in, w.hkv, pos0, batch=w.batch), 5, warm=1) * 1e3
    ccap = int(plan.rows.max().item())
    kcmp = torch.empty((w.batch, w.hkv, ccap, w.head_dim), dtype=torch.bfloat16, device=dev)
    vcmp = torch.empty_like(kcmp)
    slot = torch.empty_like(kept_idx)

    def timed(fn, n):
        return timed_ms(fn, n) * 1e3

    compact_us = timed(lambda: B.kv_compact(plan, kc, vc, kcmp, vcmp), 20)
    live_rows = int(plan.rows.sum().item()) * w.batch
    compact_bytes = live_rows * w.head_dim * 2 * 2 * 2                  # K and V rows, read and written
    remap_us = timed(lambda: B.kv_remap_lists(plan, kept_ptr, kept_idx, 1, out=slot), 20)
    dpc = B.decode_params(qs[0], kcmp, out, shared_lists=True)
    ws_c = B.decode_workspace(dpc, max_kept, dev)
    dec_c_us = timed(lambda: B.dam_sparse_attn_decode(qs[0], kcmp, vcmp, kept_ptr, slot, max_kept, out=out, ws=ws_c,
                                                      shared_lists=True), 50)
    slot_g = B.kv_remap_lists(plan, mg.kept_ptr, mg.kept_idx, 1, per_kv_head=True)
    ws_cg = B.decode_grouped_workspace(dpc, g_bound, dev)
    dec_cg_us = timed(lambda: B.dam_sparse_attn_decode_grouped(qs[0], kcmp, vcmp, mg.kept_ptr, slot_g, mg.kept_member, g_bound,
                                                              out=out, ws=ws_cg, shared_lists=True), 50)
    evict = {"rows_kept_per_kv_head": [int(x) for x in plan.rows.cpu()], "cache_rows": cap,
             "cache_bytes_ratio": ccap / cap, "plan_us_incl_two_host_syncs": plan_us, "compact_us": compact_us, "compact_bytes": compact_bytes,
             "remap_us": remap_us, "decode_from_compacted_us_list_per_head": dec_c_us,
             "decode_from_compacted_us_grouped": dec_cg_us,
             "roofline": {"bound": "hbm", "achieved": compact_bytes / (compact_us * 1e-6) / 1e9, "peak": PEAK_HBM_GBS,
                          "unit": "GB/s", "frac": compact_bytes / (compact_us * 1e-6) / 1e9 / PEAK_HBM_GBS, "traffic": None}}
    del kcmp, vcmp
    dec_us = main["decode_us"]
    res = {"workload": "c5, grouped-query form (one merged kept list per KV head, shared by the batch)"}
    res.update(main)
    res.update({"kept_per_head_list": sb / (w.hq * row_bytes), "union_bytes": ub, "sum_bytes": sb,
                "gbs_union": ub / (dec_us * 1e-6) / 1e9,
                "roofline": {"bound": "hbm", "kernel": "k_decode_group_mfma", "achieved": ub / (dec_us * 1e-6) / 1e9,
                             "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ub / (dec_us * 1e-6) / 1e9 / PEAK_HBM_GBS,
                             "traffic": None,
                             # `achieved` divides by the whole call (partial pass + merge pass) as timed by events inside
                             # the 256-step loop; the same call 50 times in a row, without events in between:
                             "achieved_back_to_back": ub / (main["decode_us_back_to_back"] * 1e-6) / 1e9,
                             "frac_back_to_back": ub / (main["decode_us_back_to_back"] * 1e-6) / 1e9 / PEAK_HBM_GBS},
                "list_per_head_form": per_head, "kv_eviction": evict})
    # the step that builds no list: its whole duration (host clock over the loop) against the same union bytes
    planned["gbs_union"] = ub / (planned["us_per_step"] * 1e-6) / 1e9
    planned["roofline"] = {"bound": "hbm", "kernel": "k_decode_group_mfma<plan>", "achieved": planned["gbs_union"],
                           "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": planned["gbs_union"] / PEAK_HBM_GBS, "traffic": None,
                           "achieved_back_to_back": ub / (planned["decode_us_back_to_back"] * 1e-6) / 1e9,
                           "frac_back_to_back": ub / (planned["decode_us_back_to_back"] * 1e-6) / 1e9 / PEAK_HBM_GBS,
                           "rows_read": planned["plan_entries"] * w.batch, "rows_in_the_union": int(ub // (w.head_dim * 2 * 2))}
    res["pattern_plan_form"] = planned
    return res


def bench_measured_peaks(torch, B):
    """What this chip sustains on nothing but bf16 matrix instructions and on nothing but streaming reads, measured
    in this run (dam_probe_mfma, dam_probe_stream_read): context for the published peaks the fractions divide by.
    The matrix probe is given random operands (the clock a kernel sustains depends on how many bits toggle in the
    multipliers: the chip is power-limited) and, for comparison, zeros."""
    dev = "cuda"
    sink = torch.zeros(4, device=dev)
    out = {}
    for name, ops in (("random_operands", (torch.randn(4096, device=dev) * 0.05).to(torch.bfloat16)),
                      ("zero_operands", torch.zeros(4096, device=dev, dtype=torch.bfloat16))):
        flop = [0.0]

        def run():
            flop[0] = B.probe_mfma(ops, sink, 1024, 1000)
        ms = timed_ms(run, 5, warm=2)
        out["mfma_bf16_tflops_" + name] = flop[0] / (ms * 1e-3) / 1e12
    src = torch.empty(1 << 30, dtype=torch.int32, device=dev).fill_(1)     # 4 GiB
    isink = torch.zeros(4, dtype=torch.int32, device=dev)
    ms = timed_ms(lambda: B.probe_stream_read(src, isink, 8192), 5, warm=2)
    out["hbm_stream_read_gbs"] = src.numel() * 4 / (ms * 1e-3) / 1e9
    out["note"] = ("1024 workgroups x 4 waves x 16000 v_mfma_f32_32x32x16_bf16, two waves per SIMD; 4 GiB read with 16-byte "
                   "non-temporal loads")
    del src
    return out


def bench_small_config(args, torch, B, wl, name):
    """c1 (fp32, S = 256) and c2 (bf16, S = 4096): a step = mask build from the captured map + sparse prefill, and the
    oracle's time for the same outputs (c1 also on one thread)."""
    import oracle
    w = wl.WORKLOADS[name]
    dev = "cuda"
    Q, K, V = wl.qkv_iid(w, std=1 / 8) if name == "c1" else wl.qkv_structured(w)
    A_np = wl.capture_map(Q[:, :w.pcl], K[:, :w.pcl], w.pcl, w.hq // w.hkv)
    A = torch.from_numpy(A_np).to(dev)
    conv = (lambda x: torch.from_numpy(x)[None].to(dev)) if w.dtype == "f32" else \
        (lambda x: torch.from_numpy(x).to(torch.bfloat16)[None].to(dev))
    q, k, v = conv(Q), conv(K), conv(V)
    sized = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=w.hq, L=w.pcl, S=w.seq, tile_m=w.tile_m, tile_n=w.tile_n, lam=w.lam,
                         eps=w.eps, tau=w.tau, mu=w.mu, attn_sum=A)
    torch.cuda.synchronize()
    p = B.MaskParams(B.DAM_FROM_ATTN_MAP, w.hq, w.pcl, w.seq, w.tile_m, w.tile_n, 0, 0, w.lam, w.eps, w.tau, w.mu, float("nan"))
    ws_mask = B.mask_workspace(p, dev)
    o = B.MaskOut()
    for nm in ("true_bits", "diag_cnt", "vert_cnt", "diag_flag", "vert_flag", "bmin", "blk_row_ptr", "blk_col", "blk_kind",
               "tile_bits"):
        setattr(o, nm, getattr(sized, nm).data_ptr())
    total = torch.zeros(1, dtype=torch.int64, device=dev)
    o.blk_capacity, o.blk_total = sized.n_tiles, total.data_ptr()
    out = torch.empty_like(q)
    ws_attn = B.prefill_workspace(B.attn_params(q, k, v, out, w.tile_m, w.tile_n), dev)

    def step(ev):
        ev[0].record()
        B.dam_mask_build(p, A, None, None, None, o, ws_mask)
        ev[1].record()
        B.dam_sparse_attn_prefill(q, k, v, sized, out=out, ws=ws_attn)
        ev[2].record()

    for _ in range(3):
        step(events(3))
    torch.cuda.synchronize()
    evs = [events(3) for _ in range(args.steps)]
    for e in evs:
        step(e)
    torch.cuda.synchronize()
    nnz = int(np.unpackbits(sized.tile_bits.cpu().numpy().view(np.uint8)).sum(dtype=np.int64))
    step_ms = float(np.median([e[0].elapsed_time(e[2]) for e in evs]))
    attn_ms = float(np.median([e[1].elapsed_time(e[2]) for e in evs]))
    flops = 4.0 * w.head_dim * nnz
    res = {"workload": f"{name}: {w.hq} Q / {w.hkv} KV heads, head_dim {w.head_dim}, seq {w.seq}, capture length {w.pcl}, "
                       f"{w.dtype}, tiles {w.tile_m}x{w.tile_n}; step = mask build from the map + sparse prefill",
           "step_ms": step_ms, "mask_build_ms": float(np.median([e[0].elapsed_time(e[1]) for e in evs])), "prefill_ms": attn_ms,
           "nnz": nnz, "density": nnz / (w.hq * w.seq * (w.seq + 1) / 2), "listed_tiles": sized.n_tiles,
           "tflops_kept_step": flops / (step_ms * 1e-3) / 1e12, "tflops_kept_prefill": flops / (attn_ms * 1e-3) / 1e12}
    if not args.no_cpu:
        art = oracle.derive(A_np, None, w.lam, w.eps, w.tau, w.mu)
        t0 = time.perf_counter()
        oracle.attend_prefill(Q, K, V, art)
        dt = time.perf_counter() - t0
        res["oracle"] = {"seconds": dt, "tflops_kept": flops / dt / 1e12, "cores": oracle.threads(), "what": "every output row, fp64"}
        if name == "c1":
            try:
                from threadpoolctl import threadpool_limits
                with threadpool_limits(limits=1, user_api="openmp"):
                    t0 = time.perf_counter()
                    oracle.attend_prefill(Q, K, V, art)
                    dt1 = time.perf_counter() - t0
                res["oracle_single_thread"] = {"seconds": dt1, "tflops_kept": flops / dt1 / 1e12, "cores": 1}
            except Exception as e:     # the limiter is optional: without it only the all-threads time is reported
                res["oracle_single_thread"] = {"unavailable": repr(e)}
    return res


def bench_mask_from_map(args, torch, B, wl, name):
    """a1-a3 from a captured attention map (true mask + matched patterns at S = L), and for c4 also the
    whole build at the configuration's S (extension, block index, tile pool)."""
    w = wl.WORKLOADS[name]
    Q, K, V = wl.qkv_structured(w)
    H, L = w.hq, w.pcl
    A = torch.from_numpy(wl.capture_map(Q[:, :L], K[:, :L], L, w.hq // w.hkv)).cuda()
    q_cap = torch.from_numpy(np.ascontiguousarray(Q[:, :L])).to(torch.bfloat16).cuda()
    k_cap = torch.from_numpy(np.ascontiguousarray(K[:, :L])).to(torch.bfloat16).cuda()
    qkv_full = None
    if name == "c4":   # the whole sequence, for the prefill over the extended masks
        qkv_full = tuple(torch.from_numpy(x).to(torch.bfloat16)[None].cuda() for x in (Q, K, V))
    del Q, K, V

    timed = timed_ms

    p = B.MaskParams(B.DAM_FROM_ATTN_MAP, H, L, L, 128, 128, 0, 0, w.lam, w.eps, w.tau, w.mu, float("nan"))
    ws = B.mask_workspace(p, "cuda")
    o = B.MaskOut()
    tb = torch.empty((H, L, L // 64), dtype=torch.int64, device="cuda")
    fl = [torch.empty((H, L), dtype=torch.uint8, device="cuda") for _ in range(2)]
    o.true_bits, o.diag_flag, o.vert_flag = tb.data_ptr(), fl[0].data_ptr(), fl[1].data_ptr()
    ms = timed(lambda: B.dam_mask_build(p, A, None, None, None, o, ws), 20)
    nbytes = 2 * H * L * (L + 1) + H * L * L // 8      # lower triangle of A once + true bits
    ms_graph = None if args.no_graph else graph_replay_ms(lambda: B.dam_mask_build(p, A, None, None, None, o, ws), 20)
    res = {"workload": f"{name} map ({H} x {L} x {L} fp32) -> true mask + matched patterns", "ms": ms, "ms_graph_replay": ms_graph,
           "bytes": nbytes,
           "roofline": {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": None}}
    # the same stage one fused with its capture (no map), and the capture alone summed into A and C
    cp = B.capture_params(q_cap, k_cap, L)
    ws_f = B.mask_from_qk_workspace(p, cp, "cuda")
    ms_f = timed(lambda: B.dam_mask_build_from_qk(p, cp, q_cap, k_cap, o, ws_f), 20)
    flops = 2.0 * w.head_dim * H * L * (L + 1) / 2     # one Q K^T over the causal triangle (the kernels take two)
    res["fused_capture"] = {"workload": f"{name} capture (Q, K of {L} tokens, {H} heads) -> true mask + matched patterns, no map",
                            "ms": ms_f, "flops": flops,
                            "roofline": {"bound": "mfma", "achieved": flops / (ms_f * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS,
                                         "unit": "TFLOP/s", "frac": flops / (ms_f * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                                         "traffic": None}}
    a_sum = torch.zeros((H, L, L), dtype=torch.float32, device="cuda")
    a_cnt = torch.zeros((H, L, L), dtype=torch.float32, device="cuda")
    ws_c = B.capture_workspace(cp, "cuda")
    ms_a = timed(lambda: B.dam_capture_accumulate(q_cap, k_cap, a_sum, a_cnt, ws=ws_c), 5)
    acc_bytes = 16.0 * H * L * (L + 1) / 2             # A and C, lower triangle, read and written
    res["capture_accumulate"] = {"workload": f"{name} capture summed into A and C ({H} x {L} x {L} fp32 each)", "ms": ms_a,
                                 "bytes": acc_bytes,
                                 "roofline": {"bound": "hbm", "achieved": acc_bytes / (ms_a * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                                              "unit": "GB/s", "frac": acc_bytes / (ms_a * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                              "traffic": None}}
    del a_sum, a_cnt, q_cap, k_cap
    if name == "c4":
        S = w.seq
        sized = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=H, L=L, S=S, lam=w.lam, eps=w.eps, tau=w.tau, mu=w.mu, attn_sum=A)
        torch.cuda.synchronize()
        p2 = B.MaskParams(B.DAM_FROM_ATTN_MAP, H, L, S, 128, 128, 0, 0, w.lam, w.eps, w.tau, w.mu, float("nan"))
        ws2 = B.mask_workspace(p2, "cuda")
        o2 = B.MaskOut()
        tb_map = tb
        o2.true_bits, o2.diag_flag, o2.vert_flag = tb.data_ptr(), fl[0].data_ptr(), fl[1].data_ptr()
        tot = torch.zeros(1, dtype=torch.int64, device="cuda")
        o2.blk_row_ptr, o2.blk_col, o2.blk_kind = sized.blk_row_ptr.data_ptr(), sized.blk_col.data_ptr(), sized.blk_kind.data_ptr()
        o2.tile_bits, o2.blk_capacity, o2.blk_total = sized.tile_bits.data_ptr(), sized.n_tiles, tot.data_ptr()
        ms2 = timed(lambda: B.dam_mask_build(p2, A, None, None, None, o2, ws2), 10)
        nb2 = nbytes + sized.n_tiles * (128 * 128 // 8 + 5) + 4 * H * (S // 128 + 1)
        res["whole_build"] = {"seq": S, "listed_tiles": sized.n_tiles, "ms": ms2, "bytes": nb2,
                              "roofline": {"bound": "hbm", "achieved": nb2 / (ms2 * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                                           "unit": "GB/s", "frac": nb2 / (ms2 * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": None}}
        # prefill over the 128k masks: plain layout, and with the matched columns gathered (the method's stripes)
        qf, kf, vf = qkv_full
        outf = torch.empty_like(qf)
        lut = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device="cuda")
        pre = {}
        for label, mk in (("plain", sized), ("gathered", None)):
            if mk is None:
                del sized
                torch.cuda.empty_cache()
                mk = B.build_mask(mode=B.DAM_FROM_ATTN_MAP, H=H, L=L, S=S, lam=w.lam, eps=w.eps, tau=w.tau, mu=w.mu, attn_sum=A,
                                  flags=B.DAM_MASK_SKIP_FULL_TILE_BITS | B.DAM_MASK_GATHER_COLUMNS)
                torch.cuda.synchronize()
            wsf = B.prefill_workspace(B.attn_params(qf, kf, vf, outf, 128, 128, gather_rows=mk.gather_rows), "cuda")
            ms_p = timed(lambda: B.dam_sparse_attn_prefill(qf, kf, vf, mk, out=outf, ws=wsf), 5)
            ms_b = None
            if label == "gathered":   # the build of the layout this prefill reads (full tiles without bits, columns gathered)
                fl_g = B.DAM_MASK_SKIP_FULL_TILE_BITS | B.DAM_MASK_GATHER_COLUMNS
                p3 = B.MaskParams(B.DAM_FROM_ATTN_MAP, H, L, S, 128, 128, 0, 0, w.lam, w.eps, w.tau, w.mu, float("nan"), fl_g)
                ws3 = B.mask_workspace(p3, "cuda")
                o3 = B.MaskOut()
                o3.true_bits, o3.diag_flag, o3.vert_flag = tb_map.data_ptr(), fl[0].data_ptr(), fl[1].data_ptr()
                o3.blk_row_ptr, o3.blk_col, o3.blk_kind = mk.blk_row_ptr.data_ptr(), mk.blk_col.data_ptr(), mk.blk_kind.data_ptr()
                o3.tile_bits, o3.blk_capacity, o3.blk_total = mk.tile_bits.data_ptr(), mk.n_tiles, tot.data_ptr()
                o3.gather_idx, o3.gather_cnt = mk.gather_idx.data_ptr(), mk.gather_cnt.data_ptr()
                ms_b = timed(lambda: B.dam_mask_build(p3, A, None, None, None, o3, ws3), 10)
                del ws3
            kd = mk.blk_kind.cpu().numpy()
            part = (mk.blk_kind & 1) == 0
            nnz = int((kd & 1).sum()) * 128 * 128
            for a0 in range(0, mk.n_tiles, 1 << 17):
                tb = mk.tile_bits[a0:a0 + (1 << 17)][part[a0:a0 + (1 << 17)]].view(torch.uint8).reshape(-1)
                nnz += int(lut[tb.long()].sum().item())
            pre[label] = {"listed_tiles": mk.n_tiles, "key_blocks_of_32": int(np.unpackbits((kd >> 1)[:, None].astype(np.uint8), axis=1).sum()),
                          "prefill_ms": ms_p, "nnz": nnz, "tflops_kept_entries": 4.0 * w.head_dim * nnz / (ms_p * 1e-3) / 1e12,
                          "frac_of_bf16_peak": 4.0 * w.head_dim * nnz / (ms_p * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
            if ms_b is not None:
                pre[label]["mask_build_ms"] = ms_b
                pre[label]["step_ms"] = ms_b + ms_p
                pre[label]["tflops_kept_entries_step"] = 4.0 * w.head_dim * nnz / ((ms_b + ms_p) * 1e-3) / 1e12
            del wsf
        res["prefill_128k"] = pre
    return res


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2506_11104_amd import binding as B
    from paper_2506_11104_amd import workloads as wl
    B.lib()                                   # fails loudly when libdam.so is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = wl.WORKLOADS[args.workload]
    if args.copy_calibration:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda")   # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    res, ctx = bench_prefill(args, w, torch, B, wl)
    line = {
        "metric": "effective TFLOP/s on kept entries (mask build + sparse prefill per step, 32k prefill)",
        "value": res["tflops_kept_step"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["step_ms"], "ms_per_step_mean_host_clock": res["step_ms_mean_host_clock"],
        "timing": "median of the timed steps, HIP events on the launch stream", "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: 1 layer, {w.hq} Q / {w.hkv} KV heads, head_dim {w.head_dim}, seq {w.seq}, "
                               f"bf16, batch 1, heterogeneous per-head masks, tiles {w.tile_m}x{w.tile_n}",
                   "density": res["density"], "nnz": res["nnz"], "listed_tiles": res["n_tiles"],
                   "full_tiles": res["n_full_tiles"], "tile_fill": res["tile_fill"],
                   "gathered_column_tiles": res["gathered_tiles"], "key_blocks_of_32": res["n_blocks"]},
        "ms_per_layer_prefill": res["prefill_ms"], "mask_build_ms": res["mask_build_ms"],
        "mask_build_gbs": res["mask_build_gbs"],
        "tflops_kept_entries_prefill_only": res["tflops_kept_prefill"],
        "tflops_issued_blocks_prefill_only": res["tflops_blocks_prefill"],
        "roofline": {"bound": "mfma", "kernel": "k_prefill_bf16_pipe", "achieved": res["tflops_kept_prefill"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": res["tflops_kept_prefill"] / PEAK_BF16_TFLOPS,
                     "traffic": None,
                     # the matrix work of the occupied 32-key blocks of the listed tiles, 4 * head_dim * 128 * 32 each
                     # (empty key quarters of a tile are not visited): the figure "on kept tiles". The kernel issues a
                     # few per cent fewer matrix instructions than that: a wave whose 32 x 32 square of a block holds
                     # no kept entry does not run that square's Q K^T products
                     "achieved_issued_blocks": res["tflops_blocks_prefill"],
                     "frac_issued_blocks": res["tflops_blocks_prefill"] / PEAK_BF16_TFLOPS,
                     "plain_layout": res["plain_layout"]},
    }
    if not args.no_cpu:
        line["cpu_baseline"] = bench_cpu_oracle(args, w, ctx, wl)
    del ctx
    torch.cuda.empty_cache()
    line["roofline"]["measured_on_this_chip"] = bench_measured_peaks(torch, B)
    line["peaks_used"] = {"bf16_mfma_tflops": PEAK_BF16_TFLOPS, "hbm_gbs": PEAK_HBM_GBS, "source": "published"}
    if not args.no_small:
        line["c1"] = bench_small_config(args, torch, B, wl, "c1")
        line["c2"] = bench_small_config(args, torch, B, wl, "c2")
        torch.cuda.empty_cache()
    if not args.no_maskmap:
        line["mask_build_from_map"] = bench_mask_from_map(args, torch, B, wl, "c2")
        torch.cuda.empty_cache()
        line["mask_build_from_map_c4"] = bench_mask_from_map(args, torch, B, wl, "c4")
        torch.cuda.empty_cache()
    if not args.no_decode:
        # The sections before this one leave the chip hot (seconds of matrix work at S = 131072), which costs the
        # HBM-bound decode 3-4 %: it starts from an idle chip, like the headline section at the top.
        time.sleep(args.pause_before_decode)
        line["decode"] = bench_decode(args, torch, B, wl)
        line["decode"]["idle_seconds_before"] = args.pause_before_decode
    print(json.dumps(line))


if __name__ == "__main__":
    main()
