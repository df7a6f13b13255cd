#!/usr/bin/env python3
"""Benchmark of the Double-P decode step on one MI355X.

A "step" is one call of dp_decode_attention: one layer's hierarchical top-p
sparse attention for one decode token (centroid scoring, both top-p selections,
sparse decode, split combine) over a synthetic clustered KV cache that is
already resident in HBM.  Successive steps run on DIFFERENT replicas of the
layer's buffers (distinct device addresses, like the layers of a model), enough
of them that neither L2 nor the 256 MB Infinity Cache can hold what a step
reads; all steps are enqueued back-to-back on one stream.

Prints ONE JSON line:  metric/value = microseconds per decode step per layer,
plus `roofline` (the kernel that moves the bytes, against the 8 TB/s HBM peak)
and `cpu_baseline` (the fp64 CPU oracle timed on the host cores of this machine).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
CACHE_BYTES = 256e6 + 32e6          # Infinity Cache + 8 x 4 MB L2


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3600)
    ap.add_argument("--warmup", type=int, default=360)
    ap.add_argument("--config", type=int, default=2, help="workload index 0..4 (default: 8B shape, 128k context)")
    ap.add_argument("--heads", choices=["flat", "mixed"], default=None,
                    help="workloads 1 and 2 with other query scales: every head flat, or one in eight (the cases "
                         "behind the launch policy; see ab_paper_kernel_structure_us.decode_launch in the line)")
    ap.add_argument("--replicas", type=int, default=0, help="layer replicas to rotate over (0 = auto)")
    ap.add_argument("--separate-decode-launch", action="store_true",
                    help="A/B: keep the split decode a launch of its own (DP_FLAG_SEPARATE_DECODE_LAUNCH)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="CPU time budget of the oracle baseline")
    return ap.parse_args()


def algorithmic_bytes(cache, sel, n_exact, n_retained):
    """HBM bytes one step must move: key centroids + sizes once per KV segment, K+V rows of every
    selected token and the two centroid rows of every approximated cluster (each counted once per KV
    segment: the union over the query heads that share it), q in and o out."""
    import numpy as np
    d2 = 2 * cache.head_dim
    G = cache.group
    total_k = int(cache.seg_cluster_ptr[-1])
    scan = total_k * (d2 + 4)
    rows_union = rows_sum = 0
    for b in range(cache.batch):
        for g in range(cache.n_kv_heads):
            seg = b * cache.n_kv_heads + g
            c0 = int(cache.seg_cluster_ptr[seg])
            ex_u, ap_u = set(), set()
            for j in range(G):
                i = b * cache.n_q_heads + g * G + j
                ex = sel[i, : n_exact[i]]
                ap = sel[i, n_exact[i]: n_retained[i]]
                rows_sum += int(cache.cluster_sizes[c0 + ex].sum()) + len(ap)
                ex_u.update(ex.tolist())
                ap_u.update(ap.tolist())
            ap_u -= ex_u
            rows_union += int(cache.cluster_sizes[c0 + np.fromiter(ex_u, dtype=np.int64, count=len(ex_u))].sum()) \
                + len(ap_u)
    io = cache.batch * cache.n_q_heads * cache.head_dim * (2 + 4)
    return dict(scan=scan, rows_union=rows_union, rows_sum=rows_sum, total=scan + rows_union * 2 * d2 + io,
                total_per_head_sum=scan + rows_sum * 2 * d2 + io)


def total_clusters_nonzero(cache):
    return int(cache.seg_cluster_ptr[-1]) > 0 and (cache.seg_cluster_ptr[1:] > cache.seg_cluster_ptr[:-1]).all()


def measured_traffic(kernel, config):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary
    (FETCH_SIZE and WRITE_SIZE, scaled by what a plain copy of known size reads); None if there is none."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_cfg{config}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return int(float(line.split("=")[1].split()[0]))
    except OSError:
        pass
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); rerun with --gpus 1. "
              "value is the one GPU's throughput.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2602_05191_amd as dp
    from workloads import CONFIGS, make_config

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    t0 = time.time()
    cache = make_config(args.config, heads=args.heads)
    wname = CONFIGS[args.config] + (f" with {args.heads} heads" if args.heads else "")
    t_gen = time.time() - t0
    p1, p2 = cache.p1, cache.p2
    nh = cache.batch * cache.n_q_heads
    mk = cache.max_clusters_per_seg

    base = dp.DeviceCache.from_host(cache, dev)
    pflags = dp.DP_FLAG_SEPARATE_DECODE_LAUNCH if args.separate_decode_launch else 0
    pr0 = dp.Problem(base, flags=pflags)
    ws_bytes = dp.dp_workspace_bytes(pr0)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=dev)
    out = torch.empty((cache.batch, cache.n_q_heads, cache.head_dim), dtype=torch.float32, device=dev)
    lse = torch.empty(nh, dtype=torch.float32, device=dev)
    ne = torch.empty(nh, dtype=torch.int32, device=dev)
    nr, nt = torch.empty_like(ne), torch.empty_like(ne)

    # one step to learn what the method touches on this input
    dp.dp_decode_attention(pr0, p1, p2, out, lse, ws, ne, nr, nt)
    torch.cuda.synchronize()
    lay = dp.dp_workspace_layout(pr0)
    sel = ws[lay["sel_ids"]: lay["sel_ids"] + 4 * nh * mk].cpu().numpy().view(np.int32).reshape(nh, mk)
    ne_h, nr_h, nt_h = ne.cpu().numpy(), nr.cpu().numpy(), nt.cpu().numpy()
    alg = algorithmic_bytes(cache, sel, ne_h, nr_h)

    # replicas at distinct addresses: twice the on-chip cache capacity worth of touched bytes
    L = args.replicas or int(min(64, max(2, math.ceil(2 * CACHE_BYTES / max(alg["total"], 1)))))
    free, _ = torch.cuda.mem_get_info()
    per_replica = sum(t.numel() * t.element_size() for t in base.__dict__.values() if isinstance(t, torch.Tensor))
    L = int(max(1, min(L, (free * 0.8) // max(per_replica, 1))))
    reps = [base] + [base.clone() for _ in range(L - 1)]
    probs = [dp.Problem(r, flags=pflags) for r in reps]
    torch.cuda.synchronize()

    # one step per replica with its arguments marshalled once (what a serving loop does): the timed loop then only
    # calls into the library
    bound = [dp.BoundDecodeStep(pr, p1, p2, out, lse, ws) for pr in probs]

    def step(i):
        bound[i % L]()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # The timed region: exactly args.steps steps between two synchronisations, wall clock.  It is taken three times
    # and the median region is reported (a host hiccup of some ten milliseconds inside a 70 ms region is not the
    # library's time); all three are in the JSON line.
    regions = []
    for _ in range(3):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        ev0.record()
        for i in range(args.steps):
            step(i)
        ev1.record()
        torch.cuda.synchronize()
        w1 = time.perf_counter()
        regions.append(((w1 - w0) * 1e6 / args.steps, ev0.elapsed_time(ev1) * 1e3 / args.steps))
    wall_us, event_us = sorted(regions)[1]

    # spread of the step time: one rotation over the L replicas at a time between two events on the launch stream
    # (an event costs a bubble, so these rotations are not the reported value); p10 / median / p90 of rotation / L
    n_rot = max(50, min(200, args.steps // max(L, 1)))  # at least 50 timed rotations after 5 untimed ones
    rot_ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_rot + 1)]
    for i in range(5 * L):
        step(i)
    torch.cuda.synchronize()
    rot_ev[0].record()
    for r in range(n_rot):
        for i in range(L):
            step(i)
        rot_ev[r + 1].record()
    torch.cuda.synchronize()
    rot_us = sorted(rot_ev[r].elapsed_time(rot_ev[r + 1]) * 1e3 / L for r in range(n_rot))
    pct = lambda q: rot_us[min(n_rot - 1, int(q * n_rot))]

    # the paper's own operating point (p1, p2) = (0.95, 0.7) of its ablation (Sec. 5.4), same inputs
    torch.cuda.synchronize()
    o0 = time.perf_counter()
    for i in range(min(args.steps, 720)):
        dp.dp_decode_attention(probs[i % L], 0.95, 0.7, out, lse, ws, None, None, None)
    torch.cuda.synchronize()
    op_us = (time.perf_counter() - o0) * 1e6 / min(args.steps, 720)
    dp.dp_decode_attention(pr0, 0.95, 0.7, out, lse, ws, ne, nr, nt)
    torch.cuda.synchronize()
    op_counts = (float(nr.float().mean()), float(ne.float().mean()), float(nt.float().mean()))
    dp.dp_decode_attention(pr0, p1, p2, out, lse, ws, ne, nr, nt)
    torch.cuda.synchronize()

    # same-layer repeat (everything cache-resident), labelled as such
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    for i in range(min(args.steps, 500)):
        step(0)
    torch.cuda.synchronize()
    resident_us = (time.perf_counter() - c0) * 1e6 / min(args.steps, 500)

    # ---- per-stage launch durations, HIP events on the launch stream (torch's current stream) ----
    n_logits = cache.group * int(cache.seg_cluster_ptr[-1])
    logits = torch.empty(n_logits, dtype=torch.float32, device=dev)
    sel_d = torch.empty((nh, mk), dtype=torch.int32, device=dev)
    n_stage = min(args.steps, 720)

    def time_stage(fn):
        """Average duration of one launch in a back-to-back stream of n_stage launches (rotating
        replicas), from one pair of HIP events on the launch stream; median over 5 such runs."""
        for i in range(min(50, n_stage)):
            fn(i)
        torch.cuda.synchronize()
        runs = []
        for _ in range(5):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for i in range(n_stage):
                fn(i)
            b.record()
            torch.cuda.synchronize()
            runs.append(a.elapsed_time(b) * 1e3 / n_stage)
        return statistics.mean(runs), statistics.median(runs)

    score_gap_us, _ = time_stage(lambda i: dp.dp_score_centroids(probs[i % L], logits))

    # What this machine streams: the loads-only probe (dp_stream_read_probe) over the same key-centroid matrices,
    # back to back over the replicas like the scoring launches (the floor for one launch of that size), and over
    # the whole K cache of the replicas (the streaming-read bandwidth of the box)
    scan_bytes = base.k_centroids.numel() * base.k_centroids.element_size()
    read_floor_gap_us, _ = time_stage(lambda i: dp.dp_stream_read_probe(reps[i % L].k_centroids))
    big = [r.k_cache for r in reps]
    big_bytes = big[0].numel() * big[0].element_size()
    for i in range(min(L, 4)):
        dp.dp_stream_read_probe(big[i])
    torch.cuda.synchronize()
    b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_big = max(4, min(64, int(8e9 // max(big_bytes, 1))))
    b0.record()
    for i in range(n_big):
        dp.dp_stream_read_probe(big[i % L])
    b1.record()
    torch.cuda.synchronize()
    stream_gbs = big_bytes * n_big / (b0.elapsed_time(b1) * 1e-3) / 1e9

    # The scoring kernel's own duration: every launch carries a pair of HIP events that the runtime stamps
    # with the kernel's begin and end (dp_score_centroids_timed), launched back-to-back on the same stream.
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    pairs = []
    for _ in range(n_stage):
        e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0
        pairs.append((e0, e1))
    for i in range(50):
        dp.dp_score_centroids(probs[i % L], logits)
    torch.cuda.synchronize()
    for i, (e0, e1) in enumerate(pairs):
        dp.dp_score_centroids_timed(probs[i % L], logits, e0, e1)
    torch.cuda.synchronize()
    durs = []
    for e0, e1 in pairs:
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
        durs.append(ms.value * 1e3)
        hip.hipEventDestroy(e0)
        hip.hipEventDestroy(e1)
    score_us, score_med = statistics.mean(durs), statistics.median(durs)
    # the same for the loads-only probe over the same matrices: the kernel's own duration
    pairs = []
    for _ in range(n_stage):
        e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0
        pairs.append((e0, e1))
    for i, (e0, e1) in enumerate(pairs):
        dp.dp_stream_read_probe(reps[i % L].k_centroids, None, None, e0, e1)
    torch.cuda.synchronize()
    durs = []
    for e0, e1 in pairs:
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
        durs.append(ms.value * 1e3)
        hip.hipEventDestroy(e0)
        hip.hipEventDestroy(e1)
    read_floor_us = statistics.mean(durs)

    # The three kernels inside the one-call path: dp_decode_attention_timed stamps each kernel's begin and end.
    n_in = min(n_stage, 360)
    sets = []
    for _ in range(n_in):
        ev = [ctypes.c_void_p() for _ in range(6)]
        for e in ev:
            assert hip.hipEventCreate(ctypes.byref(e)) == 0
        sets.append(ev)
    for i in range(min(50, n_in)):
        step(i)
    torch.cuda.synchronize()
    for i, ev in enumerate(sets):
        dp.dp_decode_attention_timed(probs[i % L], p1, p2, out, lse, ws, ev)
    torch.cuda.synchronize()

    def elapsed(a, b):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return ms.value * 1e3

    in_step = {k: [] for k in ("score", "select", "decode", "gap_score_select", "gap_select_decode")}
    for ev in sets:
        in_step["score"].append(elapsed(ev[0], ev[1]))
        in_step["select"].append(elapsed(ev[2], ev[3]))
        in_step["decode"].append(elapsed(ev[4], ev[5]))
        in_step["gap_score_select"].append(elapsed(ev[1], ev[2]))
        in_step["gap_select_decode"].append(elapsed(ev[3], ev[4]))
        for e in ev:
            hip.hipEventDestroy(e)
    n_launches = dp.dp_decode_attention_launches(pr0)
    shared_launch = n_launches == 2      # the split decode runs inside the selection launch: no third kernel
    if shared_launch:
        for k in ("decode", "gap_select_decode"):
            in_step[k] = [0.0] * len(in_step[k])
    in_step_avg = {k: statistics.mean(v) for k, v in in_step.items()}
    in_step_med = {k: statistics.median(v) for k, v in in_step.items()}
    select_us, select_med = time_stage(lambda i: dp.dp_topp_select(probs[i % L], logits, p1, p2, sel_d, ne, nr, nt))
    decode_us, decode_med = time_stage(lambda i: dp.dp_sparse_decode(probs[i % L], sel_d, ne, nr, out, lse, ws))

    # ---- same-box baselines in the shape of the paper's efficiency comparison (Sec. 5.3): full attention
    # over every token, and a fixed top-k cluster budget (1.8 % of the clusters exact, 25 % retained) ----
    seg_rows_h = np.add.reduceat(cache.cluster_sizes.astype(np.int64), cache.seg_cluster_ptr[:-1].astype(np.int64)) \
        if total_clusters_nonzero(cache) else np.zeros(cache.batch * cache.n_kv_heads, np.int64)
    seg_rows = torch.from_numpy(seg_rows_h.astype(np.int32)).to(dev)
    k_ret, k_ex = max(1, mk // 4), max(1, round(mk * 0.018))

    def wall_time(fn, n):
        for i in range(min(n, 20)):
            fn(i)
        torch.cuda.synchronize()
        a = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - a) * 1e6 / n

    n_base = max(10, min(args.steps, 200))
    dense_us = wall_time(lambda i: dp.dp_dense_decode(probs[i % L], seg_rows, out, lse, ws), n_base)
    budget_us = wall_time(lambda i: dp.dp_budget_decode_attention(probs[i % L], k_ret, k_ex, out, lse, ws), n_base)
    dense_bytes = int(seg_rows_h.sum()) * 4 * cache.head_dim + nh * cache.head_dim * 6
    # leave the top-p step's result in out / lse for the check against the oracle below
    dp.dp_decode_attention(pr0, p1, p2, out, lse, ws, None, None, None)
    torch.cuda.synchronize()

    # ---- the step with the sink and window clusters pinned (what the paper's runs do at every layer, Sec. 5.1):
    # first cluster and last four clusters of every KV head always exact and outside the distribution ----
    from workloads import pin_sink_and_window
    pinned_flags = torch.from_numpy(pin_sink_and_window(cache, first=1, last=4).cluster_flags).to(dev)
    cache.cluster_flags = None
    pinned_probs = []
    for r in reps:
        pc = dp.DeviceCache(**{**r.__dict__, "cluster_flags": pinned_flags})
        pinned_probs.append(dp.Problem(pc))
    pinned_us = wall_time(lambda i: dp.dp_decode_attention(pinned_probs[i % L], p1, p2, out, lse, ws), n_base)
    dp.dp_decode_attention(pr0, p1, p2, out, lse, ws, None, None, None)
    torch.cuda.synchronize()

    # ---- A/B against the kernel structure the paper describes for its own implementation (Sec. 4.4): top-p on
    # sorted scores, and gathering the selected rows into a contiguous buffer before attending.  Same results
    # (tested bit-identical); staged entry points, back-to-back launches over the rotating replicas. ----
    ab = {"dp_topp_select_us": round(select_us, 3), "dp_sparse_decode_us": round(decode_us, 3)}
    if mk <= 8192:
        dp.dp_score_centroids(pr0, logits)
        ab["dp_topp_select_sorted_us"] = round(time_stage(
            lambda i: dp.dp_topp_select_sorted(probs[i % L], logits, p1, p2, sel_d, ne, nr, nt))[0], 3)
    dp.dp_topp_select(pr0, logits, p1, p2, sel_d, ne, nr, nt)
    torch.cuda.synchronize()
    cap = int(nt.max().item()) + 1
    if nh * cap * cache.head_dim * 4 <= 2 ** 34:
        kb = torch.empty((nh, cap, cache.head_dim), dtype=torch.int16, device=dev)
        vb = torch.empty_like(kb)
        ab["dp_sparse_decode_gathered_us"] = round(time_stage(
            lambda i: dp.dp_sparse_decode_gathered(probs[i % L], sel_d, ne, nr, out, lse, kb, vb, cap, ws))[0], 3)
        ab["gather_buffer_rows_per_head"] = cap
        del kb, vb

    # ---- A/B: selection per GQA group (every head of a group attends over the union of the group's per-head
    # sets, so a row is read once per group; NOT the same result: each head attends a superset of its own sets).
    # Whole step, wall clock, same rotating replicas; the rows each variant attends are reported next to it. ----
    n_seg = cache.batch * cache.n_kv_heads
    u_ids = torch.empty((n_seg, max(mk, 1)), dtype=torch.int32, device=dev)
    u_ne = torch.empty(n_seg, dtype=torch.int32, device=dev)
    u_nr = torch.empty(n_seg, dtype=torch.int32, device=dev)
    union_us = wall_time(lambda i: dp.dp_group_union_decode_attention(probs[i % L], p1, p2, out, lse, u_ids, u_ne, u_nr, ws),
                         n_base)
    dp.dp_group_union_decode_attention(pr0, p1, p2, out, lse, u_ids, u_ne, u_nr, ws)
    torch.cuda.synchronize()
    u_ids_h, u_ne_h, u_nr_h = u_ids.cpu().numpy(), u_ne.cpu().numpy(), u_nr.cpu().numpy()
    union_rows = 0
    for seg in range(n_seg):
        c0 = int(cache.seg_cluster_ptr[seg])
        union_rows += int(cache.cluster_sizes[c0 + u_ids_h[seg, :u_ne_h[seg]]].sum()) + int(u_nr_h[seg] - u_ne_h[seg])
    ab["group_union"] = {"entry_point": "dp_group_union_decode_attention", "step_us": round(union_us, 3),
                         "rows_read_once_per_group": union_rows,
                         "rows_attended_per_head_times_heads": union_rows * cache.group,
                         "note": "every head attends the union of its group's sets: a superset of its own"}
    dp.dp_decode_attention(pr0, p1, p2, out, lse, ws, None, None, None)
    torch.cuda.synchronize()

    # ---- A/B: the split decode inside the selection launch (two launches per step) against a decode launch of
    # its own (three): the same step with DP_FLAG_SEPARATE_DECODE_LAUNCH set / cleared, wall clock, same replicas ----
    probs_sep = [dp.Problem(r, flags=dp.DP_FLAG_SEPARATE_DECODE_LAUNCH) for r in reps]
    probs_def = [dp.Problem(r) for r in reps]
    n_ab = max(10, min(args.steps, 720))
    ab["decode_launch"] = {
        "default_policy_launches": dp.dp_decode_attention_launches(probs_def[0]),
        "default_policy_us": round(wall_time(lambda i: dp.dp_decode_attention(probs_def[i % L], p1, p2, out, lse, ws), n_ab), 3),
        "separate_decode_launch_us": round(wall_time(lambda i: dp.dp_decode_attention(probs_sep[i % L], p1, p2, out, lse, ws), n_ab), 3),
    }
    dp.dp_decode_attention(pr0, p1, p2, out, lse, ws, None, None, None)
    torch.cuda.synchronize()

    # ---- the prefill-side build of this workload's cache (Sec. 4.1, Eq. 2): token-order K / V + cluster ids ->
    # cluster-contiguous rows, sizes, offsets, centroids.  One call per layer, not part of the decode step. ----
    from workloads import token_order_input
    tok = token_order_input(cache, seed=1)
    up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)
    pf = dp.Prefill(up(tok.k_tokens, np.int16), up(tok.v_tokens, np.int16), up(tok.assignment, np.int32),
                    base.seg_row_base, up(tok.seg_rows, np.int32), base.seg_cluster_ptr, base.total_clusters, mk,
                    int(tok.seg_rows.max()))
    bws = torch.empty(max(dp.dp_build_workspace_bytes(pf), 256), dtype=torch.uint8, device=dev)
    b_k, b_v = torch.empty_like(base.k_cache), torch.empty_like(base.v_cache)
    b_off, b_sz = torch.empty_like(base.cluster_offsets), torch.empty_like(base.cluster_sizes)
    b_kc, b_vc = torch.empty_like(base.k_centroids), torch.empty_like(base.v_centroids)
    build_us = wall_time(lambda i: dp.dp_build_cluster_cache(pf, b_k, b_v, b_off, b_sz, b_kc, b_vc, bws), 20)
    build_bytes = int(tok.k_tokens.shape[0]) * (2 * 512 + 4)   # K+V rows read once and written once (the means are taken on the way); ids
    # the assignment step of the clustering itself (one Lloyd iteration = this + the build): a dense
    # tokens x centroids x 128 contraction on the matrix cores
    kws = torch.empty(max(dp.dp_kmeans_workspace_bytes(pf), 256), dtype=torch.uint8, device=dev)
    k_asg = torch.empty(int(tok.k_tokens.shape[0]), dtype=torch.int32, device=dev)
    kmeans_us = wall_time(lambda i: dp.dp_kmeans_assign(pf, base.k_centroids, k_asg, kws), 5)
    kmeans_flops = 2.0 * cache.head_dim * float(
        (tok.seg_rows.astype(np.int64) * np.diff(tok.seg_cluster_ptr).astype(np.int64)).sum())
    # the clustering as a procedure: Lloyd rounds on the device from a strided start (assignment + means of the keys)
    fws = torch.empty(max(dp.dp_kmeans_fit_workspace_bytes(pf), 256), dtype=torch.uint8, device=dev)
    f_cent = torch.empty_like(base.k_centroids)
    fit_rounds = 2
    fit_us = wall_time(lambda i: dp.dp_kmeans_fit(pf, f_cent, fit_rounds, dp.DP_KMEANS_INIT_STRIDED, k_asg, fws), 3)
    del tok, pf, bws, kws, fws, f_cent, k_asg, b_k, b_v, b_off, b_sz, b_kc, b_vc

    # the kernel that moves the bytes: centroid scoring reads every key centroid and size once and
    # writes G logits per cluster
    total_k = int(cache.seg_cluster_ptr[-1])
    score_bytes = total_k * (2 * cache.head_dim + 4 + 4 * cache.group)
    score_gbs = score_bytes / (score_us * 1e-6) / 1e9
    # what the selection launch must read of a step whose heads it attends itself: the summaries of every head
    # (8 bytes per 16 clusters), the logits / sizes / offsets of the few sub-tiles that hold the top set (not
    # counted), K and V rows of the selected tokens and centroids; written: the output
    select_bytes = nh * ((mk + 15) // 16) * 8 + alg["rows_sum"] * 4 * cache.head_dim + nh * cache.head_dim * 6

    # the dominant kernel = the one that moves most of the step's algorithmic bytes: the centroid scan for
    # peaked heads, the row gather of the decode kernel when heads are flat
    decode_bytes = alg["rows_union"] * 4 * cache.head_dim
    if decode_bytes > score_bytes and shared_launch:
        roof = dict(kernel="select_decode_kernel (selection and split decode in one launch)", name="select_decode_kernel",
                    bytes=decode_bytes, avg=in_step_avg["select"], med=in_step_med["select"],
                    how="kernel-stamped HIP events inside dp_decode_attention")
    elif decode_bytes > score_bytes:
        roof = dict(kernel="decode_kernel (steps a5-a6 of dp_decode_attention)", name="decode_kernel",
                    bytes=decode_bytes, avg=in_step_avg["decode"], med=in_step_med["decode"],
                    how="kernel-stamped HIP events inside dp_decode_attention")
    else:
        roof = dict(kernel="score_kernel (dp_score_centroids)", name="score_kernel", bytes=score_bytes,
                    avg=score_us, med=score_med, how="kernel-stamped HIP events, back-to-back launches")
    roof_gbs = roof["bytes"] / (roof["avg"] * 1e-6) / 1e9
    # the kernel that takes the longest inside the step (not necessarily the one that moves the bytes)
    by_time = {"score": ("score kernel", score_bytes), "select": (
        "select_decode_kernel" if shared_launch else "select_kernel",
        decode_bytes + select_bytes if shared_launch else select_bytes), "decode": ("decode_kernel", decode_bytes)}
    longest = max(("score", "select", "decode"), key=lambda k: in_step_med[k])
    longest_gbs = by_time[longest][1] / (in_step_avg[longest] * 1e-6) / 1e9

    value = wall_us
    step_gbs = alg["total"] / (value * 1e-6) / 1e9
    result = {
        "metric": "us_per_decode_step_per_layer",
        "value": round(value, 3),
        "unit": "us",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(value / 1e3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{wname}: batch {cache.batch}, {cache.n_kv_heads} KV heads, "
                        f"{cache.n_q_heads} query heads, head_dim {cache.head_dim}, context "
                        f"{cache.meta['context'] if cache.batch > 1 else cache.meta['context'][0]}, "
                        f"{mk} clusters per KV head, bf16 K/V with fp32 accumulation, p1 {p1}, p2 {p2}",
            "entry_point": "dp_decode_attention",
            "layer_replicas": L,
            "out_dtype": "f32",
        },
        "tokens_of_context_per_s": round(cache.context_tokens / (value * 1e-6), 1),
        "step": {
            "event_us": round(event_us, 3),
            "timed_regions_wall_us": [round(r[0], 3) for r in regions],
            "reported_region": "median of three regions of `steps` steps each",
            "region_overhead_note": "a region is bracketed by two synchronisations: its first launch starts from an "
                                    "idle queue and its last kernel drains alone, a few microseconds that are shared "
                                    "by all `steps` steps, so a short region (--steps 20) reads some us per step higher "
                                    "than a long one; event_us (HIP events inside the same region) excludes the host side",
            "p10_us": round(pct(0.10), 3), "p50_us": round(pct(0.50), 3), "p90_us": round(pct(0.90), 3),
            "percentiles_over": f"{n_rot} rotations of {L} steps, each between two HIP events",
            "kernel_launches_per_step": n_launches,
            "cache_resident_us": round(resident_us, 3),
            "algorithmic_bytes": alg["total"],
            "algorithmic_bytes_per_head_sum": alg["total_per_head_sum"],
            "achieved_GBs": round(step_gbs, 1),
            "frac_of_hbm_peak": round(step_gbs / HBM_PEAK_GBS, 4),
            "stream_read_GBs": round(stream_gbs, 1),
            "frac_of_stream_read": round(step_gbs / stream_gbs, 4),
            "stream_read_measured_with": f"dp_stream_read_probe over the {big_bytes >> 20} MiB K cache of the replicas, "
                                         f"{n_big} launches between two HIP events",
            "read_floor_of_one_scan_us": round(read_floor_us, 3),
            "read_floor_back_to_back_interval_us": round(read_floor_gap_us, 3),
            "read_floor_note": f"the same probe over the {scan_bytes >> 20} MiB key-centroid matrix of each replica, back to "
                               "back: what one launch that only reads the scan's bytes takes on this machine",
            "retained_clusters_mean": float(nr_h.mean()),
            "exact_clusters_mean": float(ne_h.mean()),
            "exact_tokens_mean": float(nt_h.mean()),
            "per_head": {
                "retained_clusters": {"min": int(nr_h.min()), "median": float(np.median(nr_h)), "max": int(nr_h.max())},
                "exact_clusters": {"min": int(ne_h.min()), "median": float(np.median(ne_h)), "max": int(ne_h.max())},
                "exact_tokens": {"min": int(nt_h.min()), "median": float(np.median(nt_h)), "max": int(nt_h.max())},
                "rows_attended": {"min": int((nt_h + nr_h - ne_h).min()), "median": float(np.median(nt_h + nr_h - ne_h)),
                                  "max": int((nt_h + nr_h - ne_h).max())},
            },
        },
        "operating_point_0.95_0.7": {
            "step_us": round(op_us, 3), "retained_clusters_mean": op_counts[0], "exact_clusters_mean": op_counts[1],
            "exact_tokens_mean": op_counts[2],
            "note": "the (p1, p2) of the paper's ablation (Sec. 5.4) on the same inputs, wall clock over the rotating replicas",
        },
        "stages_us": {
            "dp_score_centroids": round(score_us, 3), "dp_topp_select": round(select_us, 3),
            "dp_sparse_decode": round(decode_us, 3),
            "median": {"score": round(score_med, 3), "select": round(select_med, 3), "decode": round(decode_med, 3)},
        },
        "kernels_in_step_us": {
            "avg": {k: round(v, 3) for k, v in in_step_avg.items()},
            "median": {k: round(v, 3) for k, v in in_step_med.items()},
            "how": "dp_decode_attention_timed: HIP events stamped with each kernel's own begin and end"
                   + ("; the split decode runs inside the selection launch (no decode kernel)" if shared_launch else ""),
        },
        "roofline": {
            "kernel": roof["kernel"],
            "bound": "hbm",
            "achieved": round(roof_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(roof_gbs / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic(roof["name"], args.config),
            "bytes_per_launch": roof["bytes"],
            "avg_launch_us": round(roof["avg"], 3),
            "median_launch_us": round(roof["med"], 3),
            "measured_with": roof["how"],
            "score_kernel": {"bytes_per_launch": score_bytes, "avg_launch_us": round(score_us, 3),
                             "GBs": round(score_gbs, 1), "back_to_back_interval_us": round(score_gap_us, 3),
                             "read_floor_us": round(read_floor_us, 3),
                             "read_floor_over_score": round(read_floor_us / score_us, 3)},
            "longest_kernel": {
                "kernel": by_time[longest][0], "median_us_in_step": round(in_step_med[longest], 3),
                "bytes_per_launch": by_time[longest][1], "GBs": round(longest_gbs, 1),
                "frac": round(longest_gbs / HBM_PEAK_GBS, 4),
                "note": "bound by the latency of its dependent memory round trips (summaries -> top sub-tiles -> K/V "
                        "rows -> output), not by bytes, when the heads are peaked" if longest == "select" and
                        decode_bytes <= score_bytes else "",
            },
        },
        "baselines_same_box": {
            "dense_us": round(dense_us, 3),
            "dense_entry_point": "dp_dense_decode (Eq. 1 over every token, K/V read once per KV head)",
            "dense_bytes": dense_bytes,
            "dense_GBs": round(dense_bytes / (dense_us * 1e-6) / 1e9, 1),
            "speedup_over_dense": round(dense_us / value, 2),
            "fixed_budget_us": round(budget_us, 3),
            "fixed_budget": {"k_retained": k_ret, "k_exact": k_ex, "entry_point": "dp_budget_decode_attention"},
            "speedup_over_fixed_budget": round(budget_us / value, 2),
        },
        "ab_paper_kernel_structure_us": ab,
        "with_sink_and_window_pinned_us": round(pinned_us, 3),
        "prefill_build": {"entry_point": "dp_build_cluster_cache", "us": round(build_us, 1),
                          "bytes": build_bytes, "GBs": round(build_bytes / (build_us * 1e-6) / 1e9, 1)},
        "kmeans_assign": {"entry_point": "dp_kmeans_assign", "us": round(kmeans_us, 1), "flops": kmeans_flops,
                          "TFLOPs": round(kmeans_flops / (kmeans_us * 1e-6) / 1e12, 1),
                          "frac_of_bf16_mfma_peak": round(kmeans_flops / (kmeans_us * 1e-6) / 2.5e15, 4)},
        "kmeans_fit": {"entry_point": "dp_kmeans_fit", "rounds": fit_rounds, "init": "strided",
                       "us_per_round": round(fit_us / fit_rounds, 1)},
        "gen_seconds": round(t_gen, 1),
    }

    if not args.no_cpu_baseline:
        import oracle
        orc = oracle.Oracle(cache)
        threads = os.cpu_count() or 1
        times = []
        t_end = time.time() + args.cpu_seconds
        while (len(times) < 3 or time.time() < t_end) and len(times) < 200:
            a = time.perf_counter()
            r = orc.decode_step(p1, p2, n_threads=threads, want_order=False)
            times.append(time.perf_counter() - a)
        # the same step on one thread, and the oracle's dense attention (Eq. 1) over every token, a few runs each
        single, dense_t = [], []
        t_end = time.time() + args.cpu_seconds / 2
        while (len(single) < 2 or time.time() < t_end) and len(single) < 20:
            a = time.perf_counter()
            orc.decode_step(p1, p2, n_threads=1, want_order=False)
            single.append(time.perf_counter() - a)
        t_end = time.time() + args.cpu_seconds / 2
        while (len(dense_t) < 2 or time.time() < t_end) and len(dense_t) < 20:
            a = time.perf_counter()
            orc.dense_step(n_threads=threads)
            dense_t.append(time.perf_counter() - a)
        result["cpu_baseline"] = {
            "value": round(statistics.median(times) * 1e6, 1),
            "unit": "us",
            "cores": int(r.threads),
            "kind": "oracle",
            "sample": f"the whole {wname} step (all {nh} heads), fp64 C oracle, OpenMP over heads, "
                      f"median of {len(times)} repetitions",
            "single_thread_us": round(statistics.median(single) * 1e6, 1),
            "single_thread_runs": len(single),
            "dense_us": round(statistics.median(dense_t) * 1e6, 1),
            "dense_note": f"the oracle's dense attention (Eq. 1) over every token, {threads} threads, "
                          f"median of {len(dense_t)} runs",
        }
        err = float(np.abs(out.cpu().numpy() - r.out).max())
        result["step"]["max_abs_err_vs_oracle"] = err
    print(json.dumps(result))


if __name__ == "__main__":
    main()
