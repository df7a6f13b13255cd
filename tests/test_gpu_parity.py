"""GPU parity: the HIP path (through the C ABI binding) against the fp64 CPU
oracle on the same seeded inputs.  Every test here needs a real MI355X."""
import math

import numpy as np
import pytest

import oracle
from workloads import ClusteredCache, bf16_bits_to_f32, f32_to_bf16_bits, make_cache, make_config

import harness as H

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------------------
# cases: small enough for the oracle to finish in seconds, several tiles + ragged tails
# ---------------------------------------------------------------------------
def case_cfg0():
    return make_config(0), 0.95, 0.9


def case_flat_ragged():
    # ragged batch, flat heads: hundreds of clusters retained, Kc (187 / 111) not a multiple of any tile
    c = make_cache(batch=2, n_kv_heads=2, n_q_heads=8, context=[3000, 1777], mean_cluster=16, q_scale=0.35, seed=11)
    return c, 0.95, 0.9


def case_mixed_sharpness():
    c = make_cache(batch=1, n_kv_heads=4, n_q_heads=16, context=8192, mean_cluster=16,
                   q_scale=lambda rng, b, h: [0.2, 0.5, 1.0, 3.0][h % 4], seed=12)
    return c, 0.95, 0.9


def case_gqa8_pareto():
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=16, context=16384, mean_cluster=16, size_dist="pareto",
                   size_lo=1, size_hi=512, q_scale=lambda rng, b, h: 0.5 if h % 2 == 0 else 5.0, seed=13)
    return c, 0.95, 0.9


def case_gqa1():
    return make_cache(batch=3, n_kv_heads=2, n_q_heads=2, context=[640, 1024, 333], mean_cluster=8, size_hi=32,
                      q_scale=0.5, seed=14), 0.9, 0.7


def case_gqa3_and_12():
    return make_cache(batch=1, n_kv_heads=1, n_q_heads=3, context=2000, mean_cluster=10, size_hi=40, q_scale=0.6,
                      seed=15), 0.98, 0.95


def case_gqa12():
    return make_cache(batch=1, n_kv_heads=1, n_q_heads=12, context=1500, mean_cluster=10, size_hi=40, q_scale=0.6,
                      seed=16), 0.95, 0.8


def case_many_clusters():
    # 9000 clusters per segment: the selection kernel's 16-logits-per-thread variant
    return make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=27000, mean_cluster=3, size_hi=8, q_scale=0.3,
                      seed=17), 0.95, 0.9


def case_single_cluster():
    return make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=37, n_clusters=1, size_lo=1, size_hi=64,
                      q_scale=1.0, seed=18), 0.95, 0.9


def case_giant_cluster():
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=1200, n_clusters=8, size_lo=1, size_hi=2000,
                   size_dist="pareto", mean_cluster=150, q_scale=0.2, seed=19)
    return c, 0.99, 0.9


def case_empty_clusters_and_segment():
    c = make_cache(batch=2, n_kv_heads=2, n_q_heads=4, context=[512, 256], mean_cluster=8, size_hi=32, q_scale=0.4,
                   seed=20)
    c.cluster_sizes[[1, 5, 17]] = 0
    a, e = int(c.seg_cluster_ptr[3]), int(c.seg_cluster_ptr[4])
    c.cluster_sizes[a:e] = 0          # a whole segment with nothing to attend to
    return c, 0.95, 0.9


def case_pinned_peaked():
    # sink + window clusters pinned on sharply peaked heads: the one-wave fast path carries the pinned clusters
    from workloads import pin_sink_and_window
    return pin_sink_and_window(make_config(0), first=1, last=4), 0.95, 0.9


def case_pinned_flat_ragged():
    # the same on flat heads (general path), ragged batch, one pinned cluster emptied, one segment pinned entirely
    from workloads import pin_sink_and_window
    c = make_cache(batch=2, n_kv_heads=2, n_q_heads=8, context=[3000, 1777], mean_cluster=16, q_scale=0.35, seed=21)
    pin_sink_and_window(c, first=2, last=5)
    c.cluster_sizes[int(c.seg_cluster_ptr[1]) - 2] = 0
    c.cluster_flags[int(c.seg_cluster_ptr[3]): int(c.seg_cluster_ptr[4])] = 1
    return c, 0.95, 0.9


def case_pinned_many_clusters():
    # 9000 clusters per segment (16 logits per thread) with scattered pinned clusters
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=27000, mean_cluster=3, size_hi=8, q_scale=0.3,
                   seed=22)
    c.cluster_flags = (np.random.default_rng(5).random(int(c.seg_cluster_ptr[-1])) < 0.01).astype(np.uint8)
    return c, 0.95, 0.9


def case_pinned_on_top():
    # Peaked heads on segments of 256 clusters with pinned clusters where they matter.  Segment 0: the cluster that
    # holds the most attention of head 0 is pinned (the max of the distribution moves to another cluster), and so are
    # its neighbour and two clusters far away; segment 1: sixteen pinned clusters, one of them emptied; segment 2:
    # twenty; segment 3: none.
    c = make_cache(batch=1, n_kv_heads=4, n_q_heads=8, context=4096, n_clusters=256, mean_cluster=16, size_hi=64,
                   q_scale=lambda rng, b, h: [3.0, 4.0][h % 2], seed=27)
    lg = oracle.Oracle(c).centroid_logits(0, 0)
    top = int(np.argmax(lg))
    flags = np.zeros(int(c.seg_cluster_ptr[-1]), np.uint8)
    flags[[top, top ^ 1, 7, 250]] = 1
    rng = np.random.default_rng(6)
    s1 = 256 + rng.choice(256, size=16, replace=False)
    flags[s1] = 1
    c.cluster_sizes[int(s1[3])] = 0
    flags[512 + rng.choice(256, size=20, replace=False)] = 1
    c.cluster_flags = flags
    return c, 0.95, 0.9


def case_many_heads():
    # more heads (320) than CUs: the selection kernel runs two 512-thread workgroups per CU; flat and peaked
    # heads, ragged batch, 3300 / 1500 / 600 clusters per segment, sink and window pinned
    from workloads import pin_sink_and_window
    c = make_cache(batch=10, n_kv_heads=8, n_q_heads=32, context=[26400, 12000, 4800, 900, 26400, 700, 5000, 64, 3000, 9999],
                   mean_cluster=8, size_hi=32, q_scale=lambda rng, b, h: [0.3, 3.0, 0.6, 1.5][h % 4], seed=23)
    return pin_sink_and_window(c, first=1, last=2), 0.95, 0.9


def case_very_many_heads():
    # 640 heads: four 256-thread selection workgroups per CU; up to 1700 clusters per segment (8 logits per
    # thread), flat and peaked heads, one head group with 300 - 600 rows (beyond that kernel's inline limit)
    from workloads import pin_sink_and_window
    ctx = [13600, 700, 5000, 64, 3000, 9999, 13000, 2048, 4096, 333] * 2
    c = make_cache(batch=20, n_kv_heads=8, n_q_heads=32, context=ctx, mean_cluster=8, size_hi=32,
                   q_scale=lambda rng, b, h: [0.3, 3.0, 0.8, 1.5][h % 4], seed=24)
    return pin_sink_and_window(c, first=1, last=2), 0.95, 0.9


def case_gqa16_and_6_ragged():
    # the largest supported group (16 heads share a segment: every column of the scoring kernel's matrix tile is a
    # head), ragged segments whose cluster counts are not multiples of the 16-row tile, flat and peaked heads
    c = make_cache(batch=3, n_kv_heads=2, n_q_heads=32, context=[2100, 37, 1333], mean_cluster=7, size_hi=32,
                   q_scale=lambda rng, b, h: [0.3, 2.0, 0.7, 4.0][h % 4], seed=25)
    return c, 0.95, 0.9


def case_gqa6():
    c = make_cache(batch=2, n_kv_heads=3, n_q_heads=18, context=[999, 3001], mean_cluster=9, size_hi=40,
                   q_scale=lambda rng, b, h: [0.4, 3.0][h % 2], seed=26)
    return c, 0.9, 0.8


CASES = {f.__name__[5:]: f for f in (case_gqa16_and_6_ragged, case_gqa6, case_cfg0, case_flat_ragged, case_mixed_sharpness, case_gqa8_pareto, case_gqa1,
                                     case_gqa3_and_12, case_gqa12, case_many_clusters, case_single_cluster,
                                     case_giant_cluster, case_empty_clusters_and_segment, case_pinned_peaked,
                                     case_pinned_flat_ragged, case_pinned_many_clusters, case_pinned_on_top, case_many_heads,
                                     case_very_many_heads)}


@pytest.fixture(scope="module", params=sorted(CASES))
def case(request):
    cache, p1, p2 = CASES[request.param]()
    return request.param, cache, p1, p2, oracle.Oracle(cache)


# ---------------------------------------------------------------------------
# stage 1
# ---------------------------------------------------------------------------
def test_score_centroids_matches_oracle(case):
    name, cache, p1, p2, orc = case
    per_head, _ = H.gpu_logits(cache)
    worst = 0.0
    for b in range(cache.batch):
        for h in range(cache.n_q_heads):
            ref = orc.centroid_logits(b, h)
            got = per_head[b * cache.n_q_heads + h].astype(np.float64)
            assert got.shape == ref.shape
            empty = np.isneginf(ref)
            assert np.array_equal(np.isneginf(got), empty)
            if (~empty).any():
                # fp32 accumulation of exact bf16 products: a few ulp of the largest partial sum
                tol = 4e-6 * max(1.0, np.abs(ref[~empty]).max()) + 2e-6
                err = np.abs(got[~empty] - ref[~empty]).max()
                worst = max(worst, err / tol)
                assert err <= tol, (name, b, h, err, tol)
    print(f"[{name}] logits worst err/tol = {worst:.3f}")


# ---------------------------------------------------------------------------
# stage 2 from the GPU's own fp32 logits: the decision is taken on identical numbers
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("flags", [0, 1])
def test_topp_select_matches_oracle_on_same_logits(case, flags):
    name, cache, p1, p2, orc = case
    per_head, flat = H.gpu_logits(cache)
    for (q1, q2) in ((p1, p2), (0.5, 0.5), (1.0, 1.0), (0.9, 0.0), (1.0, 0.6)):
        exact, approx, ntok = H.gpu_select(cache, flat, q1, q2, flags)
        n_tol = 0
        for i in range(cache.batch * cache.n_q_heads):
            b, h = divmod(i, cache.n_q_heads)
            lg = per_head[i].astype(np.float64)
            pins = orc.pinned_clusters(b, h)
            s = orc.select(lg, q1, q2, flags, pinned=pins)
            got_ret = np.sort(np.concatenate([exact[i], approx[i]]))
            same = np.array_equal(got_ret, s.retained) and np.array_equal(exact[i], s.exact)
            if not same:
                # both sets are judged by the near-threshold rule (the exact set on the GPU's own retained set)
                lg[pins] = -np.inf
                same = H.judge_head_sets(f"{name} head {i} p=({q1},{q2})", exact[i], approx[i], lg, pins, q1, q2,
                                         flags, orc)
                assert not same and q1 < 1.0
                n_tol += 1
            seg = b * cache.n_kv_heads + h // cache.group
            c0 = int(cache.seg_cluster_ptr[seg])
            assert int(ntok[i]) == int(cache.cluster_sizes[c0 + np.asarray(exact[i], np.int64)].sum())
        assert n_tol <= 1, (name, q1, q2, n_tol)


# ---------------------------------------------------------------------------
# stage 3 on the oracle's sets
# ---------------------------------------------------------------------------
def test_sparse_decode_matches_oracle_on_oracle_sets(case):
    name, cache, p1, p2, orc = case
    r = orc.decode_step(p1, p2)
    nh = cache.batch * cache.n_q_heads
    exact = [np.sort(np.concatenate([orc.pinned_clusters(*divmod(i, cache.n_q_heads)), r.order[i, : r.k2.flat[i]]]))
             for i in range(nh)]
    approx = [np.sort(r.order[i, r.k2.flat[i]: r.k1.flat[i]]) for i in range(nh)]
    out, lse = H.gpu_sparse_decode(cache, exact, approx)
    g = H.GpuStep(out=out, lse=lse, exact=exact, approx=approx, n_exact_tokens=np.zeros(nh))
    worst, rel = H.check_outputs(cache, orc, g, tight=2e-4)
    np.testing.assert_allclose(out, r.out, atol=H.OUT_MAX_ABS)
    print(f"[{name}] sparse_decode max-abs {worst:.2e} rel-L2 {rel:.2e}")
    # bf16 output = the fp32 output rounded to nearest even
    out16, _ = H.gpu_sparse_decode(cache, exact, approx, out_bf16=True)
    np.testing.assert_array_equal(f32_to_bf16_bits(out16), f32_to_bf16_bits(out))


# ---------------------------------------------------------------------------
# the one-call path
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("pp", ["case", (0.5, 0.5), (1.0, 1.0), (0.9, 0.0), (0.99, 1.0)])
def test_decode_attention_matches_oracle(case, pp):
    name, cache, p1, p2, orc = case
    if pp != "case":
        p1, p2 = pp
    g = H.gpu_decode_attention(cache, p1, p2)
    tolerated = H.check_sets(cache, orc, g, p1, p2)
    worst, rel = H.check_outputs(cache, orc, g, tight=2e-4)
    nh = cache.batch * cache.n_q_heads
    assert tolerated <= max(1, nh // 50), f"{tolerated} of {nh} heads differ from the oracle's sets"
    if tolerated == 0:
        r = orc.decode_step(p1, p2)
        np.testing.assert_allclose(g.out, r.out, atol=H.OUT_MAX_ABS)
    print(f"[{name} p=({p1},{p2})] sets exact on {nh - tolerated}/{nh} heads, out max-abs {worst:.2e} rel-L2 {rel:.2e}")


def test_scoring_summaries_describe_the_logits(case):
    """What the scoring stage leaves for the selection next to the logits: per head and run of 16 clusters the
    largest logit (exactly) and the sum of exp(logit - that) (fp32 rounding of 16 terms)."""
    import torch
    import paper_2602_05191_amd as dp
    name, cache, p1, p2, orc = case
    if cache.cluster_flags is not None or cache.max_clusters_per_seg == 0:
        pytest.skip("the summaries are written for the top-p rule on caches without cluster flags")
    dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc)
    nh, mk = cache.batch * cache.n_q_heads, cache.max_clusters_per_seg
    ws = torch.zeros(dp.dp_workspace_bytes(pr), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((cache.batch, cache.n_q_heads, 128), dtype=torch.float32, device="cuda:0")
    dp.dp_decode_attention(pr, 0.95, 0.9, out, None, ws)
    torch.cuda.synchronize()
    lay = dp.dp_workspace_layout(pr)
    wsh = ws.cpu().numpy()
    stride = (mk + 15) // 16
    summ = wsh[lay["summaries"]: lay["summaries"] + 8 * nh * stride].view(np.float32).reshape(nh, stride, 2)
    flat = wsh[lay["logits"]: lay["logits"] + 4 * cache.group * int(cache.seg_cluster_ptr[-1])].view(np.float32)
    for i in range(nh):
        s0, kc = H.head_logit_slice(cache, *divmod(i, cache.n_q_heads))
        lg = np.full(((kc + 15) // 16) * 16, -np.inf, np.float32)
        lg[:kc] = flat[s0:s0 + kc]
        lg = lg.reshape(-1, 16)
        mx = lg.max(axis=1)
        assert np.array_equal(summ[i, : len(mx), 0], mx), (name, i)
        with np.errstate(invalid="ignore"):
            se = np.where(np.isfinite(mx), np.exp(lg.astype(np.float64) - mx[:, None].astype(np.float64)).sum(axis=1), 0.0)
        np.testing.assert_allclose(summ[i, : len(mx), 1], se, rtol=2e-6, atol=0)


def test_split_decode_inside_the_selection_launch_and_as_a_launch_of_its_own(case):
    """A step that serves at most 128 heads runs the split decode inside the selection launch; the flag
    DP_FLAG_SEPARATE_DECODE_LAUNCH keeps the three launches.  Same sets; outputs equal up to the different
    split of a head's rows into partial results."""
    import paper_2602_05191_amd as dp
    name, cache, p1, p2, orc = case
    for q1, q2 in ((p1, p2), (1.0, 1.0)):
        a = H.gpu_decode_attention(cache, q1, q2)
        b = H.gpu_decode_attention(cache, q1, q2, flags=dp.DP_FLAG_SEPARATE_DECODE_LAUNCH)
        for x, y in zip(a.exact + a.approx, b.exact + b.approx):
            assert np.array_equal(x, y)
        assert np.array_equal(a.n_exact_tokens, b.n_exact_tokens)
        assert np.abs(a.out - b.out).max() <= 2e-5, (name, q1, q2)
        fin = np.isfinite(a.lse)
        assert np.array_equal(fin, np.isfinite(b.lse)) and np.abs(a.lse[fin] - b.lse[fin]).max(initial=0.0) <= 1e-4
        H.check_outputs(cache, orc, b, tight=2e-4)


def test_bound_step_is_the_same_call():
    """BoundDecodeStep marshals the arguments of dp_decode_attention once: same bits as the direct call, on every call."""
    import torch
    import paper_2602_05191_amd as dp
    cache = make_config(0)
    dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc)
    ws = torch.zeros(dp.dp_workspace_bytes(pr), dtype=torch.uint8, device="cuda:0")
    nh = cache.batch * cache.n_q_heads
    a = torch.full((cache.batch, cache.n_q_heads, cache.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
    b = torch.full_like(a, float("nan"))
    la = torch.empty(nh, dtype=torch.float32, device="cuda:0")
    lb, ne = torch.empty_like(la), torch.empty(nh, dtype=torch.int32, device="cuda:0")
    dp.dp_decode_attention(pr, cache.p1, cache.p2, a, la, ws)
    torch.cuda.synchronize()
    step = dp.BoundDecodeStep(pr, cache.p1, cache.p2, b, lb, ws, ne)
    for _ in range(3):
        b.fill_(float("nan"))
        step()
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int32), b.view(torch.int32)) and torch.equal(la.view(torch.int32), lb.view(torch.int32))
    assert int(ne.min().item()) >= 1


def test_decode_attention_is_bitwise_reproducible(case):
    name, cache, p1, p2, orc = case
    a = H.gpu_decode_attention(cache, p1, p2)
    b = H.gpu_decode_attention(cache, p1, p2)
    assert np.array_equal(a.out.view(np.uint32), b.out.view(np.uint32))
    assert np.array_equal(a.lse.view(np.uint32), b.lse.view(np.uint32))
    for x, y in zip(a.exact + a.approx, b.exact + b.approx):
        assert np.array_equal(x, y)


def test_dense_limit_on_gpu():
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=4096, mean_cluster=16, q_scale=0.5, seed=31)
    orc = oracle.Oracle(c)
    g = H.gpu_decode_attention(c, 1.0, 1.0)
    dense, dense_lse, _ = orc.dense_step()
    np.testing.assert_allclose(g.out, dense, atol=2e-4)
    np.testing.assert_allclose(g.lse, dense_lse, atol=1e-3)
    for i in range(8):
        assert len(g.approx[i]) == 0 and len(g.exact[i]) == 256


def test_hand_worked_case_on_gpu():
    """The three-cluster example of tests/golden/hand_worked_case.json, zero-padded to head_dim 128."""
    d = 128
    def row(x):
        r = np.zeros(d, np.float32)
        r[: len(x)] = x
        return r
    keys = np.stack([row(k) for k in ([3, 0], [1, 0], [1, 0], [0, 0], [0, 0], [0, 0], [0, 0])])
    vals = np.stack([row(v) for v in ([1, 0], [0, 1], [2, 2], [4, 0], [0, 4], [4, 4], [0, 0])])
    kc = np.stack([row(k) for k in ([2, 0], [1, 0], [0, 0])])
    vc = np.stack([row(v) for v in ([.5, .5], [2, 2], [2, 2])])
    c = ClusteredCache(batch=1, n_kv_heads=1, n_q_heads=1, head_dim=d, q=f32_to_bf16_bits(row([1, 0]).reshape(1, 1, d)),
                       k_cache=f32_to_bf16_bits(keys), v_cache=f32_to_bf16_bits(vals),
                       seg_row_base=np.zeros(1, np.int64), seg_cluster_ptr=np.array([0, 3], np.int32),
                       cluster_offsets=np.array([0, 2, 3], np.int32), cluster_sizes=np.array([2, 1, 4], np.int32),
                       k_centroids=f32_to_bf16_bits(kc), v_centroids=f32_to_bf16_bits(vc))
    g = H.gpu_decode_attention(c, 0.8, 0.5, sm_scale=math.log(2.0))
    assert g.exact[0].tolist() == [0] and g.approx[0].tolist() == [2]
    np.testing.assert_allclose(g.out[0, 0, :2], [8 / 7, 5 / 7], rtol=1e-6)
    assert g.lse[0, 0] == pytest.approx(math.log(14.0), rel=1e-6)
    ga = H.gpu_decode_attention(c, 0.8, 0.6, flags=1, sm_scale=math.log(2.0))
    assert ga.exact[0].tolist() == [0, 2] and ga.approx[0].tolist() == []
    np.testing.assert_allclose(ga.out[0, 0, :2], [16 / 14, 10 / 14], rtol=1e-6)   # Eq. 9 with c0 and c2 exact
    assert ga.lse[0, 0] == pytest.approx(math.log(14.0), rel=1e-6)
    g0 = H.gpu_decode_attention(c, 0.8, 0.0, sm_scale=math.log(2.0))
    np.testing.assert_allclose(g0.out[0, 0, :2], [1.0, 1.0], rtol=1e-6)


# ---------------------------------------------------------------------------
# ties: equal scores are cut in cluster-index order
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,p1,p2", [(2000, 0.5, 0.5), (2000, 0.3001, 1.0), (700, 0.9, 0.1), (5000, 0.77, 0.33), (2000, 0.3001, 0.4567),
                                     (3000, 0.61234, 0.4321)])
def test_all_equal_scores_are_cut_by_index(n, p1, p2):
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=2, context=n, n_clusters=n, size_dist="ones", size_lo=1,
                   size_hi=1, q_scale=0.5, seed=40)
    c.k_centroids[:] = c.k_centroids[0]          # every cluster gets the same score
    orc = oracle.Oracle(c)
    g = H.gpu_decode_attention(c, p1, p2)
    # all masses are equal (1 / n each, far above the 1e-5 of the near-threshold rule): the cut may move by one
    # element only where p * n is within that rule of an integer, which check_sets decides
    assert H.check_sets(c, orc, g, p1, p2) <= 2
    for i in range(2):
        s = orc.select(orc.centroid_logits(0, i), p1, p2)
        k1 = len(g.exact[i]) + len(g.approx[i])
        strict1 = abs(p1 * n - round(p1 * n)) > 1e-3          # the first cut is not at a multiple of 1 / n
        if strict1:
            assert k1 == s.k1, (k1, s.k1)
        if p2 >= 1.0 or (strict1 and abs(p2 * s.k1 - round(p2 * s.k1)) > 1e-3):
            assert len(g.exact[i]) == (k1 if p2 >= 1.0 else s.k2), (len(g.exact[i]), s.k2)
        assert np.array_equal(np.sort(np.concatenate([g.exact[i], g.approx[i]])), np.arange(k1))
        assert np.array_equal(g.exact[i], np.arange(len(g.exact[i])))
    H.check_outputs(c, orc, g, tight=2e-4)


def test_partial_ties_at_the_threshold():
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=1500, n_clusters=1500, size_dist="ones", size_lo=1,
                   size_hi=1, q_scale=0.3, seed=41)
    # blocks of identical centroids: many equal scores, some of them straddling the threshold
    for start in range(0, 1500, 50):
        c.k_centroids[start:start + 37] = c.k_centroids[start]
    orc = oracle.Oracle(c)
    for p1, p2 in ((0.5, 0.5), (0.9, 0.8), (0.97, 0.2)):
        g = H.gpu_decode_attention(c, p1, p2)
        assert H.check_sets(c, orc, g, p1, p2) <= 1
        H.check_outputs(c, orc, g, tight=2e-4)


def pinned_tie_case(n):
    """n singleton clusters with one and the same score, 40 of them pinned (the first, the last and 38 others)."""
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=2, context=n, n_clusters=n, size_dist="ones", size_lo=1,
                   size_hi=1, q_scale=0.5, seed=44)
    c.k_centroids[:] = c.k_centroids[0]
    flags = np.zeros(n, np.uint8)
    flags[np.random.default_rng(9).choice(n, size=38, replace=False)] = 1
    flags[[0, n - 1]] = 1
    c.cluster_flags = flags
    return c


@pytest.mark.parametrize("n", [2000, 5000])
def test_ties_with_pinned_clusters_of_the_same_score(n):
    """A run of equal scores far longer than the selection kernel ranks pairwise, with pinned clusters inside the
    run: the pinned ones are outside the distribution (they must not be counted in the cut) and all exact.  The
    masses are equal and no threshold falls on a multiple of one mass, so the sets must equal the oracle's."""
    c = pinned_tie_case(n)
    orc = oracle.Oracle(c)
    n_cand = n - int(c.cluster_flags.sum())
    per_head, flat = H.gpu_logits(c)
    for p1, p2 in ((0.3001, 0.4567), (0.61234, 1.0), (0.8765, 0.1234)):
        assert abs(p1 * n_cand - round(p1 * n_cand)) > 1e-2
        g = H.gpu_decode_attention(c, p1, p2)
        assert H.check_sets(c, orc, g, p1, p2) == 0
        H.check_outputs(c, orc, g, tight=2e-4)
        exact, approx, _ = H.gpu_select(c, flat, p1, p2)
        for i in range(2):
            s = orc.select(per_head[i].astype(np.float64), p1, p2, pinned=orc.pinned_clusters(0, i))
            assert np.array_equal(exact[i], s.exact) and np.array_equal(approx[i], s.approx), (n, p1, p2, i)
            assert np.array_equal(g.exact[i], s.exact) and np.array_equal(g.approx[i], s.approx), (n, p1, p2, i)
    for kr, ke in ((700, 300), (1, 1), (n_cand - 1, n_cand - 2), (1025, 0)):
        g = H.gpu_decode_attention(c, 0, 0, budget=(kr, ke))
        exact, approx, _ = H.gpu_select(c, flat, 0, 0, budget=(kr, ke))
        for i in range(2):
            s = orc.fixed_budget(per_head[i].astype(np.float64), kr, ke, pinned=orc.pinned_clusters(0, i))
            assert np.array_equal(exact[i], s.exact) and np.array_equal(approx[i], s.approx), (n, kr, ke, i)
            assert np.array_equal(g.exact[i], s.exact) and np.array_equal(g.approx[i], s.approx), (n, kr, ke, i)
        H.check_outputs(c, orc, g, tight=2e-4)


def test_partial_ties_with_pinned_clusters():
    """Blocks of equal scores, some straddling the thresholds, with pinned clusters inside the blocks."""
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=3000, n_clusters=3000, size_dist="ones", size_lo=1,
                   size_hi=1, q_scale=0.3, seed=45)
    for start in range(0, 3000, 1000):
        c.k_centroids[start:start + 700] = c.k_centroids[start]      # runs of 700 equal scores
    flags = np.zeros(3000, np.uint8)
    flags[np.random.default_rng(10).choice(3000, size=60, replace=False)] = 1
    c.cluster_flags = flags
    orc = oracle.Oracle(c)
    for p1, p2 in ((0.5, 0.5), (0.9, 0.8), (0.97, 0.2)):
        g = H.gpu_decode_attention(c, p1, p2)
        assert H.check_sets(c, orc, g, p1, p2) <= 1
        H.check_outputs(c, orc, g, tight=2e-4)


# ---------------------------------------------------------------------------
# more heads than one stage-3 queue serves (1024): several decode launches with their own counters
# ---------------------------------------------------------------------------
def test_more_than_1024_heads():
    """40 sequences x 32 query heads = 1280 heads, ragged short contexts, flat and peaked heads; the flat heads
    of the longer sequences have more rows than the selection kernel attends itself, so both slabs of the
    stage-3 queue get work.  One-call path and staged stage 3 on the oracle's sets."""
    rng = np.random.default_rng(77)
    ctx = [int(x) for x in rng.integers(64, 2600, size=40)]
    ctx[3], ctx[37] = 12000, 10000                                # heavy flat heads in the first and the second slab
    c = make_cache(batch=40, n_kv_heads=8, n_q_heads=32, context=ctx, mean_cluster=8, size_hi=32,
                   q_scale=lambda r, b, h: [0.3, 3.0, 0.8, 1.5][h % 4], seed=27)
    orc = oracle.Oracle(c)
    nh = c.batch * c.n_q_heads
    assert nh > 1024
    p1, p2 = 0.95, 0.9
    g = H.gpu_decode_attention(c, p1, p2)
    tolerated = H.check_sets(c, orc, g, p1, p2)
    assert tolerated <= nh // 50
    H.check_outputs(c, orc, g, tight=2e-4)
    rows = [int(g.n_exact_tokens[i]) + len(g.approx[i]) for i in range(nh)]
    assert max(rows[:1024]) > 1024 and max(rows[1024:]) > 1024     # heads beyond the inline limit in both slabs
    r = orc.decode_step(p1, p2)
    exact = [np.sort(r.order[i, : r.k2.flat[i]]) for i in range(nh)]
    approx = [np.sort(r.order[i, r.k2.flat[i]: r.k1.flat[i]]) for i in range(nh)]
    out, lse = H.gpu_sparse_decode(c, exact, approx)
    gs = H.GpuStep(out=out, lse=lse, exact=exact, approx=approx, n_exact_tokens=np.zeros(nh))
    H.check_outputs(c, orc, gs, tight=2e-4)
    np.testing.assert_allclose(out, r.out, atol=H.OUT_MAX_ABS)
    # a second run gives the same bits (per-slab counters are reset by the step itself)
    g2 = H.gpu_decode_attention(c, p1, p2)
    assert np.array_equal(g.out.view(np.uint32), g2.out.view(np.uint32))


# ---------------------------------------------------------------------------
# bf16 output of the one-call path: the fp32 result rounded to nearest even, on every way out of the step
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("which", ["cfg0", "flat_ragged", "gqa8_pareto", "empty_clusters_and_segment", "mixed_sharpness"])
def test_decode_attention_bf16_output_is_the_rounded_fp32_output(which):
    cache, p1, p2 = CASES[which]()
    a = H.gpu_decode_attention(cache, p1, p2)
    b = H.gpu_decode_attention(cache, p1, p2, out_bf16=True)
    assert np.array_equal(f32_to_bf16_bits(b.out), f32_to_bf16_bits(a.out)), which
    assert np.array_equal(a.lse.view(np.uint32), b.lse.view(np.uint32))
    for x, y in zip(a.exact + a.approx, b.exact + b.approx):
        assert np.array_equal(x, y)
    # and through the fixed-budget entry point (heads of a few hundred rows)
    a = H.gpu_decode_attention(cache, 0, 0, budget=(64, 16))
    b = H.gpu_decode_attention(cache, 0, 0, budget=(64, 16), out_bf16=True)
    assert np.array_equal(f32_to_bf16_bits(b.out), f32_to_bf16_bits(a.out)), which


# ---------------------------------------------------------------------------
# fixed budget in place of the two thresholds (dp_topk_select, dp_budget_decode_attention)
# ---------------------------------------------------------------------------
BUDGETS = [(1, 1), (1, 0), (7, 3), (64, 16), (65, 65), (300, 40), (10 ** 6, 5), (10 ** 6, 10 ** 6), (0, 0), (5, 9)]


def test_topk_select_is_the_oracle_top_k_of_the_same_logits(case):
    """Integer work on identical inputs: the sets must be identical."""
    name, cache, p1, p2, orc = case
    per_head, flat = H.gpu_logits(cache)
    for kr, ke in BUDGETS:
        exact, approx, ntok = H.gpu_select(cache, flat, 0, 0, budget=(kr, ke))
        for b in range(cache.batch):
            for h in range(cache.n_q_heads):
                i = b * cache.n_q_heads + h
                s = orc.fixed_budget(per_head[i].astype(np.float64), kr, ke, pinned=orc.pinned_clusters(b, h))
                assert np.array_equal(exact[i], s.exact) and np.array_equal(approx[i], s.approx), (name, kr, ke, i)
                seg = b * cache.n_kv_heads + h // cache.group
                c0 = int(cache.seg_cluster_ptr[seg])
                assert int(ntok[i]) == int(cache.cluster_sizes[c0 + s.exact].sum())


@pytest.mark.parametrize("budget", [(1, 1), (7, 3), (64, 16), (300, 40), (10 ** 6, 10 ** 6), (0, 0)])
def test_budget_decode_attention_matches_oracle(case, budget):
    name, cache, p1, p2, orc = case
    g = H.gpu_decode_attention(cache, 0, 0, want_logits=True, budget=budget)
    nh = cache.batch * cache.n_q_heads
    for i in range(nh):
        # the sets are the top-k of the logits the GPU itself computed (checked against the oracle's in stage 1)
        s = orc.fixed_budget(g.logits[i].astype(np.float64), *budget,
                             pinned=orc.pinned_clusters(*divmod(i, cache.n_q_heads)))
        assert np.array_equal(g.exact[i], s.exact) and np.array_equal(g.approx[i], s.approx), (name, budget, i)
    # against the oracle's own step: same counts; sets equal except where fp32 and fp64 logits order a near-tie differently
    r = orc.budget_step(*budget, n_threads=4)
    differing = 0
    for i in range(nh):
        b, h = divmod(i, cache.n_q_heads)
        pins = orc.pinned_clusters(b, h)
        assert np.isin(pins, g.exact[i]).all()
        got_ex = np.setdiff1d(g.exact[i], pins)
        assert len(got_ex) == r.k2[b, h] and len(got_ex) + len(g.approx[i]) == r.k1[b, h]
        same = (np.array_equal(got_ex, np.sort(r.order[i, : r.k2[b, h]])) and
                np.array_equal(g.approx[i], np.sort(r.order[i, r.k2[b, h]: r.k1[b, h]])))
        if not same:
            lg = orc.centroid_logits(b, h)
            for got, want in ((got_ex, r.order[i, : r.k2[b, h]]),
                              (np.concatenate([got_ex, g.approx[i]]), r.order[i, : r.k1[b, h]])):
                swapped = np.setxor1d(got, want)
                assert swapped.size == 0 or np.ptp(lg[swapped]) <= H.LOGIT_TIE_TOL, (name, budget, i, swapped)
            differing += 1
    assert differing <= max(1, nh // 8), (name, budget, differing)
    H.check_outputs(cache, orc, g, tight=2e-4)


def test_budget_ties_are_cut_by_index():
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=2, context=3000, n_clusters=3000, size_dist="ones", size_lo=1,
                   size_hi=1, q_scale=0.5, seed=42)
    c.k_centroids[:] = c.k_centroids[0]          # every cluster gets the same score
    orc = oracle.Oracle(c)
    for kr, ke in ((1, 1), (700, 699), (2999, 1), (3000, 3000), (1025, 513)):
        g = H.gpu_decode_attention(c, 0, 0, budget=(kr, ke))
        for i in range(2):
            assert np.array_equal(g.exact[i], np.arange(ke)) and np.array_equal(g.approx[i], np.arange(ke, kr))
        H.check_outputs(c, orc, g, tight=2e-4)


# ---------------------------------------------------------------------------
# the largest cluster counts: 32 and 64 logits per thread, and one over the limit
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n_clusters", [20000, 65536])
def test_very_many_clusters(n_clusters):
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=2, context=2 * n_clusters, n_clusters=n_clusters, size_lo=1,
                   size_hi=6, mean_cluster=2, q_scale=lambda rng, b, h: [0.3, 2.0][h], seed=70)
    orc = oracle.Oracle(c)
    for p1, p2 in ((0.95, 0.9), (0.6, 0.3)):
        g = H.gpu_decode_attention(c, p1, p2)
        assert H.check_sets(c, orc, g, p1, p2) <= 1
        H.check_outputs(c, orc, g, tight=2e-4)
    g = H.gpu_decode_attention(c, 0, 0, want_logits=True, budget=(3000, 700))
    for i in range(2):
        s = orc.fixed_budget(g.logits[i].astype(np.float64), 3000, 700)
        assert np.array_equal(g.exact[i], s.exact) and np.array_equal(g.approx[i], s.approx)
    H.check_outputs(c, orc, g, tight=2e-4)


def test_more_clusters_than_supported_is_refused():
    import torch
    import paper_2602_05191_amd as dp
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=70000, n_clusters=65537, size_lo=1, size_hi=3,
                   mean_cluster=1, q_scale=1.0, seed=71)
    pr = dp.Problem(dp.DeviceCache.from_host(c))
    ws = torch.empty(max(dp.dp_workspace_bytes(pr), 256), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((1, 1, 128), dtype=torch.float32, device="cuda:0")
    with pytest.raises(dp.DPError) as e:
        dp.dp_decode_attention(pr, 0.9, 0.5, out, None, ws)
    assert e.value.status == -2


# ---------------------------------------------------------------------------
# dense baseline (Eq. 1): dp_dense_decode
# ---------------------------------------------------------------------------
def check_dense(cache, orc, out, lse, tight=2e-4):
    ref, ref_lse, _ = orc.dense_step(n_threads=4)
    d = out.astype(np.float64) - ref
    worst = float(np.abs(d).max()) if d.size else 0.0
    den = float((ref * ref).sum())
    rel = (float((d * d).sum()) / den) ** 0.5 if den > 0 else 0.0
    assert worst <= min(H.OUT_MAX_ABS, tight) and rel <= H.OUT_REL_L2, (worst, rel)
    fin = np.isfinite(ref_lse)
    assert (np.abs(lse[fin] - ref_lse[fin]) <= 1e-3 + 1e-5 * np.abs(ref_lse[fin])).all()
    assert np.isneginf(lse[~fin]).all() and (out[~fin] == 0).all()
    return worst, rel


def test_dense_decode_matches_oracle(case):
    name, cache, p1, p2, orc = case
    rows = H.segment_rows(cache)
    if rows is None:
        pytest.skip("clusters with emptied sizes leave gaps: the segment is not a contiguous row range")
    out, lse = H.gpu_dense_decode(cache, rows)
    check_dense(cache, orc, out, lse)


def test_dense_decode_bf16_output_and_scale():
    c = make_cache(batch=2, n_kv_heads=2, n_q_heads=8, context=[5000, 129], mean_cluster=16, q_scale=0.6, seed=51)
    orc = oracle.Oracle(c, sm_scale=0.05)
    out, lse = H.gpu_dense_decode(c, H.segment_rows(c), sm_scale=0.05, out_bf16=True)
    ref, ref_lse, _ = orc.dense_step(n_threads=4)
    assert np.abs(out - ref).max() <= 2e-4 + np.abs(ref).max() * 2.0 ** -8   # one bf16 rounding of the result
    assert np.abs(lse - ref_lse).max() <= 1e-3


def test_dense_decode_equals_the_sparse_path_with_everything_exact():
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=6000, mean_cluster=16, q_scale=0.5, seed=52)
    out, lse = H.gpu_dense_decode(c, H.segment_rows(c))
    g = H.gpu_decode_attention(c, 1.0, 1.0)
    assert np.abs(out - g.out).max() <= 1e-5 and np.abs(lse - g.lse).max() <= 1e-4


# ---------------------------------------------------------------------------
# error paths of the boundary (host-side checks; nothing is launched)
# ---------------------------------------------------------------------------
def test_boundary_rejects_bad_arguments():
    import torch
    import paper_2602_05191_amd as dp
    c = make_config(0, shrink=4)
    dc = dp.DeviceCache.from_host(c)
    pr = dp.Problem(dc)
    nh = c.batch * c.n_q_heads
    ws = torch.empty(dp.dp_workspace_bytes(pr), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((1, 4, 128), dtype=torch.float32, device="cuda:0")
    for p1, p2 in ((0.0, 0.5), (1.5, 0.5), (0.9, -0.1), (0.9, 1.1), (float("nan"), 0.5)):
        with pytest.raises(dp.DPError) as e:
            dp.dp_decode_attention(pr, p1, p2, out, None, ws)
        assert e.value.status == -1
    with pytest.raises(dp.DPError) as e:
        dp.dp_decode_attention(pr, 0.9, 0.5, out, None, ws[:1024])
    assert e.value.status == -3
    for kr, ke in ((-1, 0), (3, -2)):
        with pytest.raises(dp.DPError) as e:
            dp.dp_budget_decode_attention(pr, kr, ke, out, None, ws)
        assert e.value.status == -1
    bad = dp.Problem(dc)
    bad.c.head_dim = 64
    with pytest.raises(dp.DPError) as e:
        dp.dp_decode_attention(bad, 0.9, 0.5, out, None, ws)
    assert e.value.status == -2
    bad = dp.Problem(dc)
    bad.c.n_kv_heads = 3                 # 4 query heads do not divide into 3 KV heads
    with pytest.raises(dp.DPError) as e:
        dp.dp_decode_attention(bad, 0.9, 0.5, out, None, ws)
    assert e.value.status == -1
    bad = dp.Problem(dc)
    bad.c.k_centroids = None
    with pytest.raises(dp.DPError) as e:
        dp.dp_score_centroids(bad, torch.empty(4 * 64, dtype=torch.float32, device="cuda:0"))
    assert e.value.status == -1
    torch.cuda.synchronize()


def test_score_centroids_timed_stamps_the_kernel():
    """The measurement entry point gives the same logits and a plausible kernel duration."""
    import ctypes
    import torch
    import paper_2602_05191_amd as dp
    c = make_config(1, shrink=4)
    dc = dp.DeviceCache.from_host(c)
    pr = dp.Problem(dc)
    n = c.group * int(c.seg_cluster_ptr[-1])
    a = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    b = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    hip = ctypes.CDLL("libamdhip64.so")
    e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0
    dp.dp_score_centroids(pr, a)
    dp.dp_score_centroids_timed(pr, b, e0, e1)
    torch.cuda.synchronize()
    ms = ctypes.c_float()
    assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
    assert 0.0 < ms.value < 5.0
    assert torch.equal(a, b)
    hip.hipEventDestroy(e0)
    hip.hipEventDestroy(e1)


def test_decode_attention_timed_stamps_the_three_kernels():
    """The measurement variant of the one-call path: same output bits, and per-kernel durations that
    are positive, ordered and shorter than the whole."""
    import ctypes
    import torch
    import paper_2602_05191_amd as dp
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=20000, mean_cluster=16, q_scale=0.4, seed=81)
    dc = dp.DeviceCache.from_host(c)
    pr = dp.Problem(dc)
    ws = torch.zeros(dp.dp_workspace_bytes(pr), dtype=torch.uint8, device="cuda:0")
    a = torch.zeros((1, 8, 128), dtype=torch.float32, device="cuda:0")
    b = torch.zeros_like(a)
    hip = ctypes.CDLL("libamdhip64.so")
    ev = [ctypes.c_void_p() for _ in range(6)]
    for e in ev:
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
    dp.dp_decode_attention(pr, 0.95, 0.9, a, None, ws)
    dp.dp_decode_attention_timed(pr, 0.95, 0.9, b, None, ws, ev)
    torch.cuda.synchronize()
    assert torch.equal(a, b)

    def us(x, y):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), x, y) == 0
        return ms.value * 1e3

    durations = [us(ev[0], ev[1]), us(ev[2], ev[3]), us(ev[4], ev[5])]
    assert all(0.0 < d < 5000.0 for d in durations), durations
    assert us(ev[1], ev[2]) >= 0.0 and us(ev[3], ev[4]) >= 0.0          # the kernels run one after the other
    assert us(ev[0], ev[5]) >= sum(durations) - 1.0
    for e in ev:
        hip.hipEventDestroy(e)


def test_launch_count_and_stream_read_probe():
    """Host-only launch count of the one-call entry point, and the loads-only measurement kernel (reads a buffer,
    writes nothing, stamps its events)."""
    import ctypes
    import torch
    import paper_2602_05191_amd as dp
    small = dp.Problem(dp.DeviceCache.from_host(make_config(0)))
    assert dp.dp_decode_attention_launches(small) == 2                      # 4 heads, 256 clusters: shared launch
    sep = dp.Problem(small.dc, flags=dp.DP_FLAG_SEPARATE_DECODE_LAUNCH)
    assert dp.dp_decode_attention_launches(sep) == 3
    mid = make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=16000, mean_cluster=8, q_scale=1.0, seed=83)
    assert dp.dp_decode_attention_launches(dp.Problem(dp.DeviceCache.from_host(mid))) == 2   # 2000 clusters per segment
    many = make_cache(batch=5, n_kv_heads=8, n_q_heads=32, context=256, mean_cluster=8, q_scale=1.0, seed=84)
    assert dp.dp_decode_attention_launches(dp.Problem(dp.DeviceCache.from_host(many))) == 3  # 160 heads: own decode launch
    buf = torch.arange(1 << 20, dtype=torch.int32, device="cuda:0")
    before = buf.clone()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    hip = ctypes.CDLL("libamdhip64.so")
    e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0
    dp.dp_stream_read_probe(buf, sink)
    dp.dp_stream_read_probe(buf[: 4 * 1000], None, None, e0, e1)           # a size that is no multiple of a tile
    torch.cuda.synchronize()
    ms = ctypes.c_float()
    assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0 and 0.0 < ms.value < 5.0
    assert torch.equal(buf, before) and int(sink.item()) == 0
    with pytest.raises(dp.DPError):
        dp.dp_stream_read_probe(buf.view(torch.int8)[1:17])                 # not 16-byte aligned
    hip.hipEventDestroy(e0)
    hip.hipEventDestroy(e1)


# ---------------------------------------------------------------------------
# the entry points hold no state: two streams at once, and HIP graph capture
# ---------------------------------------------------------------------------
def test_two_streams_with_own_workspaces_do_not_interfere():
    import torch
    import paper_2602_05191_amd as dp
    ca = make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=30000, mean_cluster=16, q_scale=0.4, seed=91)
    cb = make_cache(batch=2, n_kv_heads=2, n_q_heads=4, context=[9000, 4000], mean_cluster=16, q_scale=2.0, seed=92)
    runs = []
    for c in (ca, cb):
        pr = dp.Problem(dp.DeviceCache.from_host(c))
        ws = torch.zeros(dp.dp_workspace_bytes(pr), dtype=torch.uint8, device="cuda:0")
        ref = torch.zeros((c.batch, c.n_q_heads, 128), dtype=torch.float32, device="cuda:0")
        dp.dp_decode_attention(pr, 0.95, 0.9, ref, None, ws)
        runs.append((pr, ws, ref, torch.zeros_like(ref), torch.cuda.Stream()))
    torch.cuda.synchronize()
    for _ in range(20):
        for pr, ws, ref, out, st in runs:
            with torch.cuda.stream(st):
                dp.dp_decode_attention(pr, 0.95, 0.9, out, None, ws)
    torch.cuda.synchronize()
    for pr, ws, ref, out, st in runs:
        assert torch.equal(out, ref)


def test_one_call_path_replays_from_a_hip_graph():
    """Capture dp_decode_attention into a graph and replay it with other queries; every replay must equal
    the eager result on the same inputs (eager work and synchronisations in between)."""
    import torch
    import paper_2602_05191_amd as dp
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=24000, mean_cluster=16,
                   q_scale=lambda rng, b, h: 0.4 if h % 2 else 3.0, seed=93)
    dc = dp.DeviceCache.from_host(c)
    pr = dp.Problem(dc)
    ws = torch.zeros(dp.dp_workspace_bytes(pr), dtype=torch.uint8, device="cuda:0")
    out = torch.zeros((1, 8, 128), dtype=torch.float32, device="cuda:0")
    lse = torch.zeros(8, dtype=torch.float32, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dp.dp_decode_attention(pr, 0.95, 0.9, out, lse, ws)          # warm up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        dp.dp_decode_attention(pr, 0.95, 0.9, out, lse, ws)
    rng = np.random.default_rng(3)
    q0 = dc.q.clone()
    for rep in range(4):
        if rep:                                                      # a new query at the same address
            perm = torch.from_numpy(rng.permutation(8)).cuda()
            dc.q.copy_(q0[:, perm])
        g.replay()
        torch.cuda.synchronize()
        got, got_lse = out.clone(), lse.clone()
        eager, eager_lse = torch.zeros_like(out), torch.zeros_like(lse)
        dp.dp_decode_attention(pr, 0.95, 0.9, eager, eager_lse, ws)
        torch.cuda.synchronize()
        assert torch.equal(got, eager) and torch.equal(got_lse, eager_lse), rep


# ---------------------------------------------------------------------------
# A/B variant in the paper's own kernel structure: sort first, then prefix sums (Sec. 4.4)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("flags", [0, 1])
def test_sorted_select_variant_gives_the_same_sets(case, flags):
    """Same masses, same order, same tie-break: identical outputs to dp_topp_select, and to the oracle
    under the same rule as dp_topp_select."""
    import paper_2602_05191_amd as dp
    name, cache, p1, p2, orc = case
    if cache.max_clusters_per_seg > 8192 or cache.cluster_flags is not None:
        with pytest.raises(dp.DPError) as e:
            H.gpu_select(cache, H.gpu_logits(cache)[1], p1, p2, flags, budget="sorted")
        assert e.value.status == -2
        return
    per_head, flat = H.gpu_logits(cache)
    for (q1, q2) in ((p1, p2), (0.5, 0.5), (1.0, 1.0), (0.9, 0.0), (1.0, 0.6), (0.999, 0.999)):
        ex_a, ap_a, nt_a = H.gpu_select(cache, flat, q1, q2, flags)
        ex_b, ap_b, nt_b = H.gpu_select(cache, flat, q1, q2, flags, budget="sorted")
        for i in range(cache.batch * cache.n_q_heads):
            assert np.array_equal(ex_a[i], ex_b[i]) and np.array_equal(ap_a[i], ap_b[i]), (name, q1, q2, i)
        assert np.array_equal(nt_a, nt_b)


def test_sorted_select_variant_on_ties():
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=2, context=3000, n_clusters=3000, size_dist="ones", size_lo=1,
                   size_hi=1, q_scale=0.5, seed=43)
    for start in range(0, 3000, 60):
        c.k_centroids[start:start + 41] = c.k_centroids[start]     # runs of equal scores
    _, flat = H.gpu_logits(c)
    for q1, q2 in ((0.5, 0.5), (0.9, 0.8), (0.97, 0.2)):
        ex_a, ap_a, _ = H.gpu_select(c, flat, q1, q2)
        ex_b, ap_b, _ = H.gpu_select(c, flat, q1, q2, budget="sorted")
        for i in range(2):
            assert np.array_equal(ex_a[i], ex_b[i]) and np.array_equal(ap_a[i], ap_b[i])


@pytest.mark.parametrize("rows_cap", [64, 700, 100000])
def test_gathered_decode_variant_gives_the_same_bits(case, rows_cap):
    """Copying the exact rows into a contiguous per-head buffer first changes where the rows are read from,
    not what is computed: the output must equal dp_sparse_decode's bit for bit (heads that do not fit the
    buffer are read in place)."""
    import torch
    import paper_2602_05191_amd as dp
    name, cache, p1, p2, orc = case
    r = orc.decode_step(p1, p2)
    nh, mk = cache.batch * cache.n_q_heads, max(cache.max_clusters_per_seg, 1)
    sel = np.full((nh, mk), -1, dtype=np.int32)
    ne, nr = np.zeros(nh, np.int32), np.zeros(nh, np.int32)
    most = 0
    for i in range(nh):
        b, h = divmod(i, cache.n_q_heads)
        ex = np.sort(np.concatenate([orc.pinned_clusters(b, h), r.order[i, : r.k2.flat[i]]]))
        ap = np.sort(r.order[i, r.k2.flat[i]: r.k1.flat[i]])
        ne[i], nr[i] = len(ex), len(ex) + len(ap)
        sel[i, :ne[i]], sel[i, ne[i]:nr[i]] = ex, ap
        c0 = int(cache.seg_cluster_ptr[b * cache.n_kv_heads + h // cache.group])
        most = max(most, int(cache.cluster_sizes[c0 + ex].sum()))
    cap = min(rows_cap, max(most, 1) + 5)
    dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc)
    ws = torch.zeros(max(dp.dp_workspace_bytes(pr), 256), dtype=torch.uint8, device="cuda:0")
    sel_d, ne_d, nr_d = torch.from_numpy(sel).cuda(), torch.from_numpy(ne).cuda(), torch.from_numpy(nr).cuda()
    a = torch.full((cache.batch, cache.n_q_heads, 128), float("nan"), dtype=torch.float32, device="cuda:0")
    b_ = a.clone()
    la, lb = torch.zeros(nh, dtype=torch.float32, device="cuda:0"), torch.zeros(nh, dtype=torch.float32, device="cuda:0")
    kb = torch.zeros((nh, cap, 128), dtype=torch.int16, device="cuda:0")
    vb = torch.zeros_like(kb)
    dp.dp_sparse_decode(pr, sel_d, ne_d, nr_d, a, la, ws)
    dp.dp_sparse_decode_gathered(pr, sel_d, ne_d, nr_d, b_, lb, kb, vb, cap, ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b_) and torch.equal(la, lb), (name, rows_cap)


def test_group_union_variant_matches_oracle(case):
    """dp_group_union_decode_attention: the union lists must be exactly the union of the per-head sets that
    dp_topp_select returns on the same logits (integer work: bit-exact; those per-head sets are themselves
    checked against the oracle elsewhere), and every head's output must be the oracle's Eq. 8 / Eq. 9 over the
    union sets (the stated output tolerance)."""
    import torch
    import paper_2602_05191_amd as dp
    name, cache, p1, p2, orc = case
    n_seg, G = cache.batch * cache.n_kv_heads, cache.group
    nh, mk = cache.batch * cache.n_q_heads, max(cache.max_clusters_per_seg, 1)
    dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc)
    ws = torch.zeros(max(dp.dp_workspace_bytes(pr), 256), dtype=torch.uint8, device="cuda:0")
    out = torch.full((cache.batch, cache.n_q_heads, 128), float("nan"), dtype=torch.float32, device="cuda:0")
    lse = torch.full((nh,), float("nan"), dtype=torch.float32, device="cuda:0")
    uid = torch.full((n_seg, mk), -7, dtype=torch.int32, device="cuda:0")
    neu = torch.full((n_seg,), -7, dtype=torch.int32, device="cuda:0")
    nru = neu.clone()
    dp.dp_group_union_decode_attention(pr, p1, p2, out, lse, uid, neu, nru, ws)
    torch.cuda.synchronize()
    uid, neu, nru = uid.cpu().numpy(), neu.cpu().numpy(), nru.cpu().numpy()
    out, lse = out.cpu().numpy(), lse.cpu().numpy().reshape(cache.batch, cache.n_q_heads)
    # the per-head sets of the same library on the same logits
    _, flat = H.gpu_logits(cache)
    exact, approx, _ = H.gpu_select(cache, flat, p1, p2)
    worst = 0.0
    for seg in range(n_seg):
        b, g = divmod(seg, cache.n_kv_heads)
        heads = [b * cache.n_q_heads + g * G + j for j in range(G)]
        ex_want = set().union(*[set(exact[i].tolist()) for i in heads])
        rt_want = set().union(*[set(exact[i].tolist()) | set(approx[i].tolist()) for i in heads])
        ex_got, ap_got = uid[seg, :neu[seg]], uid[seg, neu[seg]:nru[seg]]
        assert ex_got.tolist() == sorted(ex_want), (name, seg)
        assert ap_got.tolist() == sorted(rt_want - ex_want), (name, seg)
        for i in heads:
            h = i % cache.n_q_heads
            if nru[seg] == 0:
                assert (out[b, h] == 0).all() and np.isneginf(lse[b, h])
                continue
            want, want_lse = orc.mixed_attention(b, h, ex_got, ap_got)
            err = np.abs(out[b, h] - want).max()
            worst = max(worst, err)
            assert err <= 1e-2 and err <= 2e-4, (name, seg, h, err)
            assert np.linalg.norm(out[b, h] - want) <= 5e-3 * max(np.linalg.norm(want), 1e-30) + 1e-6
            assert abs(lse[b, h] - want_lse) <= 1e-3
    print(f"[{name}] group-union variant: worst max-abs error {worst:.2e}")


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_match_oracle(seed):
    """Seeded random shapes through the one-call path: GQA groups of 1 to 16, one to three sequences of unequal
    length, cluster sizes from singletons to hundreds of tokens, flat / peaked / mixed heads, p1 and p2 at their
    limits, both readings of the second threshold, pinned and emptied clusters now and then."""
    from workloads import pin_sink_and_window
    rng = np.random.default_rng(4000 + seed)
    G = int(rng.choice([1, 2, 3, 4, 5, 6, 8, 12, 16]))
    nkv, batch = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    ctx = [int(rng.integers(40, 7000)) for _ in range(batch)]
    mc = int(rng.choice([3, 4, 8, 16, 32]))
    flat = rng.random() < 0.5
    qs = (lambda r, b, h: [0.3, 2.5, 0.7, 4.0][h % 4]) if rng.random() < 0.5 else (0.35 if flat else 3.0)
    p1 = float(rng.choice([0.8, 0.9, 0.95, 0.99, 1.0]))
    p2 = float(rng.choice([0.0, 0.5, 0.7, 0.9, 1.0]))
    c = make_cache(batch=batch, n_kv_heads=nkv, n_q_heads=nkv * G, context=ctx, mean_cluster=mc,
                   size_hi=int(rng.choice([2, 4, 8])) * mc, q_scale=qs, seed=5000 + seed)
    if rng.random() < 0.3:
        pin_sink_and_window(c, first=1, last=int(rng.integers(1, 4)))
    if rng.random() < 0.2:
        c.cluster_sizes[rng.integers(0, len(c.cluster_sizes), size=3)] = 0
    flags = int(rng.random() < 0.3)
    orc = oracle.Oracle(c)
    g = H.gpu_decode_attention(c, p1, p2, flags=flags)
    tolerated = H.check_sets(c, orc, g, p1, p2, flags)
    worst, _ = H.check_outputs(c, orc, g, tight=2e-4)
    print(f"[random {seed}] G {G}, {nkv} KV heads, contexts {ctx}, mean cluster {mc}, p {p1}/{p2}, flags {flags}: "
          f"tolerated {tolerated}, max-abs {worst:.1e}")
    assert tolerated <= max(1, (batch * nkv * G) // 20)
