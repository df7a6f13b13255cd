"""GPU parity of the k-means assignment step (dp_kmeans_assign, matrix cores) against the fp64 oracle.
Floating point decides an index here: the GPU takes the decision on fp32-accumulated scores, the oracle on
fp64 ones, so a token must get the oracle's centroid wherever the oracle's best score beats its runner-up by
more than the fp32 rounding of a 128-term sum; where it does not, the GPU's centroid must be one of the
near-best ones."""
import numpy as np
import pytest

import oracle
from workloads import bf16_bits_to_f32, make_cache, make_config, token_order_input

pytestmark = pytest.mark.gpu


def gpu_assign(t, centroids, want_score=True):
    import torch
    import paper_2602_05191_amd as dp
    dev = "cuda:0"
    up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)
    n_rows, n_cl = int(t.k_tokens.shape[0]), int(t.seg_cluster_ptr[-1])
    pf = dp.Prefill(up(t.k_tokens, np.int16), up(t.v_tokens, np.int16), up(t.assignment, np.int32),
                    up(t.seg_row_base, np.int64), up(t.seg_rows, np.int32), up(t.seg_cluster_ptr, np.int32),
                    n_cl, int(np.diff(t.seg_cluster_ptr).max()), int(t.seg_rows.max()))
    ws = torch.empty(max(dp.dp_kmeans_workspace_bytes(pf), 256), dtype=torch.uint8, device=dev)
    asg = torch.full((max(n_rows, 1),), -7, dtype=torch.int32, device=dev)
    score = torch.full((max(n_rows, 1),), float("nan"), dtype=torch.float32, device=dev) if want_score else None
    dp.dp_kmeans_assign(pf, up(centroids, np.int16), asg, ws, best_score=score)
    torch.cuda.synchronize()
    return asg.cpu().numpy()[:n_rows], (score.cpu().numpy()[:n_rows] if want_score else None)


def check_assign(t, centroids, got, got_score):
    ref, best, second = oracle.kmeans_assign(t, centroids)
    X = bf16_bits_to_f32(t.k_tokens).astype(np.float64)
    C = bf16_bits_to_f32(centroids).astype(np.float64)
    cn = np.sqrt((C ** 2).sum(1))
    n_diff = 0
    for seg in range(t.n_seg):
        r0, n = int(t.seg_row_base[seg]), int(t.seg_rows[seg])
        a, e = int(t.seg_cluster_ptr[seg]), int(t.seg_cluster_ptr[seg + 1])
        if e == a:
            assert (got[r0:r0 + n] == -1).all()
            continue
        g, r = got[r0:r0 + n], ref[r0:r0 + n]
        assert ((g >= 0) & (g < e - a)).all()
        # fp32 accumulation of 128 exact products: |error| <= 128 * 2^-24 * |x| |c|, taken with a factor 4 of slack
        tol = 4 * 128 * 2.0 ** -24 * np.sqrt((X[r0:r0 + n] ** 2).sum(1)) * cn[a:e].max() + 1e-6
        clear = (best[r0:r0 + n] - second[r0:r0 + n]) > 2 * tol
        assert np.array_equal(g[clear], r[clear]), f"segment {seg}: a token with a clear nearest centroid differs"
        # the others: the chosen centroid's exact score is within the tolerance of the best
        sc = (X[r0:r0 + n] * C[a + g]).sum(1) - 0.5 * (C[a + g] ** 2).sum(1)
        assert (sc >= best[r0:r0 + n] - 2 * tol).all()
        if got_score is not None:
            assert (np.abs(got_score[r0:r0 + n] - sc) <= tol).all()
        n_diff += int((g != r).sum())
    return n_diff


def sampled_centroids(t, seed):
    """One token of the segment per centroid (a usual k-means initialisation)."""
    rng = np.random.default_rng(seed)
    out = np.zeros((int(t.seg_cluster_ptr[-1]), t.head_dim), np.uint16)
    for seg in range(t.n_seg):
        r0, n = int(t.seg_row_base[seg]), int(t.seg_rows[seg])
        a, e = int(t.seg_cluster_ptr[seg]), int(t.seg_cluster_ptr[seg + 1])
        if n and e > a:
            out[a:e] = t.k_tokens[r0 + rng.choice(n, size=e - a, replace=(e - a) > n)]
    return out


CASES = {
    "ragged": lambda: make_cache(batch=2, n_kv_heads=2, n_q_heads=4, context=[3000, 1777], mean_cluster=16, q_scale=1.0,
                                 seed=71),
    "tiny": lambda: make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=37, n_clusters=5, size_lo=1, size_hi=30,
                               q_scale=1.0, seed=72),
    "one_centroid": lambda: make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=300, n_clusters=1, size_lo=1,
                                       size_hi=400, q_scale=1.0, seed=73),
    "many_centroids": lambda: make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=9000, mean_cluster=3, size_hi=8,
                                         q_scale=1.0, seed=74),
    "cfg1_quarter": lambda: make_config(1, shrink=4),
}


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("init", ["means", "sampled"])
def test_kmeans_assign_matches_oracle(name, init):
    c = CASES[name]()
    t = token_order_input(c, seed=5)
    cent = c.k_centroids if init == "means" else sampled_centroids(t, 6)
    got, score = gpu_assign(t, cent)
    n_diff = check_assign(t, cent, got, score)
    print(f"[{name}/{init}] {n_diff} of {len(got)} tokens took another near-tied centroid")
    assert n_diff <= max(2, len(got) // 200)


def test_kmeans_assign_exact_ties_go_to_the_lower_index():
    c = CASES["ragged"]()
    t = token_order_input(c, seed=7)
    cent = sampled_centroids(t, 8)
    a, e = int(t.seg_cluster_ptr[0]), int(t.seg_cluster_ptr[1])
    cent[a + 40:a + 60] = cent[a + 3]            # 20 copies of centroid 3, all at higher indices
    cent[e - 1] = cent[a]                        # and a copy of centroid 0 in the last, partial tile
    got, _ = gpu_assign(t, cent, want_score=False)
    ref, _, _ = oracle.kmeans_assign(t, cent)
    n0 = int(t.seg_rows[0])
    assert not np.isin(got[:n0], np.r_[np.arange(40, 60), e - a - 1]).any()
    assert (got[:n0] == 3).sum() == (ref[:n0] == 3).sum() > 0
    check_assign(t, cent, got, None)


def test_lloyd_iterations_on_the_gpu_do_not_increase_the_objective():
    """dp_kmeans_assign + dp_build_cluster_cache = one Lloyd iteration; everything stays on the device."""
    import torch
    import paper_2602_05191_amd as dp
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=2, context=6000, mean_cluster=16, q_scale=1.0, seed=75)
    t = token_order_input(c, seed=9)
    dev = "cuda:0"
    up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)
    n_rows, n_cl = int(t.k_tokens.shape[0]), int(t.seg_cluster_ptr[-1])
    asg = torch.zeros(n_rows, dtype=torch.int32, device=dev)
    pf = dp.Prefill(up(t.k_tokens, np.int16), up(t.v_tokens, np.int16), asg, up(t.seg_row_base, np.int64),
                    up(t.seg_rows, np.int32), up(t.seg_cluster_ptr, np.int32), n_cl,
                    int(np.diff(t.seg_cluster_ptr).max()), int(t.seg_rows.max()))
    ws = torch.empty(max(dp.dp_kmeans_workspace_bytes(pf), dp.dp_build_workspace_bytes(pf), 256), dtype=torch.uint8,
                     device=dev)
    cent = up(sampled_centroids(t, 10), np.int16)
    kc_, vc_ = torch.empty_like(cent), torch.empty_like(cent)
    kb, vb = torch.empty((n_rows, 128), dtype=torch.int16, device=dev), torch.empty((n_rows, 128), dtype=torch.int16, device=dev)
    off, sz = torch.empty(n_cl, dtype=torch.int32, device=dev), torch.empty(n_cl, dtype=torch.int32, device=dev)
    score = torch.empty(n_rows, dtype=torch.float32, device=dev)
    x2 = float((bf16_bits_to_f32(t.k_tokens).astype(np.float64) ** 2).sum())
    prev = None
    for it in range(5):
        dp.dp_kmeans_assign(pf, cent, asg, ws, best_score=score)
        obj = x2 - 2.0 * float(score.double().sum().item())
        assert prev is None or obj <= prev * (1 + 1e-4), (it, obj, prev)
        prev = obj
        dp.dp_build_cluster_cache(pf, kb, vb, off, sz, kc_, vc_, ws)
        cent = torch.where((sz > 0)[:, None], kc_, cent)     # an empty cluster keeps its old centroid
    assert obj < 0.9 * x2


# --------------------------------------------------------------------------
# k-means as a procedure (dp_kmeans_fit): Lloyd's rounds on the device
# --------------------------------------------------------------------------
def gpu_fit(t, centroids, n_iters, init):
    import torch
    import paper_2602_05191_amd as dp
    dev = "cuda:0"
    up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)
    n_rows, n_cl = int(t.k_tokens.shape[0]), int(t.seg_cluster_ptr[-1])
    pf = dp.Prefill(up(t.k_tokens, np.int16), up(t.v_tokens, np.int16), up(t.assignment, np.int32),
                    up(t.seg_row_base, np.int64), up(t.seg_rows, np.int32), up(t.seg_cluster_ptr, np.int32),
                    n_cl, int(np.diff(t.seg_cluster_ptr).max()), int(t.seg_rows.max()))
    ws = torch.full((max(dp.dp_kmeans_fit_workspace_bytes(pf), 256),), 0x5A, dtype=torch.uint8, device=dev)
    cent = up(centroids, np.int16) if centroids is not None else \
        torch.full((max(n_cl, 1), t.head_dim), 0x7FC0, dtype=torch.int16, device=dev)
    asg = torch.full((max(n_rows, 1),), -7, dtype=torch.int32, device=dev)
    score = torch.full((max(n_rows, 1),), float("nan"), dtype=torch.float32, device=dev)
    dp.dp_kmeans_fit(pf, cent, n_iters, init, asg, ws, best_score=score)
    torch.cuda.synchronize()
    return (cent.cpu().numpy().view(np.uint16)[:n_cl], asg.cpu().numpy()[:n_rows], score.cpu().numpy()[:n_rows])


def grouped_keys(seed, rows, clusters, groups=9):
    """Keys in well-separated groups, ragged segments (the last one has more clusters than tokens)."""
    from workloads import TokenOrderInput, f32_to_bf16_bits
    rng = np.random.default_rng(seed)
    d = 128
    ks = []
    for n in rows:
        centres = rng.normal(size=(groups, d)) * 4.0
        ks.append(centres[rng.integers(0, groups, size=n)] + 0.3 * rng.normal(size=(n, d)))
    k = f32_to_bf16_bits(np.concatenate(ks).astype(np.float32))
    rows = np.asarray(rows, np.int32)
    return TokenOrderInput(n_seg=len(rows), head_dim=d, k_tokens=k, v_tokens=k.copy(),
                           assignment=np.zeros(int(rows.sum()), np.int32),
                           seg_row_base=np.concatenate([[0], np.cumsum(rows)[:-1]]).astype(np.int64), seg_rows=rows,
                           seg_cluster_ptr=np.concatenate([[0], np.cumsum(clusters)]).astype(np.int32))


@pytest.mark.parametrize("n_iters", [0, 1, 4])
def test_kmeans_fit_matches_oracle_on_separated_groups(n_iters):
    """Points far from every boundary: the fp32 decisions of the GPU are the oracle's fp64 ones in every round, so
    centroids (bits) and assignment must be equal.  Strided start; clusters that never get a token keep it."""
    import paper_2602_05191_amd as dp
    t = grouped_keys(81, rows=[2100, 1300, 5], clusters=[12, 40, 9])
    ref_c, ref_a = oracle.kmeans_fit(t, None, n_iters, oracle.KMEANS_INIT_STRIDED)
    got_c, got_a, _ = gpu_fit(t, None, n_iters, dp.DP_KMEANS_INIT_STRIDED)
    assert np.array_equal(got_c, ref_c)
    if n_iters:
        assert np.array_equal(got_a, ref_a)
        assert (np.bincount(ref_a[-5:], minlength=9) == 0).any()      # the case does hold empty clusters
    else:
        assert (got_a == -7).all()                                     # nothing assigned, nothing written


def test_kmeans_fit_round_by_round_on_clustered_keys():
    """General keys (near-ties exist): round r is checked on its own.  From the GPU's centroids after r - 1 rounds,
    the GPU's assignment of round r must be the oracle's wherever the margin is clear (and near-best elsewhere), and
    the GPU's centroids after round r must be the oracle's means of THAT assignment bit for bit, an emptied cluster
    keeping its centroid."""
    import copy
    import paper_2602_05191_amd as dp
    c = make_cache(batch=2, n_kv_heads=1, n_q_heads=1, context=[5000, 3333], mean_cluster=16, q_scale=1.0, seed=83)
    t = token_order_input(c, seed=11)
    start = sampled_centroids(t, 12)
    start[3] = start[2]                                                # a duplicate: cluster 3 wins no token in round 1
    before = start
    for r in (1, 2, 3):
        cent, asg, score = gpu_fit(t, start, r, dp.DP_KMEANS_INIT_GIVEN)
        check_assign(t, before, asg, score)
        tt = copy.copy(t)
        tt.assignment = asg
        means = oracle.build_cluster_cache(tt)
        filled = means["cluster_sizes"] > 0
        assert r > 1 or not filled[3]
        assert np.array_equal(cent[filled], means["k_centroids"][filled])
        assert np.array_equal(cent[~filled], before[~filled])
        before = cent


def test_kmeans_fit_boundary_rejects_bad_arguments():
    import torch
    import paper_2602_05191_amd as dp
    t = grouped_keys(85, rows=[300], clusters=[4])
    dev = "cuda:0"
    up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)
    pf = dp.Prefill(up(t.k_tokens, np.int16), up(t.v_tokens, np.int16), up(t.assignment, np.int32),
                    up(t.seg_row_base, np.int64), up(t.seg_rows, np.int32), up(t.seg_cluster_ptr, np.int32), 4, 4, 300)
    need = dp.dp_kmeans_fit_workspace_bytes(pf)
    assert need >= dp.dp_kmeans_workspace_bytes(pf) and need >= dp.dp_build_workspace_bytes(pf)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    cent = torch.zeros((4, 128), dtype=torch.int16, device=dev)
    asg = torch.zeros(300, dtype=torch.int32, device=dev)
    for args, status in (((cent, -1, dp.DP_KMEANS_INIT_GIVEN, asg, ws), -1), ((cent, 1, 7, asg, ws), -1),
                         ((cent, 1, dp.DP_KMEANS_INIT_GIVEN, asg, ws[:need - 256]), -3),
                         ((cent, 1, dp.DP_KMEANS_INIT_GIVEN, None, ws), -1)):
        with pytest.raises(dp.DPError) as e:
            dp.dp_kmeans_fit(pf, *args)
        assert e.value.status == status
    dp.dp_kmeans_fit(pf, cent, 0, dp.DP_KMEANS_INIT_STRIDED, None, ws)    # only the start: no assignment needed
    torch.cuda.synchronize()
    assert np.array_equal(cent.cpu().numpy().view(np.uint16), t.k_tokens[[0, 75, 150, 225]])
