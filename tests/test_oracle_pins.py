"""Pins for the fp64 CPU oracle: each test ties it to something other than
itself -- a hand-worked example, an independent library routine (scipy
softmax / logsumexp), a closed form, brute force, or an invariant that follows
from the paper's equations.  CPU only."""
import itertools
import json
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import oracle
from workloads import ClusteredCache, bf16_bits_to_f32, f32_to_bf16_bits, make_cache, make_config

HERE = os.path.dirname(os.path.abspath(__file__))


# --------------------------------------------------------------------------
# helpers that build small caches by hand (inputs only)
# --------------------------------------------------------------------------
def cache_from_clusters(q_rows, clusters, d, n_kv_heads=1):
    """clusters: list of (keys[s,d], values[s,d], k_centroid[d], v_centroid[d]); one KV head."""
    ks, vs, kc, vc, sizes = [], [], [], [], []
    for keys, vals, c_k, c_v in clusters:
        keys = np.asarray(keys, dtype=np.float32).reshape(-1, d)
        vals = np.asarray(vals, dtype=np.float32).reshape(-1, d)
        ks.append(keys), vs.append(vals)
        kc.append(np.asarray(c_k, dtype=np.float32)), vc.append(np.asarray(c_v, dtype=np.float32))
        sizes.append(keys.shape[0])
    sizes = np.asarray(sizes, dtype=np.int32)
    offsets = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.int32)
    q = f32_to_bf16_bits(np.asarray(q_rows, dtype=np.float32).reshape(1, -1, d))
    return ClusteredCache(
        batch=1, n_kv_heads=1, n_q_heads=q.shape[1], head_dim=d, q=q,
        k_cache=f32_to_bf16_bits(np.concatenate(ks) if ks else np.zeros((0, d), np.float32)),
        v_cache=f32_to_bf16_bits(np.concatenate(vs) if vs else np.zeros((0, d), np.float32)),
        seg_row_base=np.zeros(1, np.int64), seg_cluster_ptr=np.array([0, len(clusters)], np.int32),
        cluster_offsets=offsets, cluster_sizes=sizes,
        k_centroids=f32_to_bf16_bits(np.stack(kc)), v_centroids=f32_to_bf16_bits(np.stack(vc)))


def scipy_dense(cache, b, h, rows=None, sm_scale=None):
    """Independent dense softmax attention (Eq. 1) with scipy, over `rows` of the head's segment."""
    d = cache.head_dim
    seg = b * cache.n_kv_heads + h // cache.group
    base = int(cache.seg_row_base[seg])
    a, e = int(cache.seg_cluster_ptr[seg]), int(cache.seg_cluster_ptr[seg + 1])
    if rows is None:
        rows = np.concatenate([np.arange(o, o + s) for o, s in
                               zip(cache.cluster_offsets[a:e], cache.cluster_sizes[a:e])] or [np.zeros(0, int)])
    rows = base + np.asarray(rows, dtype=np.int64)
    K = bf16_bits_to_f32(cache.k_cache[rows]).astype(np.float64)
    V = bf16_bits_to_f32(cache.v_cache[rows]).astype(np.float64)
    q = bf16_bits_to_f32(cache.q[b, h]).astype(np.float64)
    x = (K @ q) * (sm_scale if sm_scale else 1.0 / math.sqrt(d))
    return softmax(x) @ V, float(logsumexp(x))


def rows_of(cache, seg, cluster_ids):
    a = int(cache.seg_cluster_ptr[seg])
    out = [np.arange(cache.cluster_offsets[a + c], cache.cluster_offsets[a + c] + cache.cluster_sizes[a + c])
           for c in cluster_ids]
    return np.concatenate(out) if out else np.zeros(0, dtype=np.int64)


# --------------------------------------------------------------------------
# hand-worked example (tests/golden/hand_worked_case.json)
# --------------------------------------------------------------------------
@pytest.fixture(scope="module")
def hand():
    with open(os.path.join(HERE, "golden", "hand_worked_case.json")) as f:
        g = json.load(f)
    cl = [(c["keys"], c["values"], c["k_centroid"], c["v_centroid"]) for c in g["clusters"]]
    cache = cache_from_clusters([g["q"]], cl, d=2)
    return g, cache, oracle.Oracle(cache, sm_scale=math.log(2.0))


def test_hand_case_estimated_and_exact_masses(hand):
    g, cache, o = hand
    e = g["expected"]
    logit = o.centroid_logits(0, 0)
    np.testing.assert_allclose(np.exp(logit), e["Zhat"], rtol=1e-14)                      # Eq. 5
    np.testing.assert_allclose(np.exp(o.exact_cluster_log_mass(0, 0)), e["Z_exact"], rtol=1e-14)   # Eq. 4
    a_hat = o.cluster_distribution(logit)
    np.testing.assert_allclose(a_hat, np.array(e["A_hat_num"]) / e["A_hat_den"], rtol=1e-14)        # Eq. 6
    assert o.sorted_order(logit).tolist() == e["order"]


def test_hand_case_selection_and_output(hand):
    g, cache, o = hand
    e = g["expected"]
    logit = o.centroid_logits(0, 0)
    s = o.select(logit, e["p1"], 0.5)
    assert (s.k1, s.k2) == (e["k1"], e["p2_0.5"]["k2"])
    assert s.m1 == pytest.approx(e["m1_num"] / e["m1_den"], rel=1e-14)
    out, lse = o.mixed_attention(0, 0, s.exact, s.approx)
    np.testing.assert_allclose(out, np.array(e["p2_0.5"]["out_num"]) / e["p2_0.5"]["out_den"], rtol=1e-14)
    assert lse == pytest.approx(math.log(e["p2_0.5"]["Z_tilde"]), rel=1e-14)
    # the two readings of the second top-p separate at p2 = 0.6
    assert o.select(logit, e["p1"], 0.6).k2 == e["p2_0.6_renormalised"]["k2"]
    sa = o.select(logit, e["p1"], 0.6, flags=oracle.P2_ABSOLUTE)
    assert sa.k2 == e["p2_0.6_absolute"]["k2"]
    outa, lsea = o.mixed_attention(0, 0, sa.exact, sa.approx)                                # Eq. 8, Eq. 9 on those sets
    np.testing.assert_allclose(outa, np.array(e["p2_0.6_absolute"]["out_num"]) / e["p2_0.6_absolute"]["out_den"],
                               rtol=1e-14)
    assert lsea == pytest.approx(math.log(e["p2_0.6_absolute"]["Z_tilde"]), rel=1e-14)
    # p2 = 0: everything retained is approximated
    s0 = o.select(logit, e["p1"], 0.0)
    assert s0.k2 == 0
    out0, lse0 = o.mixed_attention(0, 0, s0.exact, s0.approx)
    np.testing.assert_allclose(out0, [1.0, 1.0], rtol=1e-14)
    assert lse0 == pytest.approx(math.log(e["p2_0"]["Z_tilde"]), rel=1e-14)


def test_hand_case_whole_step_and_dense(hand):
    g, cache, o = hand
    e = g["expected"]
    r = o.decode_step(e["p1"], 0.5)
    np.testing.assert_allclose(r.out[0, 0], np.array(e["p2_0.5"]["out_num"]) / e["p2_0.5"]["out_den"], rtol=1e-14)
    assert (int(r.k1[0, 0]), int(r.k2[0, 0])) == (e["k1"], e["p2_0.5"]["k2"])
    assert r.order[0, :3].tolist() == e["order"]
    dn, lse = o.dense_attention(0, 0)
    np.testing.assert_allclose(dn, np.array(e["dense"]["out_num"]) / e["dense"]["out_den"], rtol=1e-14)
    assert lse == pytest.approx(math.log(e["dense"]["Z"]), rel=1e-14)
    # p1 = p2 = 1 is the dense result
    r1 = o.decode_step(1.0, 1.0)
    np.testing.assert_allclose(r1.out[0, 0], dn, rtol=1e-14)


# --------------------------------------------------------------------------
# Eq. 1 dense limit against scipy
# --------------------------------------------------------------------------
@pytest.mark.parametrize("seed", [0, 1])
def test_dense_limit_equals_scipy_softmax_attention(seed):
    c = make_cache(batch=2, n_kv_heads=2, n_q_heads=4, context=[384, 256], mean_cluster=16, q_scale=1.0, seed=seed)
    o = oracle.Oracle(c)
    r = o.decode_step(1.0, 1.0)
    for b in range(c.batch):
        for h in range(c.n_q_heads):
            ref, ref_lse = scipy_dense(c, b, h)
            np.testing.assert_allclose(r.out[b, h], ref, rtol=1e-11, atol=1e-13)
            assert r.lse[b, h] == pytest.approx(ref_lse, rel=1e-12)
            assert r.k1[b, h] == r.k2[b, h] == o.num_clusters(b, h)
            dn, dl = o.dense_attention(b, h)
            np.testing.assert_allclose(dn, ref, rtol=1e-11, atol=1e-13)
            assert dl == pytest.approx(ref_lse, rel=1e-12)


def test_centroid_logits_and_distribution_against_numpy_scipy():
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=512, mean_cluster=8, size_hi=32, q_scale=0.5, seed=3)
    o = oracle.Oracle(c)
    for h in range(c.n_q_heads):
        seg = h // c.group
        a, e = c.seg_cluster_ptr[seg], c.seg_cluster_ptr[seg + 1]
        KC = bf16_bits_to_f32(c.k_centroids[a:e]).astype(np.float64)
        q = bf16_bits_to_f32(c.q[0, h]).astype(np.float64)
        ref = KC @ q / math.sqrt(128) + np.log(c.cluster_sizes[a:e].astype(np.float64))
        got = o.centroid_logits(0, h)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(o.cluster_distribution(got), softmax(ref), rtol=1e-11)


# --------------------------------------------------------------------------
# singleton clusters: centroids are the keys, the estimate is exact
# --------------------------------------------------------------------------
def singleton_cache(seed, n=96, scale=0.6):
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=2, context=n, n_clusters=n, size_dist="ones", size_lo=1,
                   size_hi=1, q_scale=scale, seed=seed)
    assert (c.cluster_sizes == 1).all()
    assert (c.k_centroids == c.k_cache).all() and (c.v_centroids == c.v_cache).all()
    return c


@pytest.mark.parametrize("p2", [0.0, 0.3, 0.9, 1.0])
def test_singleton_clusters_p1_one_is_dense_for_any_p2(p2):
    c = singleton_cache(5)
    o = oracle.Oracle(c)
    r = o.decode_step(1.0, p2)
    for h in range(c.n_q_heads):
        ref, ref_lse = scipy_dense(c, 0, h)
        np.testing.assert_allclose(r.out[0, h], ref, rtol=1e-11, atol=1e-13)
        assert r.lse[0, h] == pytest.approx(ref_lse, rel=1e-12)


@pytest.mark.parametrize("p1,p2", [(0.5, 0.0), (0.8, 0.5), (0.95, 0.9)])
def test_singleton_clusters_give_token_level_top_p(p1, p2):
    c = singleton_cache(6)
    o = oracle.Oracle(c)
    r = o.decode_step(p1, p2)
    for h in range(c.n_q_heads):
        # token-level top-p computed independently: sort exact attention weights
        K = bf16_bits_to_f32(c.k_cache).astype(np.float64)
        q = bf16_bits_to_f32(c.q[0, h]).astype(np.float64)
        A = softmax(K @ q / math.sqrt(128))
        idx = np.argsort(-A, kind="stable")
        k = int(np.searchsorted(np.cumsum(A[idx]), p1, side="left")) + 1
        kept = np.sort(idx[:k])
        assert r.k1[0, h] == k
        assert np.array_equal(np.sort(r.order[h, :k]), kept)
        ref, ref_lse = scipy_dense(c, 0, h, rows=kept)
        np.testing.assert_allclose(r.out[0, h], ref, rtol=1e-11, atol=1e-13)   # independent of p2
        assert r.lse[0, h] == pytest.approx(ref_lse, rel=1e-12)


# --------------------------------------------------------------------------
# zero-variance clusters: Zhat_i V_mean_i equals the exact contribution
# --------------------------------------------------------------------------
def zero_variance_cache(seed, n_clusters=24, d=128):
    rng = np.random.default_rng(seed)
    sizes = rng.choice([1, 2, 4, 8], size=n_clusters)
    cl = []
    for s in sizes:
        centre = bf16_bits_to_f32(f32_to_bf16_bits(rng.standard_normal(d).astype(np.float32)))
        keys = np.repeat(centre[None], s, axis=0)
        # values on a 1/8 grid in [-1, 1] and power-of-two sizes: the mean is k/64, exact in bf16
        vals = rng.integers(-8, 9, size=(s, d)).astype(np.float32) / 8.0
        cl.append((keys, vals, centre, vals.mean(axis=0, dtype=np.float64)))
    q = rng.standard_normal((2, d)).astype(np.float32) * 1.5
    c = cache_from_clusters(q, cl, d)
    # the stored (bf16) value means must be the exact means for the identity to be exact
    for i, (_, vals, _, vm) in enumerate(cl):
        assert np.array_equal(bf16_bits_to_f32(c.v_centroids[i]).astype(np.float64), vm), i
    return c


@pytest.mark.parametrize("p1", [1.0, 0.7])
def test_zero_variance_clusters_output_independent_of_p2(p1):
    c = zero_variance_cache(11)
    o = oracle.Oracle(c)
    base = o.decode_step(p1, 0.0)
    for p2 in (0.25, 0.6, 0.9, 1.0):
        r = o.decode_step(p1, p2)
        assert (r.k1 == base.k1).all()
        np.testing.assert_allclose(r.out, base.out, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(r.lse, base.lse, rtol=1e-12)
    for h in range(c.n_q_heads):
        kept = np.sort(base.order[h, : base.k1[0, h]])
        ref, ref_lse = scipy_dense(c, 0, h, rows=rows_of(c, 0, kept))
        np.testing.assert_allclose(base.out[0, h], ref, rtol=1e-11, atol=1e-13)
        assert base.lse[0, h] == pytest.approx(ref_lse, rel=1e-12)


# --------------------------------------------------------------------------
# Jensen: Zhat_i <= Z_i when the centroid is the exact mean of the keys
# --------------------------------------------------------------------------
def symmetric_pairs_cache(seed, n_clusters=20, d=128):
    """Every cluster is centre +/- delta pairs on a 1/8 grid: its mean key is exactly the centre."""
    rng = np.random.default_rng(seed)
    cl = []
    for _ in range(n_clusters):
        centre = rng.integers(-16, 17, size=d).astype(np.float32) / 8.0
        npairs = int(rng.integers(1, 5))
        delta = rng.integers(-8, 9, size=(npairs, d)).astype(np.float32) / 8.0
        keys = np.concatenate([centre + delta, centre - delta])
        vals = rng.integers(-8, 9, size=(2 * npairs, d)).astype(np.float32) / 8.0
        vm = vals.mean(axis=0, dtype=np.float64).astype(np.float32)
        cl.append((keys, vals, centre, vm))
    q = rng.standard_normal((2, d)).astype(np.float32) * 0.5
    return cache_from_clusters(q, cl, d)


def test_jensen_bound_and_lse_monotone_in_p2():
    c = symmetric_pairs_cache(21)
    o = oracle.Oracle(c)
    for h in range(c.n_q_heads):
        log_zhat = o.centroid_logits(0, h)
        log_z = o.exact_cluster_log_mass(0, h)
        assert (log_zhat <= log_z + 1e-12).all()
        assert (log_zhat < log_z - 1e-6).any()          # strict somewhere: the test is not vacuous
    _, dense_lse, _ = o.dense_step()
    prev = None
    for p2 in (0.0, 0.2, 0.5, 0.8, 0.95, 1.0):
        r = o.decode_step(0.9, p2)
        assert (r.lse <= dense_lse + 1e-12).all()
        if prev is not None:
            assert (r.lse >= prev - 1e-12).all()
        prev = r.lse
    full = o.decode_step(1.0, 1.0)
    np.testing.assert_allclose(full.lse, dense_lse, rtol=1e-12)


# --------------------------------------------------------------------------
# p2 = 0 closed form (Eq. 9 with no exact cluster)
# --------------------------------------------------------------------------
def test_p2_zero_closed_form():
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=512, mean_cluster=8, size_hi=32, q_scale=0.4, seed=8)
    o = oracle.Oracle(c)
    r = o.decode_step(0.9, 0.0)
    VC = bf16_bits_to_f32(c.v_centroids).astype(np.float64)
    for h in range(4):
        assert r.k2[0, h] == 0
        a_hat = softmax(o.centroid_logits(0, h))
        kept = r.order[h, : r.k1[0, h]]
        m1 = a_hat[kept].sum()
        np.testing.assert_allclose(r.out[0, h], (a_hat[kept][:, None] * VC[kept]).sum(0) / m1, rtol=1e-10, atol=1e-13)


# --------------------------------------------------------------------------
# top-p: mass >= p, minimality, prefix structure, brute force
# --------------------------------------------------------------------------
def test_mass_and_minimality_on_cfg0_and_flat_heads():
    for c in (make_config(0), make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=2048, q_scale=0.3, seed=4)):
        o = oracle.Oracle(c)
        for p1, p2 in ((0.95, 0.9), (0.5, 0.5), (0.99, 0.1)):
            for h in range(c.n_q_heads):
                logit = o.centroid_logits(0, h)
                s = o.select(logit, p1, p2)
                a = softmax(logit)
                mass1 = a[s.order[: s.k1]].sum()
                assert mass1 >= p1 - 1e-15 and a[s.order[: s.k1 - 1]].sum() < p1
                tau2 = p2 * mass1
                assert a[s.order[: s.k2]].sum() >= tau2 - 1e-15
                assert s.k2 == 0 or a[s.order[: s.k2 - 1]].sum() < tau2
                assert 0 <= s.k2 <= s.k1 <= len(s.order)
                # order is non-increasing in score, index ascending among equals
                lo = logit[s.order]
                assert (np.diff(lo) <= 0).all()
                eq = np.diff(lo) == 0
                assert (np.diff(s.order)[eq] > 0).all()
                assert s.cum[s.k1 - 1] == pytest.approx(mass1, rel=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_top_p_against_brute_force_subsets(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(3, 12))
    logit = rng.standard_normal(n) * rng.uniform(0.3, 3.0)
    a = softmax(logit)
    o = oracle.Oracle(make_config(0, shrink=16))
    for p in (0.3, 0.6, 0.9, 0.99):
        s = o.select(logit, p, 1.0)
        best_size, best_mass, best_set = None, -1.0, None
        for r in range(1, n + 1):
            for sub in itertools.combinations(range(n), r):
                m = a[list(sub)].sum()
                if m >= p and (best_size is None or r < best_size or (r == best_size and m > best_mass)):
                    best_size, best_mass, best_set = r, m, sub
            if best_size is not None:
                break
        assert s.k1 == best_size
        assert set(s.order[: s.k1].tolist()) == set(best_set)


def test_threshold_is_inclusive_and_ties_go_to_lower_index():
    o = oracle.Oracle(make_config(0, shrink=16))
    a_hat = np.array([0.25, 0.5, 0.25])
    logit = np.log(a_hat)
    order = o.sorted_order(logit)
    assert order.tolist() == [1, 0, 2]                     # equal scores: lower index first
    k1, k2, m1, cum = o.double_top_p(a_hat, order, 0.75, 1.0)
    assert (k1, k2, m1) == (2, 2, 0.75)                    # reaching p exactly is enough (>=, not >)
    k1, k2, m1, _ = o.double_top_p(a_hat, order, 0.75 + 1e-12, 0.5)
    assert (k1, m1) == (3, 1.0) and k2 == 1                # 0.5 >= 0.5 * 1.0
    k1, k2, _, _ = o.double_top_p(a_hat, order, 1.0, 1.0)
    assert (k1, k2) == (3, 3)
    # all-equal scores
    eq = np.zeros(5)
    assert o.sorted_order(eq).tolist() == [0, 1, 2, 3, 4]
    s = o.select(eq, 0.5, 0.5)
    assert (s.k1, s.k2) == (3, 2)                          # 0.6 >= 0.5 ; then 0.4 >= 0.3
    # empty clusters are never ranked
    lg = np.array([0.0, -np.inf, 1.0])
    assert o.sorted_order(lg).tolist() == [2, 0]
    assert o.cluster_distribution(lg)[1] == 0.0


# --------------------------------------------------------------------------
# convex hull, permutation and shift invariances
# --------------------------------------------------------------------------
def test_output_in_convex_hull_and_invariances():
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=768, mean_cluster=12, size_hi=40, q_scale=0.5, seed=9)
    o = oracle.Oracle(c)
    r = o.decode_step(0.9, 0.6)
    V = bf16_bits_to_f32(c.v_cache).astype(np.float64)
    VC = bf16_bits_to_f32(c.v_centroids).astype(np.float64)
    for h in range(4):
        ex, ap = r.order[h, : r.k2[0, h]], r.order[h, r.k2[0, h]: r.k1[0, h]]
        cand = np.concatenate([V[rows_of(c, 0, ex)], VC[ap]])
        assert (r.out[0, h] <= cand.max(0) + 1e-12).all() and (r.out[0, h] >= cand.min(0) - 1e-12).all()

    # permute the clusters (rows move with them): same output, sets map through the permutation
    n = c.cluster_sizes.size
    perm = np.random.default_rng(1).permutation(n)
    new_rows = np.concatenate([np.arange(c.cluster_offsets[j], c.cluster_offsets[j] + c.cluster_sizes[j]) for j in perm])
    sizes = c.cluster_sizes[perm]
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.int32)
    c2 = ClusteredCache(batch=1, n_kv_heads=1, n_q_heads=4, head_dim=128, q=c.q, k_cache=c.k_cache[new_rows],
                        v_cache=c.v_cache[new_rows], seg_row_base=c.seg_row_base, seg_cluster_ptr=c.seg_cluster_ptr,
                        cluster_offsets=offs, cluster_sizes=sizes, k_centroids=c.k_centroids[perm],
                        v_centroids=c.v_centroids[perm])
    r2 = oracle.Oracle(c2).decode_step(0.9, 0.6)
    np.testing.assert_allclose(r2.out, r.out, rtol=1e-10, atol=1e-13)
    for h in range(4):
        assert r2.k1[0, h] == r.k1[0, h] and r2.k2[0, h] == r.k2[0, h]
        assert np.array_equal(perm[r2.order[h, : r.k1[0, h]]], r.order[h, : r.k1[0, h]])

    # adding a constant to every logit (= scaling all sizes) changes neither A_hat nor the sets
    lg = o.centroid_logits(0, 1)
    s_a, s_b = o.select(lg, 0.9, 0.6), o.select(lg + math.log(3.0), 0.9, 0.6)
    assert (s_a.k1, s_a.k2) == (s_b.k1, s_b.k2) and np.array_equal(s_a.order, s_b.order)
    np.testing.assert_allclose(s_a.a_hat, s_b.a_hat, rtol=1e-12)


def test_empty_segment_and_threads_agree():
    c = make_cache(batch=2, n_kv_heads=2, n_q_heads=4, context=[256, 128], q_scale=1.0, seed=2)
    # empty one cluster and a whole segment
    c.cluster_sizes[3] = 0
    a, e = c.seg_cluster_ptr[3], c.seg_cluster_ptr[4]
    c.cluster_sizes[a:e] = 0
    o = oracle.Oracle(c)
    r1 = o.decode_step(0.9, 0.5, n_threads=1)
    r4 = o.decode_step(0.9, 0.5, n_threads=4)
    assert np.array_equal(r1.out, r4.out) and np.array_equal(r1.k1, r4.k1) and np.array_equal(r1.order, r4.order)
    assert (r1.k1[1, 2:] == 0).all() and (r1.out[1, 2:] == 0).all() and np.isneginf(r1.lse[1, 2:]).all()
    assert 3 not in r1.order[0, : r1.k1[0, 0]].tolist()


# --------------------------------------------------------------------------
# fixed budget in place of the two thresholds (Sec. 5.1, the cluster-based baseline)
# --------------------------------------------------------------------------
def test_fixed_budget_is_the_numpy_top_k_with_index_ties():
    rng = np.random.default_rng(77)
    o = oracle.Oracle(make_config(0, shrink=16))
    for trial in range(20):
        n = int(rng.integers(1, 40))
        # few distinct values: many ties; some empty clusters (-inf)
        logit = rng.integers(-3, 3, size=n).astype(np.float64) * 0.5
        logit[rng.random(n) < 0.2] = -np.inf
        nonempty = np.flatnonzero(np.isfinite(logit))
        ref = nonempty[np.lexsort((nonempty, -logit[nonempty]))]  # score descending, then index ascending
        for kr, ke in ((0, 0), (1, 0), (1, 1), (3, 2), (5, 9), (n, 1), (n + 7, n + 7), (-2, 4)):
            s = o.fixed_budget(logit, kr, ke)
            k1 = min(max(kr, 0), len(ref))
            k2 = min(max(ke, 0), k1)
            assert (s.k1, s.k2) == (k1, k2)
            assert s.order[: s.k1].tolist() == ref[:k1].tolist()
            assert set(s.exact.tolist()) == set(ref[:k2].tolist())
            assert set(s.approx.tolist()) == set(ref[k2:k1].tolist())


def test_fixed_budget_with_the_top_p_counts_reproduces_the_top_p_step():
    """Cross-consistency: the budget step run with the counts the two thresholds chose is the same step."""
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=4, context=1536, mean_cluster=8, size_hi=32, q_scale=0.35, seed=21)
    o = oracle.Oracle(c)
    r = o.decode_step(0.9, 0.6)
    for h in range(4):
        logit = o.centroid_logits(0, h)
        s = o.fixed_budget(logit, int(r.k1[0, h]), int(r.k2[0, h]))
        t = o.select(logit, 0.9, 0.6)
        assert s.exact.tolist() == t.exact.tolist() and s.approx.tolist() == t.approx.tolist()
        out, lse = o.mixed_attention(0, h, s.exact, s.approx)
        np.testing.assert_allclose(out, r.out[0, h], rtol=1e-12, atol=1e-14)
        assert lse == pytest.approx(r.lse[0, h], rel=1e-12)


def test_budget_step_limits_and_threads():
    c = make_cache(batch=2, n_kv_heads=2, n_q_heads=4, context=[700, 300], mean_cluster=8, size_hi=32, q_scale=0.5,
                   seed=22)
    o = oracle.Oracle(c)
    kmax = int(np.diff(c.seg_cluster_ptr).max())
    # everything retained and exact: dense attention (Eq. 1), checked with scipy
    r = o.budget_step(kmax, kmax)
    for b in range(2):
        for h in range(4):
            ref, ref_lse = scipy_dense(c, b, h)
            np.testing.assert_allclose(r.out[b, h], ref, rtol=1e-9, atol=1e-12)
            assert r.lse[b, h] == pytest.approx(ref_lse, rel=1e-12)
    # one exact cluster, nothing else: attention over that cluster's tokens alone
    r = o.budget_step(1, 1)
    for b in range(2):
        for h in range(4):
            seg = b * c.n_kv_heads + h // c.group
            top = int(r.order[b * 4 + h, 0])
            ref, _ = scipy_dense(c, b, h, rows=rows_of(c, seg, [top]))
            np.testing.assert_allclose(r.out[b, h], ref, rtol=1e-9, atol=1e-12)
    # nothing exact: size-weighted average of the value centroids of the top clusters
    r = o.budget_step(5, 0)
    VC = bf16_bits_to_f32(c.v_centroids).astype(np.float64)
    for b in range(2):
        for h in range(4):
            seg = b * c.n_kv_heads + h // c.group
            a0 = int(c.seg_cluster_ptr[seg])
            logit = o.centroid_logits(b, h)
            kept = r.order[b * 4 + h, : r.k1[b, h]]
            w = softmax(logit[kept])
            np.testing.assert_allclose(r.out[b, h], (w[:, None] * VC[a0 + kept]).sum(0), rtol=1e-10, atol=1e-13)
    # nothing retained: zero output, lse = -inf
    r = o.budget_step(0, 0)
    assert (r.out == 0).all() and np.isneginf(r.lse).all()
    # threads agree
    a = o.budget_step(6, 2, n_threads=1)
    t = o.budget_step(6, 2, n_threads=4)
    assert (a.out == t.out).all() and (a.k1 == t.k1).all() and (a.k2 == t.k2).all()


# --------------------------------------------------------------------------
# pinned clusters (sink / window tokens of Sec. 5.1): out of the distribution, always exact
# --------------------------------------------------------------------------
def without_clusters(c, drop):
    """The same cache with the clusters `drop` (per-segment lists of local ids) removed from the cluster arrays
    (their K/V rows stay where they are, unreferenced)."""
    keep_all, ptr = [], [0]
    for seg in range(c.n_seg):
        a, e = int(c.seg_cluster_ptr[seg]), int(c.seg_cluster_ptr[seg + 1])
        keep = [a + i for i in range(e - a) if i not in set(drop[seg])]
        keep_all += keep
        ptr.append(len(keep_all))
    k = np.asarray(keep_all, dtype=np.int64)
    return ClusteredCache(batch=c.batch, n_kv_heads=c.n_kv_heads, n_q_heads=c.n_q_heads, head_dim=c.head_dim, q=c.q,
                          k_cache=c.k_cache, v_cache=c.v_cache, seg_row_base=c.seg_row_base,
                          seg_cluster_ptr=np.asarray(ptr, np.int32), cluster_offsets=c.cluster_offsets[k],
                          cluster_sizes=c.cluster_sizes[k], k_centroids=c.k_centroids[k], v_centroids=c.v_centroids[k])


def lse_merge(parts):
    """[(out, lse)] of attention over disjoint token sets -> (out, lse) over their union (Eq. 1 identity)."""
    lses = np.array([l for _, l in parts])
    tot = logsumexp(lses)
    w = np.exp(lses - tot)
    return sum(wi * o for wi, (o, _) in zip(w, parts)), float(tot)


def test_pinned_step_equals_middle_step_merged_with_dense_over_the_pinned_tokens():
    """Independent route: delete the pinned clusters from the cache, run the (already pinned) step on the rest,
    run scipy dense attention over the pinned tokens, and merge the two by their normalisers."""
    from workloads import pin_sink_and_window
    c = make_cache(batch=2, n_kv_heads=2, n_q_heads=8, context=[1500, 700], mean_cluster=8, size_hi=32, q_scale=0.5,
                   seed=31)
    pin_sink_and_window(c, first=1, last=3)
    c.cluster_sizes[int(c.seg_cluster_ptr[1]) - 1] = 0      # an EMPTY pinned cluster is ignored
    drop = []
    for seg in range(c.n_seg):
        a, e = int(c.seg_cluster_ptr[seg]), int(c.seg_cluster_ptr[seg + 1])
        drop.append([i for i in range(e - a) if c.cluster_flags[a + i] & 1])
    middle = oracle.Oracle(without_clusters(c, drop))
    o = oracle.Oracle(c)
    for p1, p2, fl in ((0.9, 0.6, 0), (0.95, 0.0, 0), (1.0, 1.0, 0), (0.8, 0.7, oracle.P2_ABSOLUTE)):
        r = o.decode_step(p1, p2, fl)
        m = middle.decode_step(p1, p2, fl)
        for b in range(c.batch):
            for h in range(c.n_q_heads):
                seg = b * c.n_kv_heads + h // c.group
                live = [i for i in drop[seg] if c.cluster_sizes[int(c.seg_cluster_ptr[seg]) + i] > 0]
                assert o.pinned_clusters(b, h).tolist() == live
                pin_out, pin_lse = scipy_dense(c, b, h, rows=rows_of(c, seg, live))
                want, want_lse = lse_merge([(m.out[b, h], m.lse[b, h]), (pin_out, pin_lse)])
                np.testing.assert_allclose(r.out[b, h], want, rtol=1e-9, atol=1e-12)
                assert r.lse[b, h] == pytest.approx(want_lse, rel=1e-12)
                assert (r.k1[b, h], r.k2[b, h]) == (m.k1[b, h], m.k2[b, h])
    # the same identity for the fixed budget
    r, m = o.budget_step(9, 3), middle.budget_step(9, 3)
    for b in range(c.batch):
        for h in range(c.n_q_heads):
            seg = b * c.n_kv_heads + h // c.group
            live = [i for i in drop[seg] if c.cluster_sizes[int(c.seg_cluster_ptr[seg]) + i] > 0]
            pin_out, pin_lse = scipy_dense(c, b, h, rows=rows_of(c, seg, live))
            want, want_lse = lse_merge([(m.out[b, h], m.lse[b, h]), (pin_out, pin_lse)])
            np.testing.assert_allclose(r.out[b, h], want, rtol=1e-9, atol=1e-12)


def test_pinned_special_cases():
    from workloads import pin_sink_and_window
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=600, mean_cluster=8, size_hi=32, q_scale=0.6, seed=32)
    n = int(c.seg_cluster_ptr[1])
    base = oracle.Oracle(c).decode_step(0.9, 0.5)
    # no flag set: the flags array changes nothing
    c.cluster_flags = np.zeros(n, np.uint8)
    r = oracle.Oracle(c).decode_step(0.9, 0.5)
    assert (r.out == base.out).all() and (r.k1 == base.k1).all() and (r.k2 == base.k2).all()
    # every cluster pinned: dense attention whatever p is; nothing is left for the distribution
    c.cluster_flags = np.ones(n, np.uint8)
    o = oracle.Oracle(c)
    r = o.decode_step(0.5, 0.0)
    for h in range(4):
        ref, ref_lse = scipy_dense(c, 0, h)
        np.testing.assert_allclose(r.out[0, h], ref, rtol=1e-9, atol=1e-12)
        assert r.k1[0, h] == 0 and r.k2[0, h] == 0 and np.isneginf(o.candidate_logits(0, h)).all()
    # candidate logits: -inf exactly at the pinned clusters, Eq. 3 + 5 elsewhere
    pin_sink_and_window(c, first=2, last=1)
    o = oracle.Oracle(c)
    full, cand = o.centroid_logits(0, 1), o.candidate_logits(0, 1)
    pinned = np.flatnonzero(c.cluster_flags & 1)
    assert pinned.tolist() == [0, 1, n - 1] and np.isneginf(cand[pinned]).all()
    rest = np.setdiff1d(np.arange(n), pinned)
    assert (cand[rest] == full[rest]).all()
    # selection helper: pinned ids are exact and never counted in k1 / k2
    s = o.select(full, 0.9, 0.5, pinned=o.pinned_clusters(0, 1))
    assert set(pinned.tolist()) <= set(s.exact.tolist()) and not set(pinned.tolist()) & set(s.order.tolist())
    assert len(s.exact) == s.k2 + len(pinned) and len(s.retained) == s.k1 + len(pinned)
    a = softmax(cand)
    assert a[s.order[: s.k1]].sum() >= 0.9 - 1e-15 and a[s.order[: s.k1 - 1]].sum() < 0.9


# --------------------------------------------------------------------------
# prefill side: cluster-contiguous cache and metadata (Sec. 4.1, Eq. 2)
# --------------------------------------------------------------------------
def test_build_cluster_cache_layout_against_numpy_stable_sort():
    from workloads import token_order_input
    c = make_cache(batch=2, n_kv_heads=2, n_q_heads=4, context=[900, 333], mean_cluster=8, size_hi=32, q_scale=1.0,
                   seed=41)
    t = token_order_input(c, seed=3)
    t.assignment[5] = -1                       # two tokens without a valid cluster are left out
    t.assignment[int(t.seg_row_base[2]) + 7] = 10 ** 6
    m = oracle.build_cluster_cache(t)
    for seg in range(t.n_seg):
        r0, n = int(t.seg_row_base[seg]), int(t.seg_rows[seg])
        a, e = int(t.seg_cluster_ptr[seg]), int(t.seg_cluster_ptr[seg + 1])
        asg = t.assignment[r0:r0 + n]
        valid = (asg >= 0) & (asg < e - a)
        sizes = np.bincount(asg[valid], minlength=e - a)
        assert np.array_equal(m["cluster_sizes"][a:e], sizes)
        assert np.array_equal(m["cluster_offsets"][a:e], np.concatenate([[0], np.cumsum(sizes)[:-1]]))
        order = np.flatnonzero(valid)[np.argsort(asg[valid], kind="stable")]   # cluster by cluster, token order kept
        assert np.array_equal(m["k_cache"][r0:r0 + len(order)], t.k_tokens[r0 + order])
        assert np.array_equal(m["v_cache"][r0:r0 + len(order)], t.v_tokens[r0 + order])
        row = m["token_row"][r0:r0 + n]
        assert (row[~valid] == -1).all() and np.array_equal(row[order], np.arange(len(order)))


def test_build_cluster_cache_means_are_exact_means_rounded_once():
    from fractions import Fraction
    from workloads import token_order_input
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=120, mean_cluster=6, size_hi=20, q_scale=1.0, seed=42)
    m = oracle.build_cluster_cache(token_order_input(c, seed=1))
    K, V = bf16_bits_to_f32(m["k_cache"]), bf16_bits_to_f32(m["v_cache"])

    def rne_bf16(fr):
        """Exact rational -> nearest bf16 (8 significant bits), ties to even, as a float."""
        if fr == 0:
            return 0.0
        sign, fr = (-1 if fr < 0 else 1), abs(fr)
        e = 0
        while fr >= 256:
            fr /= 2
            e += 1
        while fr < 128:
            fr *= 2
            e -= 1
        q, rem = divmod(fr.numerator, fr.denominator)
        twice = 2 * rem
        if twice > fr.denominator or (twice == fr.denominator and q % 2 == 1):
            q += 1
        return sign * float(Fraction(q) * Fraction(2) ** e)

    for i in range(len(m["cluster_sizes"])):
        s, off = int(m["cluster_sizes"][i]), int(m["cluster_offsets"][i])
        for j in (0, 17, 127):
            ks = sum(Fraction(float(x)) for x in K[off:off + s, j])
            vs = sum(Fraction(float(x)) for x in V[off:off + s, j])
            assert float(bf16_bits_to_f32(m["k_centroids"][i, j:j + 1])[0]) == rne_bf16(ks / s)
            assert float(bf16_bits_to_f32(m["v_centroids"][i, j:j + 1])[0]) == rne_bf16(vs / s)
            assert m["v_sums"][i, j] == pytest.approx(float(vs), rel=1e-14, abs=1e-300)


def test_decode_on_the_rebuilt_cache_equals_decode_on_the_original():
    """The method does not depend on the order of tokens inside a cluster: rebuilding the cache from a
    shuffled token order must give the same decode step (same sets, same output up to summation order)."""
    from workloads import token_order_input
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=4, context=2000, mean_cluster=10, size_hi=40, q_scale=0.5, seed=43)
    m = oracle.build_cluster_cache(token_order_input(c, seed=9))
    assert np.array_equal(m["cluster_sizes"], c.cluster_sizes) and np.array_equal(m["cluster_offsets"], c.cluster_offsets)
    # the generator's centroids are fp64 means of the same rows in another order: equal up to one bf16 ulp, rarely
    dk = np.abs(bf16_bits_to_f32(m["k_centroids"]).astype(np.float64) - bf16_bits_to_f32(c.k_centroids))
    assert (dk > 0).mean() < 1e-3 and (dk <= np.abs(bf16_bits_to_f32(c.k_centroids)) * 2.0 ** -7).all()
    rebuilt = ClusteredCache(batch=c.batch, n_kv_heads=c.n_kv_heads, n_q_heads=c.n_q_heads, head_dim=c.head_dim, q=c.q,
                             k_cache=m["k_cache"], v_cache=m["v_cache"], seg_row_base=c.seg_row_base,
                             seg_cluster_ptr=c.seg_cluster_ptr, cluster_offsets=m["cluster_offsets"],
                             cluster_sizes=m["cluster_sizes"], k_centroids=c.k_centroids, v_centroids=c.v_centroids)
    a, b = oracle.Oracle(c).decode_step(0.95, 0.7), oracle.Oracle(rebuilt).decode_step(0.95, 0.7)
    assert (a.k1 == b.k1).all() and (a.k2 == b.k2).all() and (a.order == b.order).all()
    np.testing.assert_allclose(a.out, b.out, rtol=1e-11, atol=1e-13)


# --------------------------------------------------------------------------
# k-means assignment step (Sec. 4.1)
# --------------------------------------------------------------------------
def test_kmeans_assign_is_scipys_nearest_centroid():
    from scipy.cluster.vq import vq
    from scipy.spatial.distance import cdist
    from workloads import token_order_input
    c = make_cache(batch=2, n_kv_heads=1, n_q_heads=1, context=[400, 150], mean_cluster=10, size_hi=40, q_scale=1.0,
                   seed=51)
    t = token_order_input(c, seed=2)
    rng = np.random.default_rng(4)
    cent = c.k_centroids.copy()
    cent[::3] = t.k_tokens[rng.integers(0, 400, size=len(cent[::3]))]          # some centroids are plain tokens
    asg, best, second = oracle.kmeans_assign(t, cent)
    X, C = bf16_bits_to_f32(t.k_tokens).astype(np.float64), bf16_bits_to_f32(cent).astype(np.float64)
    for seg in range(2):
        r0, n = int(t.seg_row_base[seg]), int(t.seg_rows[seg])
        a, e = int(t.seg_cluster_ptr[seg]), int(t.seg_cluster_ptr[seg + 1])
        code, dist = vq(X[r0:r0 + n], C[a:e])                                     # scipy's nearest code-book entry
        d2 = cdist(X[r0:r0 + n], C[a:e], "sqeuclidean")
        clear = (np.sort(d2, axis=1)[:, 1] - np.sort(d2, axis=1)[:, 0]) > 1e-9    # no near-tie
        assert clear.mean() > 0.95
        assert np.array_equal(asg[r0:r0 + n][clear], code[clear])
        # the score is the distance up to the token's own norm
        np.testing.assert_allclose((X[r0:r0 + n] ** 2).sum(1) - 2 * best[r0:r0 + n], dist ** 2, rtol=1e-9, atol=1e-9)
        np.testing.assert_allclose((X[r0:r0 + n] ** 2).sum(1) - 2 * second[r0:r0 + n], np.sort(d2, axis=1)[:, 1],
                                   rtol=1e-9, atol=1e-9)


def test_kmeans_assign_ties_go_to_the_lower_index_and_lloyd_does_not_increase_the_objective():
    from workloads import TokenOrderInput, token_order_input
    d = 128
    X = np.zeros((6, d), np.float32)
    X[:, 0] = [0, 1, 2, 3, 4, 5]
    C = np.zeros((3, d), np.float32)
    C[:, 0] = [1, 3, 3]                                                           # centroid 2 duplicates centroid 1
    t = TokenOrderInput(n_seg=1, head_dim=d, k_tokens=f32_to_bf16_bits(X), v_tokens=f32_to_bf16_bits(X),
                        assignment=np.zeros(6, np.int32), seg_row_base=np.zeros(1, np.int64),
                        seg_rows=np.array([6], np.int32), seg_cluster_ptr=np.array([0, 3], np.int32))
    asg, best, second = oracle.kmeans_assign(t, f32_to_bf16_bits(C))
    assert asg.tolist() == [0, 0, 0, 1, 1, 1]            # token 2 is equidistant from 1 and 3: lower index; never centroid 2
    # one Lloyd iteration (assign, then means) never increases the sum of squared distances in exact arithmetic;
    # with means rounded to bf16 it may move by the rounding, hence the small slack
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=1500, mean_cluster=12, size_hi=40, q_scale=1.0, seed=52)
    t = token_order_input(c, seed=3)
    cent = t.k_tokens[np.random.default_rng(5).choice(1500, size=int(c.seg_cluster_ptr[1]), replace=False)].copy()
    Xf = bf16_bits_to_f32(t.k_tokens).astype(np.float64)
    prev = None
    for it in range(4):
        asg, best, _ = oracle.kmeans_assign(t, cent)
        obj = float(((Xf ** 2).sum(1) - 2 * best).sum())
        assert prev is None or obj <= prev * (1 + 1e-4), (it, obj, prev)
        prev = obj
        t.assignment = asg
        m = oracle.build_cluster_cache(t)
        keep = m["cluster_sizes"] > 0                      # an empty cluster keeps its old centroid
        cent = np.where(keep[:, None], m["k_centroids"], cent)


def test_kmeans_fit_is_lloyds_iteration_as_a_library_runs_it():
    """Round r of the procedure against one iteration of scikit-learn's Lloyd started from the procedure's own
    centroids after r - 1 rounds (bf16 values, exact in fp64, so both sides assign on the same numbers): the
    library's new centres are the procedure's centroids up to the one rounding to bf16 (a wrongly assigned point
    would move a mean by more), and its assignment of the round is the procedure's."""
    from sklearn.cluster import KMeans
    from workloads import TokenOrderInput
    rng = np.random.default_rng(77)
    d, k, n = 128, 7, 900
    centres = rng.normal(size=(k, d)) * 4.0
    label = rng.integers(0, k, size=n)
    X = bf16_bits_to_f32(f32_to_bf16_bits((centres[label] + 0.3 * rng.normal(size=(n, d))).astype(np.float32)))
    t = TokenOrderInput(n_seg=1, head_dim=d, k_tokens=f32_to_bf16_bits(X), v_tokens=f32_to_bf16_bits(X),
                        assignment=np.zeros(n, np.int32), seg_row_base=np.zeros(1, np.int64),
                        seg_rows=np.array([n], np.int32), seg_cluster_ptr=np.array([0, k], np.int32))
    # a poor start on purpose (k arbitrary points: some groups are hit twice, some not at all): several rounds move
    start = f32_to_bf16_bits(X[rng.choice(n, size=k, replace=False)])
    prev, moved = start, 0
    for rounds in range(1, 7):
        cent, asg = oracle.kmeans_fit(t, start, rounds)
        km = KMeans(n_clusters=k, init=bf16_bits_to_f32(prev).astype(np.float64), n_init=1, max_iter=1, tol=0.0,
                    algorithm="lloyd")
        km.fit(X.astype(np.float64))
        # within half a bf16 step of the library's fp64 centres (bf16 inputs and small counts put many means exactly on
        # a rounding tie, where the library's last fp64 bit decides otherwise than the exact mean; the exact rounding
        # of the means is pinned with rational arithmetic in the build tests)
        ours = bf16_bits_to_f32(cent).astype(np.float64)
        assert (np.abs(ours - km.cluster_centers_) <= 2.0 ** -8 * np.abs(km.cluster_centers_) * (1 + 1e-9) + 1e-30).all()
        # the round's assignment = nearest of the previous centroids (the library's own predict on them)
        km.cluster_centers_ = bf16_bits_to_f32(prev).astype(np.float64)
        assert np.array_equal(asg, km.predict(X.astype(np.float64))), rounds
        moved += int(not np.array_equal(cent, prev))
        prev = cent
    assert moved >= 3            # the start was poor enough for the iteration to do something


def test_kmeans_fit_strided_start_empty_clusters_and_zero_rounds():
    from workloads import TokenOrderInput
    d = 128
    X = np.zeros((8, d), np.float32)
    X[:, 0] = [0, 0, 1, 1, 10, 10, 11, 11]
    t = TokenOrderInput(n_seg=2, head_dim=d, k_tokens=f32_to_bf16_bits(np.r_[X, X[:3]]),
                        v_tokens=f32_to_bf16_bits(np.r_[X, X[:3]]), assignment=np.zeros(11, np.int32),
                        seg_row_base=np.array([0, 8], np.int64), seg_rows=np.array([8, 3], np.int32),
                        seg_cluster_ptr=np.array([0, 4, 9], np.int32))
    cent, asg = oracle.kmeans_fit(t, None, 0, oracle.KMEANS_INIT_STRIDED)
    assert asg is None
    # segment 0: tokens 0, 2, 4, 6; segment 1 (3 tokens, 5 clusters): tokens 0, 0, 1, 1, 2
    assert bf16_bits_to_f32(cent)[:, 0].tolist() == [0, 1, 10, 11, 0, 0, 0, 0, 1]
    cent, asg = oracle.kmeans_fit(t, None, 2, oracle.KMEANS_INIT_STRIDED)
    assert asg[:8].tolist() == [0, 0, 1, 1, 2, 2, 3, 3]
    # duplicated start centroids: ties go to the lower index, the twin stays empty and keeps its centroid
    assert asg[8:].tolist() == [0, 0, 4]
    assert bf16_bits_to_f32(cent)[:, 0].tolist() == [0, 1, 10, 11, 0, 0, 0, 0, 1]


# --------------------------------------------------------------------------
# selection per GQA group (the union of the heads' sets; the paper states the method for one query)
# --------------------------------------------------------------------------
def test_group_union_with_one_head_per_group_is_the_per_head_step():
    c = make_cache(batch=2, n_kv_heads=3, n_q_heads=3, context=[300, 170], mean_cluster=8, size_hi=32, q_scale=0.5, seed=31)
    o = oracle.Oracle(c)
    out, lse, sets = o.group_union_step(0.9, 0.6)
    ref = o.decode_step(0.9, 0.6)
    assert np.array_equal(out, ref.out) and np.array_equal(lse, ref.lse)
    for (b, g), (ex, ap) in sets.items():
        assert ex.size == ref.k2[b, g] and ex.size + ap.size == ref.k1[b, g]


def test_group_union_sets_are_supersets_and_full_selection_is_dense():
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=600, mean_cluster=8, size_hi=32,
                   q_scale=lambda rng, b, h: [0.3, 3.0][h % 2], seed=32)
    o = oracle.Oracle(c)
    G = 4
    out, lse, sets = o.group_union_step(0.9, 0.7)
    for g in range(2):
        ex_u, ap_u = sets[(0, g)]
        assert not set(ex_u) & set(ap_u)
        exact_of, retained_of = [], []
        for h in range(g * G, (g + 1) * G):
            sel = o.select(o.centroid_logits(0, h), 0.9, 0.7)
            assert set(sel.exact) <= set(ex_u) and set(sel.retained) <= set(ex_u) | set(ap_u)
            exact_of.append(set(sel.exact)), retained_of.append(set(sel.retained))
            # every head's own retained mass is still covered: the union keeps at least p1 of its distribution
            a_hat = o.cluster_distribution(o.centroid_logits(0, h))
            assert a_hat[np.r_[ex_u, ap_u]].sum() >= 0.9 - 1e-12
        assert set(ex_u) == set().union(*exact_of) and set(ex_u) | set(ap_u) == set().union(*retained_of)
        # a cluster that one head approximates and another takes exactly is exact for the group
        assert all(i in ex_u for s_ex in exact_of for i in s_ex)
    # p1 = p2 = 1: every non-empty cluster exact for every head: dense attention (Eq. 1)
    out1, lse1, _ = o.group_union_step(1.0, 1.0)
    dense, dense_lse, _ = o.dense_step()
    assert np.allclose(out1, dense, rtol=0, atol=1e-12) and np.allclose(lse1, dense_lse, rtol=0, atol=1e-12)


def test_group_union_of_identical_queries_is_the_per_head_result():
    c = make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=400, mean_cluster=8, size_hi=32, q_scale=0.6, seed=33)
    c.q[0, 1:] = c.q[0, 0]
    o = oracle.Oracle(c)
    out, lse, sets = o.group_union_step(0.85, 0.5)
    ref = o.decode_step(0.85, 0.5)
    assert np.array_equal(out, ref.out) and np.array_equal(lse, ref.lse)
