"""GPU parity of the prefill-side build (dp_build_cluster_cache) against the oracle's: integer and byte work
(sizes, offsets, token rows, moved K / V rows) and the means (fp64 sums in row order, rounded once) are all
bit-exact by construction, so every output is compared for equality."""
import numpy as np
import pytest

import oracle
from workloads import bf16_bits_to_f32, make_cache, make_config, token_order_input

import harness as H

pytestmark = pytest.mark.gpu


def gpu_build(t, with_optional=True):
    import torch
    import paper_2602_05191_amd as dp
    dev = "cuda:0"
    up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)
    n_rows, n_cl, d = int(t.k_tokens.shape[0]), int(t.seg_cluster_ptr[-1]), t.head_dim
    kc_max = int(np.diff(t.seg_cluster_ptr).max()) if t.n_seg else 0
    rows_max = int(t.seg_rows.max()) if t.n_seg else 0
    pf = dp.Prefill(up(t.k_tokens, np.int16), up(t.v_tokens, np.int16), up(t.assignment, np.int32),
                    up(t.seg_row_base, np.int64), up(t.seg_rows, np.int32), up(t.seg_cluster_ptr, np.int32),
                    n_cl, kc_max, rows_max)
    ws = torch.full((max(dp.dp_build_workspace_bytes(pf), 256),), 0x5A, dtype=torch.uint8, device=dev)
    out = dict(k_cache=torch.full((max(n_rows, 1), d), 0x7FC0, dtype=torch.int16, device=dev),
               v_cache=torch.full((max(n_rows, 1), d), 0x7FC0, dtype=torch.int16, device=dev),
               cluster_offsets=torch.full((max(n_cl, 1),), -7, dtype=torch.int32, device=dev),
               cluster_sizes=torch.full((max(n_cl, 1),), -7, dtype=torch.int32, device=dev),
               k_centroids=torch.full((max(n_cl, 1), d), 0x7FC0, dtype=torch.int16, device=dev),
               v_centroids=torch.full((max(n_cl, 1), d), 0x7FC0, dtype=torch.int16, device=dev))
    v_sums = torch.full((max(n_cl, 1), d), float("nan"), dtype=torch.float32, device=dev) if with_optional else None
    token_row = torch.full((max(n_rows, 1),), -7, dtype=torch.int32, device=dev) if with_optional else None
    dp.dp_build_cluster_cache(pf, out["k_cache"], out["v_cache"], out["cluster_offsets"], out["cluster_sizes"],
                              out["k_centroids"], out["v_centroids"], ws, v_sums=v_sums, token_row=token_row)
    torch.cuda.synchronize()
    res = {k: v.cpu().numpy() for k, v in out.items()}
    for k in ("k_cache", "v_cache", "k_centroids", "v_centroids"):
        res[k] = res[k].view(np.uint16)
    res["k_cache"], res["v_cache"] = res["k_cache"][:n_rows], res["v_cache"][:n_rows]
    for k in ("cluster_offsets", "cluster_sizes", "k_centroids", "v_centroids"):
        res[k] = res[k][:n_cl]
    if with_optional:
        res["v_sums"], res["token_row"] = v_sums.cpu().numpy()[:n_cl], token_row.cpu().numpy()[:n_rows]
    return res


def check_build(t, got, ref):
    for k in ("cluster_sizes", "cluster_offsets", "token_row"):
        if k in got:
            assert np.array_equal(got[k], ref[k]), k
    # rows that hold a token (all rows unless tokens were left out)
    placed = ref["token_row"] >= 0
    for seg in range(t.n_seg):
        r0, n = int(t.seg_row_base[seg]), int(t.seg_rows[seg])
        used = int(placed[r0:r0 + n].sum())
        assert np.array_equal(got["k_cache"][r0:r0 + used], ref["k_cache"][r0:r0 + used]), ("k rows", seg)
        assert np.array_equal(got["v_cache"][r0:r0 + used], ref["v_cache"][r0:r0 + used]), ("v rows", seg)
    assert np.array_equal(got["k_centroids"], ref["k_centroids"])
    assert np.array_equal(got["v_centroids"], ref["v_centroids"])
    if "v_sums" in got:
        assert np.array_equal(got["v_sums"], ref["v_sums"].astype(np.float32))


CASES = {
    "ragged_small": lambda: make_cache(batch=2, n_kv_heads=2, n_q_heads=4, context=[3000, 1777], mean_cluster=16,
                                       q_scale=1.0, seed=61),
    "one_block": lambda: make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=700, mean_cluster=8, size_hi=32,
                                    q_scale=1.0, seed=62),
    "giant_clusters": lambda: make_cache(batch=1, n_kv_heads=2, n_q_heads=2, context=5000, n_clusters=6, size_lo=1,
                                         size_hi=4000, size_dist="pareto", mean_cluster=300, q_scale=1.0, seed=63),
    "singletons": lambda: make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=2500, n_clusters=2500,
                                     size_dist="ones", size_lo=1, size_hi=1, q_scale=1.0, seed=64),
    "many_clusters": lambda: make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=27000, mean_cluster=3, size_hi=8,
                                        q_scale=1.0, seed=65),
    # more than 16384 clusters in a segment: the per-block count table needs more LDS than a kernel gets by default
    "singletons_20k": lambda: make_cache(batch=1, n_kv_heads=1, n_q_heads=1, context=20000, n_clusters=20000,
                                         size_dist="ones", size_lo=1, size_hi=1, q_scale=1.0, seed=66),
    "cfg1_quarter": lambda: make_config(1, shrink=4),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_build_matches_oracle(name):
    t = token_order_input(CASES[name](), seed=5)
    got, ref = gpu_build(t), oracle.build_cluster_cache(t)
    check_build(t, got, ref)


def test_build_leaves_out_tokens_without_a_valid_cluster_and_handles_empty_clusters():
    c = make_cache(batch=2, n_kv_heads=1, n_q_heads=1, context=[2100, 900], mean_cluster=10, size_hi=40, q_scale=1.0,
                   seed=66)
    t = token_order_input(c, seed=6)
    rng = np.random.default_rng(7)
    bad = rng.choice(t.k_tokens.shape[0], size=40, replace=False)
    t.assignment[bad[:20]] = -3
    t.assignment[bad[20:]] = 10 ** 6
    t.assignment[t.assignment == 2] = 3          # cluster 2 of both segments ends up empty
    got, ref = gpu_build(t), oracle.build_cluster_cache(t)
    assert (ref["token_row"] == -1).sum() == 40 and (ref["cluster_sizes"] == 0).any()
    check_build(t, got, ref)
    empty = ref["cluster_sizes"] == 0
    assert (got["k_centroids"][empty] == 0).all() and (got["v_centroids"][empty] == 0).all()


def test_build_without_optional_outputs_and_twice_the_same_bits():
    t = token_order_input(CASES["ragged_small"](), seed=8)
    a, b = gpu_build(t, with_optional=False), gpu_build(t, with_optional=True)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_decode_on_a_gpu_built_cache_matches_the_oracle():
    """End to end: build on the GPU, then run the decode step on the built cache (device-resident) and
    compare with the oracle's step on the oracle-built cache."""
    import torch
    import paper_2602_05191_amd as dp
    from workloads import ClusteredCache
    c = make_cache(batch=1, n_kv_heads=2, n_q_heads=8, context=6000, mean_cluster=16, q_scale=0.5, seed=67)
    t = token_order_input(c, seed=9)
    got, ref = gpu_build(t), oracle.build_cluster_cache(t)
    check_build(t, got, ref)
    built = ClusteredCache(batch=c.batch, n_kv_heads=c.n_kv_heads, n_q_heads=c.n_q_heads, head_dim=c.head_dim, q=c.q,
                           k_cache=got["k_cache"], v_cache=got["v_cache"], seg_row_base=c.seg_row_base,
                           seg_cluster_ptr=c.seg_cluster_ptr, cluster_offsets=got["cluster_offsets"],
                           cluster_sizes=got["cluster_sizes"], k_centroids=got["k_centroids"],
                           v_centroids=got["v_centroids"])
    orc = oracle.Oracle(built)
    g = H.gpu_decode_attention(built, 0.95, 0.8)
    assert H.check_sets(built, orc, g, 0.95, 0.8) <= 1
    H.check_outputs(built, orc, g, tight=2e-4)


def test_build_boundary_rejects_bad_arguments():
    import torch
    import paper_2602_05191_amd as dp
    t = token_order_input(CASES["one_block"](), seed=1)
    dev = "cuda:0"
    up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)
    n_cl = int(t.seg_cluster_ptr[-1])
    pf = dp.Prefill(up(t.k_tokens, np.int16), up(t.v_tokens, np.int16), up(t.assignment, np.int32),
                    up(t.seg_row_base, np.int64), up(t.seg_rows, np.int32), up(t.seg_cluster_ptr, np.int32),
                    n_cl, n_cl, int(t.seg_rows.max()))
    need = dp.dp_build_workspace_bytes(pf)
    assert need > 0
    k = torch.empty((700, 128), dtype=torch.int16, device=dev)
    v, off, sz = torch.empty_like(k), torch.empty(n_cl, dtype=torch.int32, device=dev), torch.empty(n_cl, dtype=torch.int32, device=dev)
    kc, vc = torch.empty((n_cl, 128), dtype=torch.int16, device=dev), torch.empty((n_cl, 128), dtype=torch.int16, device=dev)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    with pytest.raises(dp.DPError) as e:
        dp.dp_build_cluster_cache(pf, k, v, off, sz, kc, vc, ws[: need // 2])
    assert e.value.status == -3
    pf.c.head_dim = 64
    with pytest.raises(dp.DPError) as e:
        dp.dp_build_cluster_cache(pf, k, v, off, sz, kc, vc, ws)
    assert e.value.status == -2
    pf.c.head_dim = 128
    pf.c.assignment = None
    with pytest.raises(dp.DPError) as e:
        dp.dp_build_cluster_cache(pf, k, v, off, sz, kc, vc, ws)
    assert e.value.status == -1
    pf.c.max_clusters_per_seg = n_cl + 5      # larger than the total
    assert dp.dp_build_workspace_bytes(pf) == 0
    torch.cuda.synchronize()


def test_build_full_size_cfg2():
    """cfg 2: 8 KV heads x 131072 tokens, 8192 clusters each; every output compared with the oracle's."""
    t = token_order_input(make_config(2), seed=11)
    got = gpu_build(t)
    print("[build cfg2] gpu done", flush=True)
    check_build(t, got, oracle.build_cluster_cache(t))
