"""The entry point that allocates nothing (dp_decode_attention_static: its workspace is a device array inside
the library) against dp_decode_attention with a caller-owned workspace, through the C ABI: same kernels, so the
outputs, the normalisers and the counts must be equal bit for bit.  Two calls in a row, the second on a smaller
input, so that what the first call left in the shared array is still there when the second runs."""
import numpy as np
import pytest

from workloads import make_cache, make_config

pytestmark = pytest.mark.gpu


def run_both(cache, p1, p2):
    import torch
    import paper_2602_05191_amd as dp
    dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc)
    nh = cache.batch * cache.n_q_heads
    assert dp.dp_workspace_bytes(pr) <= dp.DP_STATIC_SCRATCH_BYTES

    def buffers():
        out = torch.full((cache.batch, cache.n_q_heads, 128), float("nan"), dtype=torch.float32, device="cuda:0")
        lse = torch.full((nh,), float("nan"), dtype=torch.float32, device="cuda:0")
        cnt = [torch.full((nh,), -7, dtype=torch.int32, device="cuda:0") for _ in range(3)]
        return out, lse, cnt

    out_a, lse_a, cnt_a = buffers()
    ws = torch.zeros(dp.dp_workspace_bytes(pr), dtype=torch.uint8, device="cuda:0")
    dp.dp_decode_attention(pr, p1, p2, out_a, lse_a, ws, *cnt_a)
    out_b, lse_b, cnt_b = buffers()
    dp.dp_decode_attention_static(pr, p1, p2, out_b, lse_b, *cnt_b)
    torch.cuda.synchronize()
    assert torch.equal(out_a.view(torch.int32), out_b.view(torch.int32))
    assert torch.equal(lse_a.view(torch.int32), lse_b.view(torch.int32))
    for x, y in zip(cnt_a, cnt_b):
        assert torch.equal(x, y) and int(x.min()) >= 0
    return out_b.cpu().numpy(), [c.cpu().numpy() for c in cnt_b]


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    import oracle
    import harness as H
    # first call: flat and peaked heads, thousands of rows on the flat ones (split decode, partials in the scratch)
    big = make_cache(batch=2, n_kv_heads=2, n_q_heads=8, context=[30000, 9000], mean_cluster=16,
                     q_scale=lambda rng, b, h: 0.35 if h % 2 else 3.0, seed=61)
    out_big, cnt_big = run_both(big, 0.95, 0.9)
    assert cnt_big[2].max() > 2048
    # second call, smaller input, other shape: the array still holds the first call's lists, counters and partials
    small = make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=3000, mean_cluster=8, size_hi=32,
                       q_scale=lambda rng, b, h: [0.3, 2.0, 0.5, 4.0][h], seed=62)
    out_small, cnt_small = run_both(small, 0.9, 0.5)
    # and once more the first input: the results of the first call come back
    out_again, cnt_again = run_both(big, 0.95, 0.9)
    assert np.array_equal(out_big.view(np.uint32), out_again.view(np.uint32))
    # against the oracle as well (the stated bar), on the smaller input
    orc = oracle.Oracle(small)
    r = orc.decode_step(0.9, 0.5)
    assert np.abs(out_small - r.out).max() <= H.OUT_MAX_ABS
    assert cnt_small[1].tolist() == r.k1.ravel().tolist() and cnt_small[0].tolist() == r.k2.ravel().tolist()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    import paper_2602_05191_amd as dp
    c = make_config(0)
    dc = dp.DeviceCache.from_host(c)
    pr = dp.Problem(dc)
    pr.c.batch, pr.c.total_clusters = 64, 64 * int(c.seg_cluster_ptr[-1])     # only the host-known sizes grow
    pr.c.max_rows_per_seg = 1 << 22
    pr.nh = 64 * 4
    assert dp.dp_workspace_bytes(pr) > dp.DP_STATIC_SCRATCH_BYTES
    out = torch.empty((64, 4, 128), dtype=torch.float32, device="cuda:0")
    with pytest.raises(dp.DPError) as e:
        dp.dp_decode_attention_static(pr, 0.9, 0.5, out, None)
    assert e.value.status == -5
