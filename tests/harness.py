"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI
binding, run the fp64 oracle on the same inputs, and compare under the stated
bars.  (Not a test module.)"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

import oracle
from workloads import ClusteredCache

# bars -----------------------------------------------------------------------
OUT_MAX_ABS = 1e-2        # bf16 K/V, fp32 accumulation
OUT_REL_L2 = 5e-3
MASS_TOL = 1e-5           # a set may differ only where the cumulative mass is this close to the threshold
LOGIT_TIE_TOL = 1e-4      # ... and only by swapping clusters whose fp64 logits are this close


@dataclass
class GpuStep:
    out: np.ndarray            # [B, Hq, d] float32
    lse: np.ndarray            # [B, Hq]
    exact: List[np.ndarray]    # per head, ascending ids
    approx: List[np.ndarray]
    n_exact_tokens: np.ndarray
    logits: Optional[List[np.ndarray]] = None   # per head, fp32


def head_logit_slice(cache: ClusteredCache, b: int, h: int):
    G = cache.group
    seg = b * cache.n_kv_heads + h // G
    c0, c1 = int(cache.seg_cluster_ptr[seg]), int(cache.seg_cluster_ptr[seg + 1])
    kc = c1 - c0
    start = G * c0 + (h % G) * kc
    return start, kc


def gpu_logits(cache: ClusteredCache, sm_scale: float = 0.0):
    import torch
    import paper_2602_05191_amd as dp
    dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc, sm_scale=sm_scale)
    n = cache.group * int(cache.seg_cluster_ptr[-1])
    lg = torch.full((max(n, 1),), float("nan"), dtype=torch.float32, device="cuda:0")
    dp.dp_score_centroids(pr, lg)
    torch.cuda.synchronize()
    lg = lg.cpu().numpy()
    out = []
    for b in range(cache.batch):
        for h in range(cache.n_q_heads):
            s, kc = head_logit_slice(cache, b, h)
            out.append(lg[s:s + kc].copy())
    return out, lg


CANARY = 0xA5


class Guarded:
    """A device buffer with 256 bytes of canary on either side: `t` is the tensor handed to the library, check()
    asserts that nothing was written outside it."""

    def __init__(self, shape, dtype, fill):
        import torch
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        self.pad = 256
        self.n = n
        self.raw = torch.full((self.pad + (n + 255) // 256 * 256 + self.pad,), CANARY, dtype=torch.uint8, device="cuda:0")
        self.t = self.raw[self.pad: self.pad + n].view(dtype).reshape(shape)
        self.t.fill_(fill)

    def check(self, what):
        lo = self.raw[: self.pad].cpu().numpy()
        hi = self.raw[self.pad + self.n:].cpu().numpy()
        assert (lo == CANARY).all(), f"{what}: bytes in front of the buffer were overwritten"
        assert (hi == CANARY).all(), f"{what}: bytes behind the buffer were overwritten"


def gpu_select(cache: ClusteredCache, flat_logits: np.ndarray, p1: float, p2: float, flags: int = 0, budget=None):
    """budget = (k_retained, k_exact): dp_topk_select instead of dp_topp_select (p1, p2 unused);
    budget = "sorted": the sort-based A/B variant dp_topp_select_sorted."""
    import torch
    import paper_2602_05191_amd as dp
    dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc, flags=flags)
    nh, mk = cache.batch * cache.n_q_heads, max(cache.max_clusters_per_seg, 1)
    lg = torch.from_numpy(np.ascontiguousarray(flat_logits, dtype=np.float32)).cuda()
    g_sel = Guarded((nh, mk), torch.int32, -7)
    g_cnt = [Guarded((nh,), torch.int32, -7) for _ in range(3)]
    sel = g_sel.t
    ne, nr, nt = (g.t for g in g_cnt)
    if budget == "sorted":
        dp.dp_topp_select_sorted(pr, lg, p1, p2, sel, ne, nr, nt)
    elif budget is None:
        dp.dp_topp_select(pr, lg, p1, p2, sel, ne, nr, nt)
    else:
        dp.dp_topk_select(pr, lg, int(budget[0]), int(budget[1]), sel, ne, nr, nt)
    torch.cuda.synchronize()
    g_sel.check("sel_ids")
    for g in g_cnt:
        g.check("counts")
    sel, ne, nr, nt = sel.cpu().numpy(), ne.cpu().numpy(), nr.cpu().numpy(), nt.cpu().numpy()
    exact = [sel[i, :ne[i]].copy() for i in range(nh)]
    approx = [sel[i, ne[i]:nr[i]].copy() for i in range(nh)]
    return exact, approx, nt


def gpu_sparse_decode(cache: ClusteredCache, exact: List[np.ndarray], approx: List[np.ndarray], sm_scale: float = 0.0,
                      out_bf16: bool = False):
    import torch
    import paper_2602_05191_amd as dp
    dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc, sm_scale=sm_scale)
    nh, mk = cache.batch * cache.n_q_heads, max(cache.max_clusters_per_seg, 1)
    sel = np.full((nh, mk), -1, dtype=np.int32)
    ne = np.zeros(nh, dtype=np.int32)
    nr = np.zeros(nh, dtype=np.int32)
    for i in range(nh):
        ne[i], nr[i] = len(exact[i]), len(exact[i]) + len(approx[i])
        sel[i, :ne[i]] = exact[i]
        sel[i, ne[i]:nr[i]] = approx[i]
    g_ws = Guarded((max(dp.dp_workspace_bytes(pr), 256),), torch.uint8, 0)
    g_out = Guarded((cache.batch, cache.n_q_heads, cache.head_dim), torch.bfloat16 if out_bf16 else torch.float32,
                    float("nan"))
    g_lse = Guarded((nh,), torch.float32, float("nan"))
    ws, out, lse = g_ws.t, g_out.t, g_lse.t
    dp.dp_sparse_decode(pr, torch.from_numpy(sel).cuda(), torch.from_numpy(ne).cuda(), torch.from_numpy(nr).cuda(),
                        out, lse, ws)
    torch.cuda.synchronize()
    for g, what in ((g_ws, "workspace"), (g_out, "out"), (g_lse, "lse")):
        g.check(what)
    return out.float().cpu().numpy(), lse.cpu().numpy().reshape(cache.batch, cache.n_q_heads)


def gpu_decode_attention(cache: ClusteredCache, p1: float, p2: float, flags: int = 0, sm_scale: float = 0.0,
                         want_logits: bool = False, dc=None, budget=None, out_bf16: bool = False) -> GpuStep:
    """budget = (k_retained, k_exact): dp_budget_decode_attention instead of dp_decode_attention.
    out_bf16: ask the library for a bf16 output (returned widened to float32)."""
    import torch
    import paper_2602_05191_amd as dp
    if dc is None:
        dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc, sm_scale=sm_scale, flags=flags)
    nh, mk = cache.batch * cache.n_q_heads, max(cache.max_clusters_per_seg, 1)
    nbytes = dp.dp_workspace_bytes(pr)
    # every buffer the call writes sits between canaries: the workspace (exactly the size the library asks for),
    # the output, the normalisers and the three count vectors
    g_ws = Guarded((max(nbytes, 256),), torch.uint8, 0)
    g_out = Guarded((cache.batch, cache.n_q_heads, cache.head_dim), torch.bfloat16 if out_bf16 else torch.float32,
                    float("nan"))
    g_lse = Guarded((nh,), torch.float32, float("nan"))
    g_cnt = [Guarded((nh,), torch.int32, -7) for _ in range(3)]
    ws, out, lse = g_ws.t, g_out.t, g_lse.t
    ne, nr, nt = (g.t for g in g_cnt)
    if budget is None:
        dp.dp_decode_attention(pr, p1, p2, out, lse, ws, ne, nr, nt)
    else:
        dp.dp_budget_decode_attention(pr, int(budget[0]), int(budget[1]), out, lse, ws, ne, nr, nt)
    torch.cuda.synchronize()
    for g, what in [(g_ws, "workspace"), (g_out, "out"), (g_lse, "lse")] + [(g, "counts") for g in g_cnt]:
        g.check(what)
    lay = dp.dp_workspace_layout(pr)
    wsh = ws.cpu().numpy()
    sel = wsh[lay["sel_ids"]: lay["sel_ids"] + 4 * nh * mk].view(np.int32).reshape(nh, mk)
    ne, nr, nt = ne.cpu().numpy(), nr.cpu().numpy(), nt.cpu().numpy()
    logits = None
    if want_logits:
        n = cache.group * int(cache.seg_cluster_ptr[-1])
        flat = wsh[lay["logits"]: lay["logits"] + 4 * n].view(np.float32)
        logits = []
        for b in range(cache.batch):
            for h in range(cache.n_q_heads):
                s, kc = head_logit_slice(cache, b, h)
                logits.append(flat[s:s + kc].copy())
    return GpuStep(out=out.float().cpu().numpy(), lse=lse.cpu().numpy().reshape(cache.batch, cache.n_q_heads),
                   exact=[sel[i, :ne[i]].copy() for i in range(nh)],
                   approx=[sel[i, ne[i]:nr[i]].copy() for i in range(nh)], n_exact_tokens=nt, logits=logits)


def segment_rows(cache: ClusteredCache) -> np.ndarray:
    """Rows of each KV segment, or None when the clusters of some segment do not tile [0, rows)
    without gaps (then the segment's tokens are not one contiguous row range)."""
    n_seg = cache.batch * cache.n_kv_heads
    rows = np.zeros(n_seg, dtype=np.int32)
    for seg in range(n_seg):
        a, e = int(cache.seg_cluster_ptr[seg]), int(cache.seg_cluster_ptr[seg + 1])
        off, sz = cache.cluster_offsets[a:e].astype(np.int64), cache.cluster_sizes[a:e].astype(np.int64)
        order = np.argsort(off, kind="stable")
        if e > a and not (off[order][0] == 0 and (off[order][1:] == np.cumsum(sz[order])[:-1]).all()):
            return None
        rows[seg] = int(sz.sum())
    return rows


def gpu_dense_decode(cache: ClusteredCache, seg_rows: np.ndarray, sm_scale: float = 0.0, out_bf16: bool = False):
    import torch
    import paper_2602_05191_amd as dp
    dc = dp.DeviceCache.from_host(cache)
    pr = dp.Problem(dc, sm_scale=sm_scale)
    nh = cache.batch * cache.n_q_heads
    ws = torch.empty(max(dp.dp_workspace_bytes(pr), 256), dtype=torch.uint8, device="cuda:0")
    out = torch.full((cache.batch, cache.n_q_heads, cache.head_dim), float("nan"),
                     dtype=torch.bfloat16 if out_bf16 else torch.float32, device="cuda:0")
    lse = torch.full((nh,), float("nan"), dtype=torch.float32, device="cuda:0")
    dp.dp_dense_decode(pr, torch.from_numpy(np.ascontiguousarray(seg_rows, dtype=np.int32)).cuda(), out, lse, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), lse.cpu().numpy().reshape(cache.batch, cache.n_q_heads)


# ---------------------------------------------------------------------------
# comparison rules
# ---------------------------------------------------------------------------
def prefix_set_ok(got: np.ndarray, want: np.ndarray, a_hat: np.ndarray, logit: np.ndarray, tau: float):
    """`got`, `want`: sorted id arrays.  Returns (ok, exact_match).  A set that is not the oracle's is
    accepted only if its mass is within MASS_TOL of the threshold on both sides and it is a top set of the
    fp64 logits up to LOGIT_TIE_TOL."""
    if np.array_equal(got, want):
        return True, True
    if len(got) == 0:
        return bool(tau <= MASS_TOL), False
    mass = a_hat[got].sum()
    smallest = a_hat[got].min()
    inside = np.zeros(a_hat.size, dtype=bool)
    inside[got] = True
    nonempty = np.isfinite(logit)
    outside = nonempty & ~inside
    top_ok = (not outside.any()) or logit[got].min() >= logit[outside].max() - LOGIT_TIE_TOL
    ok = (mass >= tau - MASS_TOL) and (mass - smallest < tau + MASS_TOL) and top_ok
    return bool(ok), False


def judge_head_sets(where, got_exact, got_approx, cand_logit, pins, p1, p2, flags, orc):
    """One head's retained / exact sets against the oracle's selection on `cand_logit` (fp64 logits of the
    candidates: pinned and empty clusters at -inf).  Pinned clusters must all be exact; the rest is judged as a
    selection among the candidates, the second stage conditionally on the GPU's own retained set.  Raises on a
    difference beyond the near-threshold rule; returns True when both sets equal the oracle's."""
    assert (np.diff(got_exact) > 0).all() and (np.diff(got_approx) > 0).all(), f"{where}: ids not ascending"
    assert len(np.intersect1d(got_exact, got_approx)) == 0
    assert np.isin(pins, got_exact).all() and not np.isin(pins, got_approx).any(), f"{where}: pinned"
    s = orc.select(cand_logit, p1, p2, flags)
    got_ex = np.setdiff1d(got_exact, pins).astype(np.int64)
    got_ret = np.sort(np.concatenate([got_ex, got_approx])).astype(np.int64)
    if s.order.size == 0:
        assert got_ret.size == 0, f"{where}: selected {got_ret[:8]} although no cluster is a candidate"
        return True
    if p1 >= 1.0:
        ok1 = same1 = np.array_equal(got_ret, s.retained)
    else:
        ok1, same1 = prefix_set_ok(got_ret, s.retained.astype(np.int64), s.a_hat, cand_logit, p1)
    assert ok1, f"{where}: retained set differs beyond tolerance: gpu {got_ret[:16]} oracle {s.retained[:16]}"
    m1 = s.a_hat[got_ret].sum()
    if p2 >= 1.0:
        ok2 = same2 = np.array_equal(got_ex, got_ret)
    elif p2 <= 0.0:
        ok2 = same2 = got_ex.size == 0
    else:
        tau2 = min(p2, m1) if (flags & 1) else p2 * m1
        want = s.exact.astype(np.int64) if same1 else oracle_prefix(s, tau2)
        ok2, same2 = prefix_set_ok(got_ex, want, s.a_hat, cand_logit, tau2)
    assert ok2, f"{where}: exact set differs beyond tolerance: gpu {got_ex[:16]} oracle {s.exact[:16]}"
    return bool(same1 and same2)


def check_sets(cache: ClusteredCache, orc: "oracle.Oracle", g: GpuStep, p1: float, p2: float, flags: int = 0):
    """Compare the GPU's retained / exact sets with the oracle's for every head.  Returns the
    number of heads with a tolerated (near-threshold) difference; raises on a real mismatch."""
    tolerated = 0
    for b in range(cache.batch):
        for h in range(cache.n_q_heads):
            i = b * cache.n_q_heads + h
            pins = orc.pinned_clusters(b, h)
            logit = orc.candidate_logits(b, h)   # pinned logits are -inf here: the candidates alone
            full = orc.select(logit, p1, p2, flags, pinned=pins)
            assert np.array_equal(full.exact, np.sort(np.concatenate([pins, orc.select(logit, p1, p2, flags).exact])))
            same = judge_head_sets(f"head ({b},{h})", g.exact[i], g.approx[i], logit, pins, p1, p2, flags, orc)
            tolerated += int(not same)
            seg = b * cache.n_kv_heads + h // cache.group
            c0 = int(cache.seg_cluster_ptr[seg])
            assert int(g.n_exact_tokens[i]) == int(cache.cluster_sizes[c0 + np.asarray(g.exact[i], np.int64)].sum())
    return tolerated


def oracle_prefix(s: "oracle.Selection", tau: float) -> np.ndarray:
    k = int(np.searchsorted(s.cum, tau, side="left")) + 1
    return np.sort(s.order[: min(k, s.order.size)]).astype(np.int64)


def check_outputs(cache: ClusteredCache, orc: "oracle.Oracle", g: GpuStep, tight: Optional[float] = None):
    """GPU output vs the oracle evaluated on the GPU's own sets (identical to the oracle's step
    whenever the sets are identical).  Returns (max_abs, rel_l2)."""
    worst_abs, num, den = 0.0, 0.0, 0.0
    for b in range(cache.batch):
        for h in range(cache.n_q_heads):
            i = b * cache.n_q_heads + h
            ref, ref_lse = orc.mixed_attention(b, h, g.exact[i], g.approx[i])
            d = g.out[b, h].astype(np.float64) - ref
            worst_abs = max(worst_abs, float(np.abs(d).max()))
            num += float((d * d).sum())
            den += float((ref * ref).sum())
            if np.isfinite(ref_lse):
                assert abs(float(g.lse[b, h]) - ref_lse) <= 1e-3 + 1e-5 * abs(ref_lse), (b, h, g.lse[b, h], ref_lse)
            else:
                assert np.isneginf(g.lse[b, h])
    rel = (num / den) ** 0.5 if den > 0 else 0.0
    assert worst_abs <= OUT_MAX_ABS and rel <= OUT_REL_L2, (worst_abs, rel)
    if tight is not None:
        assert worst_abs <= tight, f"max-abs {worst_abs} above the expected fp32-accumulation level {tight}"
    return worst_abs, rel
