"""Seeded generator of clustered KV caches shaped like the paper's long-context
decode workloads (Llama-3-8B attention shape, 32k-128k tokens, GQA).

What it draws, per (batch, KV head) segment, each from its own numpy PCG64
stream ``SeedSequence([seed, tag, b, g])`` so that segments are reproducible
independently of generation order:

* cluster sizes (Poisson or Pareto, clamped, then nudged round-robin so that
  they sum to the context length), stored as int32 ``sizes`` with int32
  ``offsets`` = exclusive prefix sum (tokens are stored cluster-contiguous);
* keys  = 2*z_c + 0.5*eps  (z_c, eps ~ N(0, I)), values ~ N(0, I), rounded to
  bf16 (round-to-nearest-even);
* the per-cluster means of the *stored* (bf16) key and value rows, accumulated
  in fp64 and rounded to bf16: what the prefill stage would have written next
  to the cache (Eq. 2 of the paper and the k-means centroid of its Sec. 4.1);
* one query per query head: scale * (Dirichlet(1,1,1,1) mix of 4 distinct
  cluster centres of the head's own segment) + N(0, I), rounded to bf16.

bf16 tensors are carried as ``uint16`` bit patterns: numpy has no bf16 and both
consumers (the fp64 CPU oracle, the HIP library) want the raw stored bits.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

HEAD_DIM = 128


CLUSTER_PINNED = 1


# --------------------------------------------------------------------------
# bf16 storage format helpers (format conversion only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> float32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# container
# --------------------------------------------------------------------------
@dataclass
class ClusteredCache:
    """One decode step's inputs. Segment ``seg = b * n_kv_heads + g``."""

    batch: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    q: np.ndarray                # uint16 [batch, n_q_heads, d]           bf16 bits
    k_cache: np.ndarray          # uint16 [total_rows, d]                 bf16 bits
    v_cache: np.ndarray          # uint16 [total_rows, d]
    seg_row_base: np.ndarray     # int64  [n_seg]   first cache row of the segment
    seg_cluster_ptr: np.ndarray  # int32  [n_seg+1] CSR into the per-cluster arrays
    cluster_offsets: np.ndarray  # int32  [total_clusters] first row, relative to seg_row_base
    cluster_sizes: np.ndarray    # int32  [total_clusters]
    k_centroids: np.ndarray      # uint16 [total_clusters, d]
    v_centroids: np.ndarray      # uint16 [total_clusters, d]
    p1: float = 0.95
    p2: float = 0.9
    name: str = ""
    meta: Dict[str, object] = field(default_factory=dict)
    cluster_flags: Optional[np.ndarray] = None  # uint8 [total_clusters]; bit 0: pinned (sink / window tokens)

    @property
    def n_seg(self) -> int:
        return self.batch * self.n_kv_heads

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def max_clusters_per_seg(self) -> int:
        d = np.diff(self.seg_cluster_ptr)
        return int(d.max()) if d.size else 0

    @property
    def max_rows_per_seg(self) -> int:
        m = 0
        for s in range(self.n_seg):
            a, b = int(self.seg_cluster_ptr[s]), int(self.seg_cluster_ptr[s + 1])
            if b > a:
                m = max(m, int((self.cluster_offsets[a:b].astype(np.int64) + self.cluster_sizes[a:b]).max()))
        return m

    @property
    def context_tokens(self) -> int:
        """Sum over sequences of the context length (one KV head's rows)."""
        tot = 0
        for b in range(self.batch):
            s = b * self.n_kv_heads
            a, e = int(self.seg_cluster_ptr[s]), int(self.seg_cluster_ptr[s + 1])
            tot += int(self.cluster_sizes[a:e].sum())
        return tot


# --------------------------------------------------------------------------
# pieces
# --------------------------------------------------------------------------
def _fit_sizes_to_total(sizes: np.ndarray, total: int, lo: int, hi: int) -> np.ndarray:
    """Add or subtract 1 round-robin in cluster-index order, skipping clusters
    at a clamp bound, until the sizes sum to ``total``."""
    s = sizes.astype(np.int64).copy()
    n = s.size
    if not (n * lo <= total <= n * hi):
        raise ValueError(f"cannot fit {n} clusters in [{lo},{hi}] to total {total}")
    diff = int(total - s.sum())
    while diff != 0:
        step = 1 if diff > 0 else -1
        movable = np.nonzero(s < hi)[0] if step > 0 else np.nonzero(s > lo)[0]
        take = movable[: abs(diff)]
        s[take] += step
        diff -= step * take.size
    return s.astype(np.int32)


def draw_cluster_sizes(rng: np.random.Generator, n_clusters: int, total: int, dist: str,
                       mean: float, lo: int, hi: int) -> np.ndarray:
    if dist == "poisson":
        raw = rng.poisson(mean, size=n_clusters)
    elif dist == "pareto":
        # classical Pareto(alpha=1.5, x_m = mean/3): mean = alpha*x_m/(alpha-1) = mean
        alpha = 1.5
        raw = np.rint((mean / 3.0) * (1.0 + rng.pareto(alpha, size=n_clusters)))
    elif dist == "ones":
        raw = np.ones(n_clusters)
    else:
        raise ValueError(dist)
    raw = np.clip(raw, lo, hi).astype(np.int64)
    return _fit_sizes_to_total(raw, total, lo, hi)


def _cluster_means_bf16(rows_bits: np.ndarray, offsets: np.ndarray, sizes: np.ndarray) -> np.ndarray:
    """fp64 mean of the stored bf16 rows of each cluster, rounded to bf16."""
    x = bf16_bits_to_f32(rows_bits).astype(np.float64)
    n, d = sizes.size, rows_bits.shape[1]
    out = np.zeros((n, d), dtype=np.float64)
    nz = sizes > 0
    if nz.any():
        # reduceat over the starts of non-empty clusters (cluster-contiguous rows)
        starts = offsets[nz].astype(np.int64)
        order = np.argsort(starts, kind="stable")
        starts_sorted = starts[order]
        sums = np.add.reduceat(x, starts_sorted, axis=0)
        # reduceat sums up to the next start; valid because clusters tile the rows
        idx = np.nonzero(nz)[0][order]
        out[idx] = sums / sizes[idx][:, None]
    return f32_to_bf16_bits(out.astype(np.float32))


def make_segment(rng: np.random.Generator, n_tokens: int, n_clusters: int, size_dist: str,
                 size_mean: float, size_lo: int, size_hi: int, d: int = HEAD_DIM,
                 key_spread: float = 0.5, centre_scale: float = 2.0):
    """Draw one (batch, KV head) segment. Returns a dict of arrays plus the
    (unrounded) cluster centres used to aim queries."""
    sizes = draw_cluster_sizes(rng, n_clusters, n_tokens, size_dist, size_mean, size_lo, size_hi)
    offsets = np.zeros(n_clusters, dtype=np.int32)
    np.cumsum(sizes[:-1], out=offsets[1:])
    centres = (centre_scale * rng.standard_normal((n_clusters, d), dtype=np.float32))
    owner = np.repeat(np.arange(n_clusters, dtype=np.int64), sizes)
    keys = centres[owner]
    keys += np.float32(key_spread) * rng.standard_normal((n_tokens, d), dtype=np.float32)
    k_bits = f32_to_bf16_bits(keys)
    del keys
    v_bits = f32_to_bf16_bits(rng.standard_normal((n_tokens, d), dtype=np.float32))
    kc_bits = _cluster_means_bf16(k_bits, offsets, sizes)
    vc_bits = _cluster_means_bf16(v_bits, offsets, sizes)
    return dict(sizes=sizes, offsets=offsets, centres=centres, k=k_bits, v=v_bits, kc=kc_bits, vc=vc_bits)


def draw_query(rng: np.random.Generator, centres: np.ndarray, scale: float, n_mix: int = 4) -> np.ndarray:
    n = centres.shape[0]
    m = min(n_mix, n)
    picks = rng.choice(n, size=m, replace=False)
    a = rng.dirichlet(np.ones(m))
    q = scale * (a[:, None] * centres[picks].astype(np.float64)).sum(axis=0)
    q = q + rng.standard_normal(centres.shape[1])
    return f32_to_bf16_bits(q.astype(np.float32))


# --------------------------------------------------------------------------
# whole caches
# --------------------------------------------------------------------------
def make_cache(*, batch: int, n_kv_heads: int, n_q_heads: int, context: Sequence[int] | int,
               mean_cluster: int = 16, size_dist: str = "poisson", size_lo: int = 1, size_hi: int = 64,
               q_scale=3.0, p1: float = 0.95, p2: float = 0.9, seed: int = 0, tag: int = 0,
               d: int = HEAD_DIM, name: str = "", n_clusters: Optional[Sequence[int] | int] = None,
               key_spread: float = 0.5) -> ClusteredCache:
    """Build a cache. ``context`` is one length or one per sequence; ``q_scale``
    is a number, a per-query-head sequence, or a callable
    ``(rng, b, h) -> scale``. ``n_clusters`` overrides context/mean_cluster."""
    if n_q_heads % n_kv_heads:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    G = n_q_heads // n_kv_heads
    ctx = [int(context)] * batch if np.isscalar(context) else [int(c) for c in context]
    if len(ctx) != batch:
        raise ValueError("one context length per sequence")
    if n_clusters is None:
        ncl = [max(1, c // mean_cluster) for c in ctx]
    else:
        ncl = [int(n_clusters)] * batch if np.isscalar(n_clusters) else [int(c) for c in n_clusters]

    n_seg = batch * n_kv_heads
    tot_rows = sum(ctx) * n_kv_heads
    tot_cl = sum(ncl) * n_kv_heads
    k_cache = np.empty((tot_rows, d), dtype=np.uint16)
    v_cache = np.empty((tot_rows, d), dtype=np.uint16)
    kc = np.empty((tot_cl, d), dtype=np.uint16)
    vc = np.empty((tot_cl, d), dtype=np.uint16)
    offsets = np.empty(tot_cl, dtype=np.int32)
    sizes = np.empty(tot_cl, dtype=np.int32)
    seg_row_base = np.zeros(n_seg, dtype=np.int64)
    seg_cluster_ptr = np.zeros(n_seg + 1, dtype=np.int32)
    q = np.empty((batch, n_q_heads, d), dtype=np.uint16)
    scales = np.empty((batch, n_q_heads), dtype=np.float64)

    # every segment has its own random stream, so segments can be drawn by a thread pool
    # (numpy releases the GIL while it draws) without changing a single value
    row_of, cl_of = [], []
    row, cl = 0, 0
    for b in range(batch):
        for g in range(n_kv_heads):
            row_of.append(row)
            cl_of.append(cl)
            row += ctx[b]
            cl += ncl[b]

    def draw(seg):
        b, g = divmod(seg, n_kv_heads)
        rng = np.random.default_rng(np.random.SeedSequence([seed, tag, b, g]))
        s = make_segment(rng, ctx[b], ncl[b], size_dist, float(mean_cluster), size_lo, size_hi, d,
                         key_spread=key_spread)
        n, k, r0, c0 = ctx[b], ncl[b], row_of[seg], cl_of[seg]
        seg_row_base[seg] = r0
        seg_cluster_ptr[seg] = c0
        k_cache[r0:r0 + n] = s["k"]
        v_cache[r0:r0 + n] = s["v"]
        kc[c0:c0 + k] = s["kc"]
        vc[c0:c0 + k] = s["vc"]
        offsets[c0:c0 + k] = s["offsets"]
        sizes[c0:c0 + k] = s["sizes"]
        for j in range(G):
            h = g * G + j
            if callable(q_scale):
                sc = float(q_scale(rng, b, h))
            elif np.isscalar(q_scale):
                sc = float(q_scale)
            else:
                sc = float(q_scale[h])
            scales[b, h] = sc
            q[b, h] = draw_query(rng, s["centres"], sc)

    workers = min(n_seg, max(1, min(16, os.cpu_count() or 1)))
    if workers > 1 and tot_rows >= (1 << 18):
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(draw, range(n_seg)))
    else:
        for seg in range(n_seg):
            draw(seg)
    seg_cluster_ptr[n_seg] = cl
    return ClusteredCache(batch=batch, n_kv_heads=n_kv_heads, n_q_heads=n_q_heads, head_dim=d, q=q,
                          k_cache=k_cache, v_cache=v_cache, seg_row_base=seg_row_base,
                          seg_cluster_ptr=seg_cluster_ptr, cluster_offsets=offsets, cluster_sizes=sizes,
                          k_centroids=kc, v_centroids=vc, p1=p1, p2=p2, name=name,
                          meta=dict(context=ctx, n_clusters=ncl, q_scale=scales, seed=seed, tag=tag))


# The five workload shapes of this build. cfg0 is the small case an fp64 CPU
# oracle finishes in well under a second; cfg1/cfg2 are the Llama-3-8B
# attention shape at 32k and 128k tokens.
CONFIGS: List[str] = ["cfg0_tiny", "cfg1_8b_32k", "cfg2_8b_128k", "cfg3_batch16", "cfg4_gqa8_128k"]


def make_config(idx: int, *, seed: Optional[int] = None, shrink: int = 1,
                heads: Optional[str] = None) -> ClusteredCache:
    """Workload ``idx`` (0..4). ``shrink`` divides every context length (kept a
    multiple of the mean cluster size) to get a same-shaped but smaller case.
    ``heads`` (workloads 1 and 2 only) replaces the query scales: "flat" makes every
    head flat (scale 0.4: hundreds of clusters retained), "mixed" one head in eight."""
    if seed is None:
        seed = idx  # cfg0 uses seed 0
    if heads is not None:
        if idx not in (1, 2) or heads not in ("flat", "mixed"):
            raise ValueError("heads: 'flat' or 'mixed', for workloads 1 and 2")
        scale = 0.4 if heads == "flat" else (lambda rng, b, h: 0.4 if h % 8 == 0 else 3.0)
        return make_cache(batch=1, n_kv_heads=8, n_q_heads=32, context=(32768 if idx == 1 else 131072) // shrink,
                          mean_cluster=16, size_lo=1, size_hi=64, q_scale=scale, p1=0.95, p2=0.9, seed=seed,
                          tag=10 + idx, name=f"{CONFIGS[idx]}_{heads}_heads")
    if idx == 0:
        return make_cache(batch=1, n_kv_heads=1, n_q_heads=4, context=4096 // shrink, mean_cluster=16,
                          size_lo=1, size_hi=64, q_scale=3.0, p1=0.95, p2=0.9, seed=seed, tag=0,
                          name=CONFIGS[0])
    if idx == 1:
        return make_cache(batch=1, n_kv_heads=8, n_q_heads=32, context=32768 // shrink, mean_cluster=16,
                          size_lo=1, size_hi=64, q_scale=3.0, p1=0.95, p2=0.9, seed=seed, tag=1,
                          name=CONFIGS[1])
    if idx == 2:
        return make_cache(batch=1, n_kv_heads=8, n_q_heads=32, context=131072 // shrink, mean_cluster=16,
                          size_lo=1, size_hi=64, q_scale=lambda rng, b, h: rng.uniform(1.0, 5.0),
                          p1=0.95, p2=0.9, seed=seed, tag=2, name=CONFIGS[2])
    if idx == 3:
        lrng = np.random.default_rng(np.random.SeedSequence([seed, 3, 0xC0]))
        ctx = (lrng.integers(16384, 65536, size=16, endpoint=True) // shrink // 32) * 32
        return make_cache(batch=16, n_kv_heads=8, n_q_heads=32, context=[int(c) for c in ctx],
                          mean_cluster=32, size_lo=1, size_hi=128, q_scale=3.0, p1=0.98, p2=0.95,
                          seed=seed, tag=3, name=CONFIGS[3])
    if idx == 4:
        return make_cache(batch=4, n_kv_heads=8, n_q_heads=64, context=131072 // shrink, mean_cluster=16,
                          size_dist="pareto", size_lo=1, size_hi=512,
                          q_scale=lambda rng, b, h: 0.5 if h % 2 == 0 else 5.0,
                          p1=0.95, p2=0.9, seed=seed, tag=4, name=CONFIGS[4])
    raise ValueError(f"no config {idx}")


def pin_sink_and_window(cache: ClusteredCache, first: int = 1, last: int = 4) -> ClusteredCache:
    """Flag the first ``first`` and the last ``last`` clusters of every segment as pinned, in place:
    the stand-in for a cache that keeps its attention-sink tokens and its most recent tokens in
    clusters of their own (4 + 64 tokens in the paper's runs; here whatever sizes those clusters
    drew, about 16 tokens each).  Returns the cache."""
    flags = np.zeros(int(cache.seg_cluster_ptr[-1]), dtype=np.uint8)
    for seg in range(cache.n_seg):
        a, e = int(cache.seg_cluster_ptr[seg]), int(cache.seg_cluster_ptr[seg + 1])
        flags[a:min(e, a + first)] |= CLUSTER_PINNED
        flags[max(a, e - last):e] |= CLUSTER_PINNED
    cache.cluster_flags = flags
    return cache


@dataclass
class TokenOrderInput:
    """What the prefill stage hands to the metadata build: K / V in token order and a cluster id per token."""
    n_seg: int
    head_dim: int
    k_tokens: np.ndarray         # uint16 [total_rows, d]
    v_tokens: np.ndarray         # uint16 [total_rows, d]
    assignment: np.ndarray       # int32  [total_rows]  segment-local cluster id of each token
    seg_row_base: np.ndarray     # int64  [n_seg]
    seg_rows: np.ndarray         # int32  [n_seg]
    seg_cluster_ptr: np.ndarray  # int32  [n_seg+1]


def token_order_input(cache: ClusteredCache, seed: int = 0) -> TokenOrderInput:
    """Undo the cluster-contiguous layout of a generated cache: the rows of every segment are put into a
    seeded random "token order" and each token remembers the cluster it came from.  (The clusters of the
    cache must tile their segment without gaps.)"""
    k_tok, v_tok = np.empty_like(cache.k_cache), np.empty_like(cache.v_cache)
    asg = np.empty(cache.k_cache.shape[0], dtype=np.int32)
    rows = np.zeros(cache.n_seg, dtype=np.int32)
    for seg in range(cache.n_seg):
        a, e = int(cache.seg_cluster_ptr[seg]), int(cache.seg_cluster_ptr[seg + 1])
        n, r0 = int(cache.cluster_sizes[a:e].sum()), int(cache.seg_row_base[seg])
        cluster_of_row = np.repeat(np.arange(e - a, dtype=np.int32), cache.cluster_sizes[a:e])
        row_of = np.empty(n, dtype=np.int64)   # rows listed cluster by cluster, at their actual offsets
        pos = 0
        for i in range(a, e):
            s = int(cache.cluster_sizes[i])
            row_of[pos:pos + s] = int(cache.cluster_offsets[i]) + np.arange(s)
            pos += s
        perm = np.random.default_rng(np.random.SeedSequence([seed, 77, seg])).permutation(n)
        k_tok[r0:r0 + n] = cache.k_cache[r0 + row_of[perm]]
        v_tok[r0:r0 + n] = cache.v_cache[r0 + row_of[perm]]
        asg[r0:r0 + n] = cluster_of_row[perm]
        rows[seg] = n
    return TokenOrderInput(n_seg=cache.n_seg, head_dim=cache.head_dim, k_tokens=k_tok, v_tokens=v_tok,
                           assignment=asg, seg_row_base=cache.seg_row_base.copy(), seg_rows=rows,
                           seg_cluster_ptr=cache.seg_cluster_ptr.copy())
