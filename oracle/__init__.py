"""fp64 CPU oracle of the Double-P decode step (TEST INFRASTRUCTURE ONLY).

``dp_oracle.c`` holds the arithmetic (plain C, IEEE double, scalar loops, one
function per equation of the paper); this module is a ctypes wrapper that hands
it numpy arrays.  Nothing under ``oracle/`` is imported by the HIP package; the
only users are ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py``.

Stored bf16 tensors are passed as uint16 bit patterns and widened exactly
inside the C code.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dp_oracle.c")
_LIB = os.path.join(_HERE, "libdp_oracle.so")

P2_ABSOLUTE = 1


def build(force: bool = False) -> str:
    """Compile dp_oracle.c with gcc (-O2, OpenMP) into oracle/libdp_oracle.so."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "dp_oracle.h")))
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Cache(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_kv_heads", C.c_int32), ("n_q_heads", C.c_int32), ("head_dim", C.c_int32),
                ("q", C.c_void_p), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
                ("seg_row_base", C.c_void_p), ("seg_cluster_ptr", C.c_void_p),
                ("cluster_offsets", C.c_void_p), ("cluster_sizes", C.c_void_p),
                ("k_centroids", C.c_void_p), ("v_centroids", C.c_void_p), ("sm_scale", C.c_double),
                ("cluster_flags", C.c_void_p)]


_lib = None


def build_sanitized(out_path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (-O1), for the CPU test that runs the
    pins through it (host code only; the GPU never sees this build)."""
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-omit-frame-pointer",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-Wall", "-Wextra",
                           "-o", out_path, _SRC, "-lm"])
    return out_path


def _load():
    global _lib
    if _lib is None:
        # DP_ORACLE_LIB: a build of dp_oracle.c to load instead (the sanitized one of tests/test_oracle_sanitized.py)
        path = os.environ.get("DP_ORACLE_LIB") or build()
        L = C.CDLL(path)
        P, I, D, U = C.c_void_p, C.c_int32, C.c_double, C.c_uint32
        CP = C.POINTER(_Cache)
        L.dpo_num_clusters.restype = I
        L.dpo_num_clusters.argtypes = [CP, I, I]
        L.dpo_centroid_logits.restype = None
        L.dpo_centroid_logits.argtypes = [CP, I, I, P]
        L.dpo_candidate_logits.restype = None
        L.dpo_candidate_logits.argtypes = [CP, I, I, P]
        L.dpo_pinned_clusters.restype = I
        L.dpo_pinned_clusters.argtypes = [CP, I, I, P]
        L.dpo_cluster_distribution.restype = None
        L.dpo_cluster_distribution.argtypes = [P, I, P]
        L.dpo_sorted_order.restype = I
        L.dpo_sorted_order.argtypes = [P, I, P]
        L.dpo_double_top_p.restype = None
        L.dpo_double_top_p.argtypes = [P, P, I, D, D, U, P, P, P, P]
        L.dpo_mixed_attention.restype = None
        L.dpo_mixed_attention.argtypes = [CP, I, I, P, I, P, I, P, P]
        L.dpo_dense_attention.restype = None
        L.dpo_dense_attention.argtypes = [CP, I, I, P, P]
        L.dpo_exact_cluster_log_mass.restype = None
        L.dpo_exact_cluster_log_mass.argtypes = [CP, I, I, P]
        L.dpo_decode_step.restype = I
        L.dpo_decode_step.argtypes = [CP, D, D, U, P, P, P, P, P, C.c_int64, I]
        L.dpo_fixed_budget.restype = None
        L.dpo_fixed_budget.argtypes = [I, I, I, P, P]
        L.dpo_budget_step.restype = I
        L.dpo_budget_step.argtypes = [CP, I, I, P, P, P, P, P, C.c_int64, I]
        L.dpo_build_cluster_cache.restype = None
        L.dpo_build_cluster_cache.argtypes = [I, I] + [P] * 14
        L.dpo_kmeans_assign.restype = None
        L.dpo_kmeans_assign.argtypes = [I, I] + [P] * 8
        L.dpo_dense_step.restype = I
        L.dpo_dense_step.argtypes = [CP, P, P, I]
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


class Oracle:
    """Binds one set of inputs (any object with the ClusteredCache fields)."""

    def __init__(self, cache, sm_scale: float = 0.0):
        self.lib = _load()
        self.batch, self.n_kv_heads = int(cache.batch), int(cache.n_kv_heads)
        self.n_q_heads, self.d = int(cache.n_q_heads), int(cache.head_dim)
        # keep contiguous, correctly typed copies alive for the C side
        self._a = dict(
            q=np.ascontiguousarray(cache.q, dtype=np.uint16),
            k_cache=np.ascontiguousarray(cache.k_cache, dtype=np.uint16),
            v_cache=np.ascontiguousarray(cache.v_cache, dtype=np.uint16),
            seg_row_base=np.ascontiguousarray(cache.seg_row_base, dtype=np.int64),
            seg_cluster_ptr=np.ascontiguousarray(cache.seg_cluster_ptr, dtype=np.int32),
            cluster_offsets=np.ascontiguousarray(cache.cluster_offsets, dtype=np.int32),
            cluster_sizes=np.ascontiguousarray(cache.cluster_sizes, dtype=np.int32),
            k_centroids=np.ascontiguousarray(cache.k_centroids, dtype=np.uint16),
            v_centroids=np.ascontiguousarray(cache.v_centroids, dtype=np.uint16),
        )
        flags = getattr(cache, "cluster_flags", None)
        if flags is not None:
            self._a["cluster_flags"] = np.ascontiguousarray(flags, dtype=np.uint8)
        a = self._a
        self.c = _Cache(self.batch, self.n_kv_heads, self.n_q_heads, self.d, _ptr(a["q"]), _ptr(a["k_cache"]),
                        _ptr(a["v_cache"]), _ptr(a["seg_row_base"]), _ptr(a["seg_cluster_ptr"]),
                        _ptr(a["cluster_offsets"]), _ptr(a["cluster_sizes"]), _ptr(a["k_centroids"]),
                        _ptr(a["v_centroids"]), float(sm_scale),
                        _ptr(a["cluster_flags"]) if flags is not None else None)
        self.cp = C.byref(self.c)

    # ---- per-head stages -------------------------------------------------
    def num_clusters(self, b: int, h: int) -> int:
        return int(self.lib.dpo_num_clusters(self.cp, b, h))

    def centroid_logits(self, b: int, h: int) -> np.ndarray:
        out = np.empty(max(1, self.num_clusters(b, h)), dtype=np.float64)
        self.lib.dpo_centroid_logits(self.cp, b, h, _ptr(out))
        return out[: self.num_clusters(b, h)]

    def candidate_logits(self, b: int, h: int) -> np.ndarray:
        """centroid_logits with the pinned clusters at -inf: what the selection runs on."""
        out = np.empty(max(1, self.num_clusters(b, h)), dtype=np.float64)
        self.lib.dpo_candidate_logits(self.cp, b, h, _ptr(out))
        return out[: self.num_clusters(b, h)]

    def pinned_clusters(self, b: int, h: int) -> np.ndarray:
        out = np.empty(max(1, self.num_clusters(b, h)), dtype=np.int32)
        n = self.lib.dpo_pinned_clusters(self.cp, b, h, _ptr(out))
        return out[:n].copy()

    def cluster_distribution(self, logit: np.ndarray) -> np.ndarray:
        logit = np.ascontiguousarray(logit, dtype=np.float64)
        out = np.empty(max(1, logit.size), dtype=np.float64)
        self.lib.dpo_cluster_distribution(_ptr(logit), logit.size, _ptr(out))
        return out[: logit.size]

    def sorted_order(self, logit: np.ndarray) -> np.ndarray:
        logit = np.ascontiguousarray(logit, dtype=np.float64)
        out = np.empty(max(1, logit.size), dtype=np.int32)
        n = self.lib.dpo_sorted_order(_ptr(logit), logit.size, _ptr(out))
        return out[:n]

    def double_top_p(self, a_hat: np.ndarray, order: np.ndarray, p1: float, p2: float, flags: int = 0):
        """-> (k1, k2, m1, cum)"""
        a_hat = np.ascontiguousarray(a_hat, dtype=np.float64)
        order = np.ascontiguousarray(order, dtype=np.int32)
        cum = np.empty(max(1, order.size), dtype=np.float64)
        k1, k2, m1 = C.c_int32(), C.c_int32(), C.c_double()
        self.lib.dpo_double_top_p(_ptr(a_hat), _ptr(order), order.size, float(p1), float(p2), int(flags), _ptr(cum),
                                  C.addressof(k1), C.addressof(k2), C.addressof(m1))
        return k1.value, k2.value, m1.value, cum[: order.size]

    @staticmethod
    def _candidates(logit: np.ndarray, pinned) -> np.ndarray:
        logit = np.array(logit, dtype=np.float64)
        if pinned is not None and len(pinned):
            logit[np.asarray(pinned, dtype=np.int64)] = -np.inf
        return logit

    def select(self, logit: np.ndarray, p1: float, p2: float, flags: int = 0, pinned=None) -> "Selection":
        """Stage 2 from given logits (any float dtype; widened to double).  pinned: ids of the non-empty
        pinned clusters of the head (pinned_clusters): out of the distribution, always exact."""
        logit = self._candidates(logit, pinned)
        a_hat = self.cluster_distribution(logit)
        order = self.sorted_order(logit)
        k1, k2, m1, cum = self.double_top_p(a_hat, order, p1, p2, flags)
        return Selection(order=order, k1=k1, k2=k2, m1=m1, cum=cum, a_hat=a_hat,
                         pinned=np.asarray(pinned if pinned is not None else [], dtype=np.int32))

    def fixed_budget(self, logit: np.ndarray, k_retained: int, k_exact: int, pinned=None) -> "Selection":
        """Fixed-budget selection from given logits (Sec. 5.1, cluster-based baseline)."""
        logit = self._candidates(logit, pinned)
        a_hat = self.cluster_distribution(logit)
        order = self.sorted_order(logit)
        k1, k2 = C.c_int32(), C.c_int32()
        self.lib.dpo_fixed_budget(order.size, int(k_retained), int(k_exact), C.addressof(k1), C.addressof(k2))
        cum = np.cumsum(a_hat[order]) if order.size else np.zeros(0)
        m1 = float(cum[k1.value - 1]) if k1.value > 0 else 0.0
        return Selection(order=order, k1=k1.value, k2=k2.value, m1=m1, cum=cum, a_hat=a_hat,
                         pinned=np.asarray(pinned if pinned is not None else [], dtype=np.int32))

    def mixed_attention(self, b: int, h: int, exact_ids: Sequence[int], approx_ids: Sequence[int]):
        ex = np.ascontiguousarray(exact_ids, dtype=np.int32)
        ap = np.ascontiguousarray(approx_ids, dtype=np.int32)
        ex_p = np.concatenate([ex, np.zeros(1, np.int32)])  # non-null pointers for empty sets
        ap_p = np.concatenate([ap, np.zeros(1, np.int32)])
        out = np.empty(self.d, dtype=np.float64)
        lse = C.c_double()
        self.lib.dpo_mixed_attention(self.cp, b, h, _ptr(ex_p), ex.size, _ptr(ap_p), ap.size, _ptr(out),
                                     C.addressof(lse))
        return out, lse.value

    def dense_attention(self, b: int, h: int):
        out = np.empty(self.d, dtype=np.float64)
        lse = C.c_double()
        self.lib.dpo_dense_attention(self.cp, b, h, _ptr(out), C.addressof(lse))
        return out, lse.value

    def exact_cluster_log_mass(self, b: int, h: int) -> np.ndarray:
        out = np.empty(max(1, self.num_clusters(b, h)), dtype=np.float64)
        self.lib.dpo_exact_cluster_log_mass(self.cp, b, h, _ptr(out))
        return out[: self.num_clusters(b, h)]

    # ---- whole step ------------------------------------------------------
    def decode_step(self, p1: float, p2: float, flags: int = 0, n_threads: int = 1, want_order: bool = True):
        nh = self.batch * self.n_q_heads
        out = np.empty((self.batch, self.n_q_heads, self.d), dtype=np.float64)
        lse = np.empty(nh, dtype=np.float64)
        k1 = np.empty(nh, dtype=np.int32)
        k2 = np.empty(nh, dtype=np.int32)
        stride = int(np.diff(self._a["seg_cluster_ptr"]).max()) if nh else 0
        order = np.full((nh, max(1, stride)), -1, dtype=np.int32) if want_order else None
        used = self.lib.dpo_decode_step(self.cp, float(p1), float(p2), int(flags), _ptr(out), _ptr(lse), _ptr(k1),
                                        _ptr(k2), _ptr(order) if want_order else None, max(1, stride),
                                        int(n_threads))
        return StepResult(out=out, lse=lse.reshape(self.batch, self.n_q_heads),
                          k1=k1.reshape(self.batch, self.n_q_heads), k2=k2.reshape(self.batch, self.n_q_heads),
                          order=order, threads=int(used))

    def budget_step(self, k_retained: int, k_exact: int, n_threads: int = 1, want_order: bool = True):
        nh = self.batch * self.n_q_heads
        out = np.empty((self.batch, self.n_q_heads, self.d), dtype=np.float64)
        lse = np.empty(nh, dtype=np.float64)
        k1 = np.empty(nh, dtype=np.int32)
        k2 = np.empty(nh, dtype=np.int32)
        stride = int(np.diff(self._a["seg_cluster_ptr"]).max()) if nh else 0
        order = np.full((nh, max(1, stride)), -1, dtype=np.int32) if want_order else None
        used = self.lib.dpo_budget_step(self.cp, int(k_retained), int(k_exact), _ptr(out), _ptr(lse), _ptr(k1),
                                        _ptr(k2), _ptr(order) if want_order else None, max(1, stride),
                                        int(n_threads))
        return StepResult(out=out, lse=lse.reshape(self.batch, self.n_q_heads),
                          k1=k1.reshape(self.batch, self.n_q_heads), k2=k2.reshape(self.batch, self.n_q_heads),
                          order=order, threads=int(used))

    # ---- selection per GQA group (a reading the paper leaves open: it states the method for one query,
    # its model shares a KV head among 4 query heads, Sec. 5.1) ----------------------------------
    def group_union_sets(self, b: int, g: int, p1: float, p2: float, flags: int = 0):
        """Union of the per-head sets of KV head g of sequence b: (exact ids, approximated ids), ascending.
        exact = union of the heads' exact sets; approximated = union of their retained sets minus that."""
        G = self.n_q_heads // self.n_kv_heads
        exact, retained = set(), set()
        for h in range(g * G, (g + 1) * G):
            sel = self.select(self.centroid_logits(b, h), p1, p2, flags, pinned=self.pinned_clusters(b, h))
            exact.update(int(i) for i in sel.exact)
            retained.update(int(i) for i in sel.retained)
        return np.array(sorted(exact), dtype=np.int32), np.array(sorted(retained - exact), dtype=np.int32)

    def group_union_step(self, p1: float, p2: float, flags: int = 0):
        """Every head attends (Eq. 8, Eq. 9) over the union sets of its group.
        -> out [batch, n_q_heads, d], lse [batch, n_q_heads], {(b, g): (exact ids, approximated ids)}"""
        G = self.n_q_heads // self.n_kv_heads
        out = np.zeros((self.batch, self.n_q_heads, self.d), dtype=np.float64)
        lse = np.full((self.batch, self.n_q_heads), -np.inf, dtype=np.float64)
        sets = {}
        for b in range(self.batch):
            for g in range(self.n_kv_heads):
                ex, ap = self.group_union_sets(b, g, p1, p2, flags)
                sets[(b, g)] = (ex, ap)
                for h in range(g * G, (g + 1) * G):
                    if ex.size + ap.size:
                        out[b, h], lse[b, h] = self.mixed_attention(b, h, ex, ap)
        return out, lse, sets

    def dense_step(self, n_threads: int = 1):
        nh = self.batch * self.n_q_heads
        out = np.empty((self.batch, self.n_q_heads, self.d), dtype=np.float64)
        lse = np.empty(nh, dtype=np.float64)
        used = self.lib.dpo_dense_step(self.cp, _ptr(out), _ptr(lse), int(n_threads))
        return out, lse.reshape(self.batch, self.n_q_heads), int(used)


@dataclass
class Selection:
    order: np.ndarray   # non-empty clusters, score descending, index ascending among equals
    k1: int             # order[:k1] retained by the first top-p
    k2: int             # order[:k2] exact, order[k2:k1] approximated
    m1: float           # mass of the retained set under A_hat
    cum: np.ndarray     # cum[k] = mass of order[:k+1]
    a_hat: np.ndarray   # Eq. 6 distribution, by cluster index
    pinned: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))  # always exact, outside the order

    @property
    def exact(self) -> np.ndarray:
        return np.sort(np.concatenate([self.pinned, self.order[: self.k2]]).astype(np.int32))

    @property
    def approx(self) -> np.ndarray:
        return np.sort(self.order[self.k2: self.k1])

    @property
    def retained(self) -> np.ndarray:
        return np.sort(np.concatenate([self.pinned, self.order[: self.k1]]).astype(np.int32))


@dataclass
class StepResult:
    out: np.ndarray
    lse: np.ndarray
    k1: np.ndarray
    k2: np.ndarray
    order: Optional[np.ndarray]
    threads: int


def build_cluster_cache(tokens) -> dict:
    """Prefill side (Sec. 4.1, Eq. 2) for a workloads.TokenOrderInput: the cluster-contiguous cache and
    the cluster metadata, as numpy arrays keyed like the ClusteredCache fields (+ v_sums, token_row)."""
    lib = _load()
    t = tokens
    d = int(t.head_dim)
    n_rows, n_cl = int(t.k_tokens.shape[0]), int(t.seg_cluster_ptr[-1])
    a = dict(k=np.ascontiguousarray(t.k_tokens, np.uint16), v=np.ascontiguousarray(t.v_tokens, np.uint16),
             asg=np.ascontiguousarray(t.assignment, np.int32), base=np.ascontiguousarray(t.seg_row_base, np.int64),
             rows=np.ascontiguousarray(t.seg_rows, np.int32), ptr=np.ascontiguousarray(t.seg_cluster_ptr, np.int32))
    out = dict(k_cache=np.zeros((n_rows, d), np.uint16), v_cache=np.zeros((n_rows, d), np.uint16),
               cluster_offsets=np.zeros(max(n_cl, 1), np.int32), cluster_sizes=np.zeros(max(n_cl, 1), np.int32),
               k_centroids=np.zeros((max(n_cl, 1), d), np.uint16), v_centroids=np.zeros((max(n_cl, 1), d), np.uint16),
               v_sums=np.zeros((max(n_cl, 1), d), np.float64), token_row=np.zeros(max(n_rows, 1), np.int32))
    lib.dpo_build_cluster_cache(len(a["rows"]), d, _ptr(a["k"]), _ptr(a["v"]), _ptr(a["asg"]), _ptr(a["base"]),
                                _ptr(a["rows"]), _ptr(a["ptr"]), _ptr(out["k_cache"]), _ptr(out["v_cache"]),
                                _ptr(out["cluster_offsets"]), _ptr(out["cluster_sizes"]), _ptr(out["k_centroids"]),
                                _ptr(out["v_centroids"]), _ptr(out["v_sums"]), _ptr(out["token_row"]))
    for k in ("cluster_offsets", "cluster_sizes", "k_centroids", "v_centroids", "v_sums"):
        out[k] = out[k][:n_cl]
    out["token_row"] = out["token_row"][:n_rows]
    return out


def kmeans_assign(tokens, centroids: np.ndarray):
    """Nearest centroid of every token of a workloads.TokenOrderInput (Sec. 4.1, the assignment step of k-means).
    centroids: uint16 bf16 bits [total_clusters, d].  -> (assignment int32, best score, runner-up score)"""
    lib = _load()
    t = tokens
    n_rows = int(t.k_tokens.shape[0])
    k = np.ascontiguousarray(t.k_tokens, np.uint16)
    c = np.ascontiguousarray(centroids, np.uint16)
    base, rows = np.ascontiguousarray(t.seg_row_base, np.int64), np.ascontiguousarray(t.seg_rows, np.int32)
    ptr = np.ascontiguousarray(t.seg_cluster_ptr, np.int32)
    asg = np.full(max(n_rows, 1), -7, np.int32)
    best, second = np.zeros(max(n_rows, 1)), np.zeros(max(n_rows, 1))
    lib.dpo_kmeans_assign(len(rows), int(t.head_dim), _ptr(k), _ptr(c), _ptr(base), _ptr(rows), _ptr(ptr), _ptr(asg),
                          _ptr(best), _ptr(second))
    return asg[:n_rows], best[:n_rows], second[:n_rows]


KMEANS_INIT_GIVEN, KMEANS_INIT_STRIDED = 0, 1


def kmeans_fit(tokens, centroids, n_iters: int, init: int = KMEANS_INIT_GIVEN):
    """k-means over the keys of every segment as a procedure (Sec. 4.1 names k-means; initial centroids, iteration
    count and the fate of an emptied cluster are this build's reading): Lloyd's iteration, n_iters rounds of
    kmeans_assign on the current centroids followed by centroid = mean key of the cluster (build_cluster_cache's
    means: fp64 sums in token order, one rounding to bf16); a cluster without tokens keeps its centroid.
    init STRIDED: centroid c of a segment with n tokens and kc clusters starts as the key of token floor(c n / kc)
    (a zero row if n == 0); GIVEN: `centroids` (uint16 bf16 bits [total_clusters, d]).
    -> (centroids after the last update, assignment of the last round or None if n_iters == 0)"""
    import copy
    t = copy.copy(tokens)
    n_cl, d = int(t.seg_cluster_ptr[-1]), int(t.head_dim)
    if init == KMEANS_INIT_STRIDED:
        cent = np.zeros((n_cl, d), np.uint16)
        for seg in range(t.n_seg):
            a, e = int(t.seg_cluster_ptr[seg]), int(t.seg_cluster_ptr[seg + 1])
            n, r0 = int(t.seg_rows[seg]), int(t.seg_row_base[seg])
            for c in range(e - a):
                if n > 0:
                    cent[a + c] = t.k_tokens[r0 + (c * n) // (e - a)]
    else:
        cent = np.array(centroids, dtype=np.uint16, copy=True)
    asg = None
    for _ in range(n_iters):
        asg, _best, _second = kmeans_assign(t, cent)
        t.assignment = asg
        means = build_cluster_cache(t)
        keep = means["cluster_sizes"] > 0
        cent = np.where(keep[:, None], means["k_centroids"], cent)
    return cent, asg
