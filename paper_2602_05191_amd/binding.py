"""ctypes binding of libdp_hip.so: argument marshalling only.

Every function has the name and the meaning of the C entry point in
include/dp.h.  torch is used for device memory and for the current stream;
all arithmetic of the decode step happens inside the HIP kernels.  There is no
CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

DP_BF16, DP_F32 = 0, 1
DP_FLAG_P2_ABSOLUTE = 1
DP_FLAG_SEPARATE_DECODE_LAUNCH = 2
DP_CLUSTER_PINNED = 1

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libdp_hip.so")

EXPORTS = ["dp_workspace_bytes", "dp_logits_count", "dp_get_workspace_layout", "dp_score_centroids",
           "dp_score_centroids_timed",
           "dp_topp_select", "dp_topp_select_sorted", "dp_topk_select", "dp_sparse_decode", "dp_sparse_decode_gathered", "dp_decode_attention",
           "dp_group_union_decode_attention",
           "dp_decode_attention_timed", "dp_budget_decode_attention", "dp_dense_decode", "dp_build_workspace_bytes", "dp_build_cluster_cache", "dp_kmeans_workspace_bytes",
           "dp_kmeans_assign", "dp_kmeans_fit_workspace_bytes", "dp_kmeans_fit",
           "dp_decode_attention_static", "dp_stream_read_probe", "dp_decode_attention_launches",
           "dp_status_string"]


class DPError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_status_string(status)} ({status})")


class _Problem(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_kv_heads", C.c_int32), ("n_q_heads", C.c_int32), ("head_dim", C.c_int32),
                ("q", C.c_void_p), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
                ("seg_row_base", C.c_void_p), ("seg_cluster_ptr", C.c_void_p),
                ("cluster_offsets", C.c_void_p), ("cluster_sizes", C.c_void_p),
                ("k_centroids", C.c_void_p), ("v_centroids", C.c_void_p),
                ("total_clusters", C.c_int32), ("max_clusters_per_seg", C.c_int32),
                ("max_rows_per_seg", C.c_int32), ("sm_scale", C.c_float), ("flags", C.c_uint32),
                ("cluster_flags", C.c_void_p)]


class _Prefill(C.Structure):
    _fields_ = [("n_seg", C.c_int32), ("head_dim", C.c_int32), ("k_tokens", C.c_void_p), ("v_tokens", C.c_void_p),
                ("assignment", C.c_void_p), ("seg_row_base", C.c_void_p), ("seg_rows", C.c_void_p),
                ("seg_cluster_ptr", C.c_void_p), ("total_clusters", C.c_int32),
                ("max_clusters_per_seg", C.c_int32), ("max_rows_per_seg", C.c_int32)]


class _Layout(C.Structure):
    _fields_ = [("logits", C.c_size_t), ("sel_ids", C.c_size_t), ("row_start", C.c_size_t),
                ("chunk_entry", C.c_size_t), ("counts", C.c_size_t), ("partials", C.c_size_t),
                ("total", C.c_size_t), ("splits", C.c_int32), ("chunk_rows", C.c_int32), ("summaries", C.c_size_t)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libdp_hip.so (built by paper_2602_05191_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    L = C.CDLL(_LIB_PATH)
    PP, V, F, I = C.POINTER(_Problem), C.c_void_p, C.c_float, C.c_int
    L.dp_workspace_bytes.restype = C.c_size_t
    L.dp_workspace_bytes.argtypes = [PP]
    L.dp_logits_count.restype = C.c_size_t
    L.dp_logits_count.argtypes = [PP]
    L.dp_get_workspace_layout.restype = I
    L.dp_get_workspace_layout.argtypes = [PP, C.POINTER(_Layout)]
    L.dp_score_centroids.restype = I
    L.dp_score_centroids.argtypes = [PP, V, V]
    L.dp_score_centroids_timed.restype = I
    L.dp_score_centroids_timed.argtypes = [PP, V, V, V, V]
    L.dp_topp_select.restype = I
    L.dp_topp_select.argtypes = [PP, V, F, F, V, V, V, V, V]
    L.dp_sparse_decode.restype = I
    L.dp_sparse_decode.argtypes = [PP, V, V, V, V, V, I, V, V, C.c_size_t, V]
    L.dp_decode_attention.restype = I
    L.dp_decode_attention.argtypes = [PP, F, F, V, I, V, V, V, V, V, C.c_size_t, V]
    L.dp_decode_attention_static.restype = I
    L.dp_decode_attention_static.argtypes = [PP, F, F, V, I, V, V, V, V, V]
    L.dp_decode_attention_timed.restype = I
    L.dp_decode_attention_timed.argtypes = [PP, F, F, V, I, V, V, C.c_size_t, V, C.POINTER(C.c_void_p)]
    L.dp_topp_select_sorted.restype = I
    L.dp_topp_select_sorted.argtypes = [PP, V, F, F, V, V, V, V, V]
    L.dp_sparse_decode_gathered.restype = I
    L.dp_sparse_decode_gathered.argtypes = [PP, V, V, V, V, I, V, V, V, I, V, C.c_size_t, V]
    L.dp_group_union_decode_attention.restype = I
    L.dp_group_union_decode_attention.argtypes = [PP, F, F, V, I, V, V, V, V, V, C.c_size_t, V]
    L.dp_topk_select.restype = I
    L.dp_topk_select.argtypes = [PP, V, I, I, V, V, V, V, V]
    L.dp_budget_decode_attention.restype = I
    L.dp_budget_decode_attention.argtypes = [PP, I, I, V, I, V, V, V, V, V, C.c_size_t, V]
    L.dp_dense_decode.restype = I
    L.dp_dense_decode.argtypes = [PP, V, V, I, V, V, C.c_size_t, V]
    L.dp_build_workspace_bytes.restype = C.c_size_t
    L.dp_build_workspace_bytes.argtypes = [C.POINTER(_Prefill)]
    L.dp_build_cluster_cache.restype = I
    L.dp_build_cluster_cache.argtypes = [C.POINTER(_Prefill), V, V, V, V, V, V, V, V, V, C.c_size_t, V]
    L.dp_kmeans_workspace_bytes.restype = C.c_size_t
    L.dp_kmeans_workspace_bytes.argtypes = [C.POINTER(_Prefill)]
    L.dp_kmeans_assign.restype = I
    L.dp_kmeans_assign.argtypes = [C.POINTER(_Prefill), V, V, V, V, C.c_size_t, V]
    L.dp_kmeans_fit_workspace_bytes.restype = C.c_size_t
    L.dp_kmeans_fit_workspace_bytes.argtypes = [C.POINTER(_Prefill)]
    L.dp_kmeans_fit.restype = I
    L.dp_kmeans_fit.argtypes = [C.POINTER(_Prefill), V, C.c_int32, C.c_uint32, V, V, V, C.c_size_t, V]
    L.dp_decode_attention_launches.restype = C.c_int32
    L.dp_decode_attention_launches.argtypes = [PP]
    L.dp_stream_read_probe.restype = I
    L.dp_stream_read_probe.argtypes = [V, C.c_size_t, V, V, V, V]
    L.dp_status_string.restype = C.c_char_p
    L.dp_status_string.argtypes = [I]
    _lib = L
    return L


def _status_string(status: int) -> str:
    return load_library().dp_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise DPError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    return t.data_ptr() if t.numel() else None


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


@dataclass
class DeviceCache:
    """Device-resident copies of one decode step's inputs (bf16 kept as raw int16 bits)."""
    batch: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    q: torch.Tensor
    k_cache: torch.Tensor
    v_cache: torch.Tensor
    seg_row_base: torch.Tensor
    seg_cluster_ptr: torch.Tensor
    cluster_offsets: torch.Tensor
    cluster_sizes: torch.Tensor
    k_centroids: torch.Tensor
    v_centroids: torch.Tensor
    total_clusters: int
    max_clusters_per_seg: int
    max_rows_per_seg: int
    cluster_flags: Optional[torch.Tensor] = None  # uint8 [total_clusters], DP_CLUSTER_* bits

    @staticmethod
    def from_host(cache, device="cuda:0") -> "DeviceCache":
        """Upload a workloads.ClusteredCache (numpy, bf16 as uint16 bits)."""
        def up(a, dt):
            return torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(device)
        return DeviceCache(
            batch=cache.batch, n_kv_heads=cache.n_kv_heads, n_q_heads=cache.n_q_heads, head_dim=cache.head_dim,
            q=up(cache.q, np.int16), k_cache=up(cache.k_cache, np.int16), v_cache=up(cache.v_cache, np.int16),
            seg_row_base=up(cache.seg_row_base, np.int64), seg_cluster_ptr=up(cache.seg_cluster_ptr, np.int32),
            cluster_offsets=up(cache.cluster_offsets, np.int32), cluster_sizes=up(cache.cluster_sizes, np.int32),
            k_centroids=up(cache.k_centroids, np.int16), v_centroids=up(cache.v_centroids, np.int16),
            total_clusters=int(cache.seg_cluster_ptr[-1]), max_clusters_per_seg=cache.max_clusters_per_seg,
            max_rows_per_seg=cache.max_rows_per_seg,
            cluster_flags=(up(cache.cluster_flags, np.uint8)
                           if getattr(cache, "cluster_flags", None) is not None else None))

    def clone(self) -> "DeviceCache":
        """A copy at distinct device addresses (used to rotate layers in the bench)."""
        kw = {k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in self.__dict__.items()}
        return DeviceCache(**kw)


class Problem:
    """Host-side dp_problem that points at a DeviceCache's tensors."""

    def __init__(self, dc: DeviceCache, sm_scale: float = 0.0, flags: int = 0):
        self.dc = dc
        self.nh = dc.batch * dc.n_q_heads
        self.c = _Problem(dc.batch, dc.n_kv_heads, dc.n_q_heads, dc.head_dim, _ptr(dc.q), _ptr(dc.k_cache),
                          _ptr(dc.v_cache), _ptr(dc.seg_row_base), _ptr(dc.seg_cluster_ptr),
                          _ptr(dc.cluster_offsets), _ptr(dc.cluster_sizes), _ptr(dc.k_centroids),
                          _ptr(dc.v_centroids), dc.total_clusters, dc.max_clusters_per_seg, dc.max_rows_per_seg,
                          float(sm_scale), int(flags), _ptr(dc.cluster_flags))

    @property
    def ref(self):
        return C.byref(self.c)

    @property
    def device(self):
        return self.dc.q.device


def dp_workspace_bytes(problem: Problem) -> int:
    return int(load_library().dp_workspace_bytes(problem.ref))


def dp_workspace_layout(problem: Problem) -> dict:
    lay = _Layout()
    _check(load_library().dp_get_workspace_layout(problem.ref, C.byref(lay)), "dp_get_workspace_layout")
    return {n: int(getattr(lay, n)) for n, _ in _Layout._fields_}


def dp_score_centroids(problem: Problem, logits: torch.Tensor, stream=None) -> None:
    L = load_library()
    assert logits.dtype == torch.float32 and logits.is_contiguous() and logits.numel() >= L.dp_logits_count(problem.ref)
    _check(L.dp_score_centroids(problem.ref, _ptr(logits), _stream(stream)), "dp_score_centroids")


def dp_score_centroids_timed(problem: Problem, logits: torch.Tensor, start_event: int, stop_event: int,
                             stream=None) -> None:
    """start_event / stop_event: raw hipEvent_t handles (ints) that receive the kernel's own timestamps."""
    _check(load_library().dp_score_centroids_timed(problem.ref, _ptr(logits), _stream(stream), start_event,
                                                   stop_event), "dp_score_centroids_timed")


def dp_topp_select(problem: Problem, logits: torch.Tensor, p1: float, p2: float, sel_ids: torch.Tensor,
                   n_exact: torch.Tensor, n_retained: torch.Tensor, n_exact_tokens: torch.Tensor, stream=None) -> None:
    for t in (sel_ids, n_exact, n_retained, n_exact_tokens):
        assert t.dtype == torch.int32 and t.is_contiguous()
    assert sel_ids.numel() >= problem.nh * problem.dc.max_clusters_per_seg and n_exact.numel() >= problem.nh
    _check(load_library().dp_topp_select(problem.ref, _ptr(logits), p1, p2, _ptr(sel_ids), _ptr(n_exact),
                                         _ptr(n_retained), _ptr(n_exact_tokens), _stream(stream)), "dp_topp_select")


def dp_topk_select(problem: Problem, logits: torch.Tensor, k_retained: int, k_exact: int, sel_ids: torch.Tensor,
                   n_exact: torch.Tensor, n_retained: torch.Tensor, n_exact_tokens: torch.Tensor, stream=None) -> None:
    for t in (sel_ids, n_exact, n_retained, n_exact_tokens):
        assert t.dtype == torch.int32 and t.is_contiguous()
    assert sel_ids.numel() >= problem.nh * problem.dc.max_clusters_per_seg and n_exact.numel() >= problem.nh
    _check(load_library().dp_topk_select(problem.ref, _ptr(logits), k_retained, k_exact, _ptr(sel_ids), _ptr(n_exact),
                                         _ptr(n_retained), _ptr(n_exact_tokens), _stream(stream)), "dp_topk_select")


def dp_sparse_decode(problem: Problem, sel_ids: torch.Tensor, n_exact: torch.Tensor, n_retained: torch.Tensor,
                     out: torch.Tensor, lse: Optional[torch.Tensor], workspace: torch.Tensor, stream=None) -> None:
    dt = {torch.float32: DP_F32, torch.bfloat16: DP_BF16}[out.dtype]
    assert out.is_contiguous() and out.numel() == problem.nh * problem.dc.head_dim
    _check(load_library().dp_sparse_decode(problem.ref, _ptr(sel_ids), _ptr(n_exact), _ptr(n_retained), None,
                                           _ptr(out), dt, _ptr(lse), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream(stream)),
           "dp_sparse_decode")


def dp_decode_attention(problem: Problem, p1: float, p2: float, out: torch.Tensor, lse: Optional[torch.Tensor],
                        workspace: torch.Tensor, n_exact: Optional[torch.Tensor] = None,
                        n_retained: Optional[torch.Tensor] = None, n_exact_tokens: Optional[torch.Tensor] = None,
                        stream=None) -> None:
    dt = {torch.float32: DP_F32, torch.bfloat16: DP_BF16}[out.dtype]
    assert out.is_contiguous() and out.numel() == problem.nh * problem.dc.head_dim
    _check(load_library().dp_decode_attention(problem.ref, p1, p2, _ptr(out), dt, _ptr(lse), _ptr(n_exact),
                                              _ptr(n_retained), _ptr(n_exact_tokens), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream(stream)),
           "dp_decode_attention")


class BoundDecodeStep:
    """dp_decode_attention with its arguments marshalled once: calling the object enqueues one step (a serving loop
    calls the same step many times; converting the same pointers again on every call costs the host several
    microseconds, as much as a third of a small step).  The tensors are kept alive by the object and must not be
    resized; ``stream`` (default: the stream current at construction) is fixed too."""

    def __init__(self, problem: Problem, p1: float, p2: float, out: torch.Tensor, lse: Optional[torch.Tensor],
                 workspace: torch.Tensor, n_exact: Optional[torch.Tensor] = None,
                 n_retained: Optional[torch.Tensor] = None, n_exact_tokens: Optional[torch.Tensor] = None,
                 stream=None):
        dt = {torch.float32: DP_F32, torch.bfloat16: DP_BF16}[out.dtype]
        assert out.is_contiguous() and out.numel() == problem.nh * problem.dc.head_dim
        self._keep = (problem, out, lse, workspace, n_exact, n_retained, n_exact_tokens)
        self._fn = load_library().dp_decode_attention
        V = C.c_void_p
        self._args = (problem.ref, C.c_float(p1), C.c_float(p2), V(_ptr(out)), C.c_int(dt), V(_ptr(lse)),
                      V(_ptr(n_exact)), V(_ptr(n_retained)), V(_ptr(n_exact_tokens)), V(_ptr(workspace)),
                      C.c_size_t(workspace.numel() * workspace.element_size()), V(_stream(stream)))

    def __call__(self) -> None:
        status = self._fn(*self._args)
        if status != 0:
            raise DPError(status, "dp_decode_attention")


DP_STATIC_SCRATCH_BYTES = 16 << 20


def dp_decode_attention_static(problem: Problem, p1: float, p2: float, out: torch.Tensor,
                               lse: Optional[torch.Tensor], n_exact: Optional[torch.Tensor] = None,
                               n_retained: Optional[torch.Tensor] = None,
                               n_exact_tokens: Optional[torch.Tensor] = None, stream=None) -> None:
    """dp_decode_attention with the library's own static scratch array in place of a workspace."""
    dt = {torch.float32: DP_F32, torch.bfloat16: DP_BF16}[out.dtype]
    assert out.is_contiguous() and out.numel() == problem.nh * problem.dc.head_dim
    _check(load_library().dp_decode_attention_static(problem.ref, p1, p2, _ptr(out), dt, _ptr(lse), _ptr(n_exact),
                                                     _ptr(n_retained), _ptr(n_exact_tokens), _stream(stream)),
           "dp_decode_attention_static")


def dp_budget_decode_attention(problem: Problem, k_retained: int, k_exact: int, out: torch.Tensor,
                               lse: Optional[torch.Tensor], workspace: torch.Tensor,
                               n_exact: Optional[torch.Tensor] = None, n_retained: Optional[torch.Tensor] = None,
                               n_exact_tokens: Optional[torch.Tensor] = None, stream=None) -> None:
    dt = {torch.float32: DP_F32, torch.bfloat16: DP_BF16}[out.dtype]
    assert out.is_contiguous() and out.numel() == problem.nh * problem.dc.head_dim
    _check(load_library().dp_budget_decode_attention(problem.ref, k_retained, k_exact, _ptr(out), dt, _ptr(lse),
                                                     _ptr(n_exact), _ptr(n_retained), _ptr(n_exact_tokens),
                                                     _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                     _stream(stream)),
           "dp_budget_decode_attention")


def dp_dense_decode(problem: Problem, seg_rows: torch.Tensor, out: torch.Tensor, lse: Optional[torch.Tensor],
                    workspace: torch.Tensor, stream=None) -> None:
    dt = {torch.float32: DP_F32, torch.bfloat16: DP_BF16}[out.dtype]
    assert out.is_contiguous() and out.numel() == problem.nh * problem.dc.head_dim
    assert seg_rows.dtype == torch.int32 and seg_rows.is_contiguous()
    assert seg_rows.numel() == problem.c.batch * problem.c.n_kv_heads
    _check(load_library().dp_dense_decode(problem.ref, _ptr(seg_rows), _ptr(out), dt, _ptr(lse), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)),
           "dp_dense_decode")


class Prefill:
    """Host-side dp_prefill over device tensors (bf16 as int16 bits)."""

    def __init__(self, k_tokens: torch.Tensor, v_tokens: torch.Tensor, assignment: torch.Tensor,
                 seg_row_base: torch.Tensor, seg_rows: torch.Tensor, seg_cluster_ptr: torch.Tensor,
                 total_clusters: int, max_clusters_per_seg: int, max_rows_per_seg: int, head_dim: int = 128):
        self.tensors = (k_tokens, v_tokens, assignment, seg_row_base, seg_rows, seg_cluster_ptr)
        assert assignment.dtype == torch.int32 and seg_rows.dtype == torch.int32
        assert seg_row_base.dtype == torch.int64 and seg_cluster_ptr.dtype == torch.int32
        self.n_seg = int(seg_rows.numel())
        self.total_rows, self.total_clusters = int(k_tokens.shape[0]), int(total_clusters)
        self.c = _Prefill(self.n_seg, head_dim, _ptr(k_tokens), _ptr(v_tokens), _ptr(assignment), _ptr(seg_row_base),
                          _ptr(seg_rows), _ptr(seg_cluster_ptr), int(total_clusters), int(max_clusters_per_seg),
                          int(max_rows_per_seg))

    @property
    def ref(self):
        return C.byref(self.c)


def dp_build_workspace_bytes(prefill: Prefill) -> int:
    return int(load_library().dp_build_workspace_bytes(prefill.ref))


def dp_build_cluster_cache(prefill: Prefill, k_cache: torch.Tensor, v_cache: torch.Tensor,
                           cluster_offsets: torch.Tensor, cluster_sizes: torch.Tensor, k_centroids: torch.Tensor,
                           v_centroids: torch.Tensor, workspace: torch.Tensor, v_sums: Optional[torch.Tensor] = None,
                           token_row: Optional[torch.Tensor] = None, stream=None) -> None:
    for t in (cluster_offsets, cluster_sizes):
        assert t.dtype == torch.int32 and t.is_contiguous() and t.numel() >= prefill.total_clusters
    for t in (k_cache, v_cache):
        assert t.is_contiguous() and t.element_size() == 2 and t.numel() >= prefill.total_rows * prefill.c.head_dim
    for t in (k_centroids, v_centroids):
        assert t.is_contiguous() and t.element_size() == 2 and t.numel() >= prefill.total_clusters * prefill.c.head_dim
    assert v_sums is None or (v_sums.dtype == torch.float32 and v_sums.is_contiguous())
    assert token_row is None or (token_row.dtype == torch.int32 and token_row.numel() >= prefill.total_rows)
    _check(load_library().dp_build_cluster_cache(prefill.ref, _ptr(k_cache), _ptr(v_cache), _ptr(cluster_offsets),
                                                 _ptr(cluster_sizes), _ptr(k_centroids), _ptr(v_centroids),
                                                 _ptr(v_sums), _ptr(token_row), _ptr(workspace),
                                                 workspace.numel() * workspace.element_size(), _stream(stream)),
           "dp_build_cluster_cache")


def dp_decode_attention_timed(problem: Problem, p1: float, p2: float, out: torch.Tensor, lse: Optional[torch.Tensor],
                              workspace: torch.Tensor, events, stream=None) -> None:
    """events: 6 raw hipEvent_t handles (ints or ctypes.c_void_p; None to skip one):
    score begin / end, select begin / end, decode begin / end."""
    dt = {torch.float32: DP_F32, torch.bfloat16: DP_BF16}[out.dtype]
    assert len(events) == 6
    arr = (C.c_void_p * 6)(*[e.value if isinstance(e, C.c_void_p) else e for e in events])
    _check(load_library().dp_decode_attention_timed(problem.ref, p1, p2, _ptr(out), dt, _ptr(lse), _ptr(workspace),
                                                    workspace.numel() * workspace.element_size(), _stream(stream),
                                                    arr),
           "dp_decode_attention_timed")


def dp_topp_select_sorted(problem: Problem, logits: torch.Tensor, p1: float, p2: float, sel_ids: torch.Tensor,
                          n_exact: torch.Tensor, n_retained: torch.Tensor, n_exact_tokens: torch.Tensor,
                          stream=None) -> None:
    """A/B variant of dp_topp_select (sort first, then prefix sums); same outputs."""
    for t in (sel_ids, n_exact, n_retained, n_exact_tokens):
        assert t.dtype == torch.int32 and t.is_contiguous()
    assert sel_ids.numel() >= problem.nh * problem.dc.max_clusters_per_seg and n_exact.numel() >= problem.nh
    _check(load_library().dp_topp_select_sorted(problem.ref, _ptr(logits), p1, p2, _ptr(sel_ids), _ptr(n_exact),
                                                _ptr(n_retained), _ptr(n_exact_tokens), _stream(stream)),
           "dp_topp_select_sorted")


def dp_sparse_decode_gathered(problem: Problem, sel_ids: torch.Tensor, n_exact: torch.Tensor, n_retained: torch.Tensor,
                              out: torch.Tensor, lse: Optional[torch.Tensor], k_buf: torch.Tensor, v_buf: torch.Tensor,
                              rows_cap: int, workspace: torch.Tensor, stream=None) -> None:
    """A/B variant of dp_sparse_decode (gather into contiguous buffers, then attend); same outputs."""
    dt = {torch.float32: DP_F32, torch.bfloat16: DP_BF16}[out.dtype]
    assert out.is_contiguous() and out.numel() == problem.nh * problem.dc.head_dim
    for t in (k_buf, v_buf):
        assert t.is_contiguous() and t.element_size() == 2 and t.numel() >= problem.nh * rows_cap * problem.dc.head_dim
    _check(load_library().dp_sparse_decode_gathered(problem.ref, _ptr(sel_ids), _ptr(n_exact), _ptr(n_retained),
                                                    _ptr(out), dt, _ptr(lse), _ptr(k_buf), _ptr(v_buf), int(rows_cap),
                                                    _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                    _stream(stream)),
           "dp_sparse_decode_gathered")


def dp_group_union_decode_attention(problem: Problem, p1: float, p2: float, out: torch.Tensor,
                                    lse: Optional[torch.Tensor], union_ids: torch.Tensor, n_exact_u: torch.Tensor,
                                    n_retained_u: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """A/B variant: every head of a GQA group attends over the union of the group's per-head sets."""
    dt = {torch.float32: DP_F32, torch.bfloat16: DP_BF16}[out.dtype]
    n_seg = problem.dc.batch * problem.dc.n_kv_heads
    assert out.is_contiguous() and out.numel() == problem.nh * problem.dc.head_dim
    assert union_ids.dtype == torch.int32 and union_ids.numel() >= n_seg * problem.dc.max_clusters_per_seg
    for t in (n_exact_u, n_retained_u):
        assert t.dtype == torch.int32 and t.numel() >= n_seg
    _check(load_library().dp_group_union_decode_attention(problem.ref, p1, p2, _ptr(out), dt, _ptr(lse),
                                                          _ptr(union_ids), _ptr(n_exact_u), _ptr(n_retained_u),
                                                          _ptr(workspace),
                                                          workspace.numel() * workspace.element_size(),
                                                          _stream(stream)),
           "dp_group_union_decode_attention")


def dp_decode_attention_launches(problem: Problem) -> int:
    return int(load_library().dp_decode_attention_launches(problem.ref))


def dp_stream_read_probe(buffer: torch.Tensor, sink: Optional[torch.Tensor] = None, stream=None, start_event=None,
                         stop_event=None) -> None:
    """Measurement aid: one launch that reads the whole tensor once and writes nothing.  start_event / stop_event:
    raw hipEvent_t handles that receive the kernel's own timestamps."""
    assert buffer.is_contiguous()
    _check(load_library().dp_stream_read_probe(_ptr(buffer), buffer.numel() * buffer.element_size(), _ptr(sink),
                                               _stream(stream), start_event, stop_event), "dp_stream_read_probe")


def dp_kmeans_workspace_bytes(prefill: Prefill) -> int:
    return int(load_library().dp_kmeans_workspace_bytes(prefill.ref))


def dp_kmeans_assign(prefill: Prefill, centroids: torch.Tensor, assignment: torch.Tensor, workspace: torch.Tensor,
                     best_score: Optional[torch.Tensor] = None, stream=None) -> None:
    assert centroids.is_contiguous() and centroids.element_size() == 2
    assert centroids.numel() >= prefill.total_clusters * prefill.c.head_dim
    assert assignment.dtype == torch.int32 and assignment.is_contiguous() and assignment.numel() >= prefill.total_rows
    assert best_score is None or (best_score.dtype == torch.float32 and best_score.numel() >= prefill.total_rows)
    _check(load_library().dp_kmeans_assign(prefill.ref, _ptr(centroids), _ptr(assignment), _ptr(best_score),
                                           _ptr(workspace), workspace.numel() * workspace.element_size(),
                                           _stream(stream)),
           "dp_kmeans_assign")


DP_KMEANS_INIT_GIVEN = 0
DP_KMEANS_INIT_STRIDED = 1


def dp_kmeans_fit_workspace_bytes(prefill: Prefill) -> int:
    return int(load_library().dp_kmeans_fit_workspace_bytes(prefill.ref))


def dp_kmeans_fit(prefill: Prefill, centroids: torch.Tensor, n_iters: int, init: int, assignment: Optional[torch.Tensor],
                  workspace: torch.Tensor, best_score: Optional[torch.Tensor] = None, stream=None) -> None:
    assert centroids.is_contiguous() and centroids.element_size() == 2
    assert centroids.numel() >= prefill.total_clusters * prefill.c.head_dim
    assert assignment is None or (assignment.dtype == torch.int32 and assignment.is_contiguous() and
                                  assignment.numel() >= prefill.total_rows)
    assert best_score is None or (best_score.dtype == torch.float32 and best_score.numel() >= prefill.total_rows)
    _check(load_library().dp_kmeans_fit(prefill.ref, _ptr(centroids), int(n_iters), int(init), _ptr(assignment),
                                        _ptr(best_score), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)),
           "dp_kmeans_fit")
