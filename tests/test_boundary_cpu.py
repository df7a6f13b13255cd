"""CPU-only checks of the C ABI library: it loads, exports every symbol that
include/dp.h declares, and its host-only functions behave (no kernel is
launched here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2602_05191_amd as dp
    if not os.path.exists(dp.library_path()):
        from paper_2602_05191_amd import build
        build.build()
    return dp.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"dp_score_centroids", "dp_topp_select", "dp_sparse_decode", "dp_decode_attention"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/dp.h but not exported"
    from paper_2602_05191_amd.binding import EXPORTS
    assert sorted(EXPORTS) == names


def _problem(**kw):
    from paper_2602_05191_amd.binding import _Problem
    base = dict(batch=1, n_kv_heads=8, n_q_heads=32, head_dim=128, q=1, k_cache=1, v_cache=1, seg_row_base=1,
                seg_cluster_ptr=1, cluster_offsets=1, cluster_sizes=1, k_centroids=1, v_centroids=1,
                total_clusters=65536, max_clusters_per_seg=8192, max_rows_per_seg=131072, sm_scale=0.0, flags=0)
    base.update(kw)
    return _Problem(**base)


def test_workspace_size_and_layout(lib):
    from paper_2602_05191_amd.binding import _Layout
    p = _problem()
    total = lib.dp_workspace_bytes(C.byref(p))
    lay = _Layout()
    assert lib.dp_get_workspace_layout(C.byref(p), C.byref(lay)) == 0
    assert lay.total == total > 0
    offs = [lay.logits, lay.sel_ids, lay.row_start, lay.chunk_entry, lay.counts, lay.partials, lay.summaries, lay.total]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert lay.sel_ids - lay.logits >= 4 * 4 * 65536                  # G * total_clusters floats
    assert lay.summaries - lay.partials >= 4 * 32 * lay.splits * 130  # (m, l, acc[128]) per head and split
    assert lay.total - lay.summaries >= 8 * 32 * (8192 // 16)         # (max, sum exp) per head and 16 clusters
    assert lib.dp_logits_count(C.byref(p)) == 4 * 65536
    # invalid shapes have no workspace
    assert lib.dp_workspace_bytes(C.byref(_problem(n_q_heads=30))) == 0
    assert lib.dp_workspace_bytes(C.byref(_problem(batch=0))) == 0


def test_host_side_argument_checks_without_launch(lib):
    p = _problem()
    one = C.c_void_p(256)
    # p out of its domain, null output, unsupported head_dim: all rejected before any HIP call
    assert lib.dp_decode_attention(C.byref(p), 0.0, 0.5, one, 1, None, None, None, None, one, 1 << 30, None) == -1
    assert lib.dp_decode_attention(C.byref(p), 0.9, 1.5, one, 1, None, None, None, None, one, 1 << 30, None) == -1
    assert lib.dp_decode_attention(C.byref(p), 0.9, 0.5, None, 1, None, None, None, None, one, 1 << 30, None) == -1
    assert lib.dp_decode_attention(C.byref(p), 0.9, 0.5, one, 1, None, None, None, None, one, 1024, None) == -3
    assert lib.dp_decode_attention(C.byref(p), 0.9, 0.5, one, 7, None, None, None, None, one, 1 << 30, None) == -2
    q = _problem(head_dim=64)
    assert lib.dp_score_centroids(C.byref(q), one, None) == -2
    q = _problem(n_kv_heads=1, n_q_heads=32)
    assert lib.dp_score_centroids(C.byref(q), one, None) == -2       # GQA group 32 > 16
    q = _problem(max_clusters_per_seg=70000, total_clusters=70000)
    assert lib.dp_topp_select(C.byref(q), one, 0.9, 0.5, one, one, one, one, None) == -2
    q = _problem(k_centroids=None)
    assert lib.dp_score_centroids(C.byref(q), one, None) == -1
    for s in (0, -1, -2, -3, -4, -5):
        assert lib.dp_status_string(s).decode().startswith("DP_")
    # the entry point with the static scratch: a problem whose workspace exceeds the array is refused on the host
    big = _problem(batch=4, n_q_heads=64, total_clusters=4 * 65536)
    assert lib.dp_workspace_bytes(C.byref(big)) > (16 << 20)
    assert lib.dp_decode_attention_static(C.byref(big), 0.9, 0.5, one, 1, None, None, None, None, None) == -5
    assert lib.dp_decode_attention_static(C.byref(p), 0.0, 0.5, one, 1, None, None, None, None, None) == -1
    assert lib.dp_workspace_bytes(C.byref(p)) <= (16 << 20)         # the 8B shape at 131072 tokens fits


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_05191_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
