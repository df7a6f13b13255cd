"""Builds the gfx950 shared library ``libdp_hip.so`` in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG), "include")
LIB = os.path.join(PKG, "libdp_hip.so")
OBJ_DIR = os.path.join(PKG, "_build")
SOURCES = ["dp_api.hip", "dp_score.hip", "dp_select.hip", "dp_decode.hip", "dp_dense.hip", "dp_build.hip",
           "dp_variants.hip", "dp_kmeans.hip", "dp_union.hip", "dp_probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are switched off for every device function
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         # leading scalar kernel parameters arrive in registers at wave launch (no argument load in front of the work)
         "-mllvm", "-amdgpu-kernarg-preload-count=16"]
NOISE = "is not a recognized feature for this target"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def _newest_header() -> float:
    hdrs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))]
    hdrs += [os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE)]
    return max(os.path.getmtime(h) for h in hdrs)


def build(verbose: bool = False, only_changed: bool = False) -> str:
    """Compile every HIP source (in parallel, one object each) and link paper_2602_05191_amd/libdp_hip.so.
    Always recompiles everything unless only_changed is set (then a source is skipped when its object is newer
    than the source and than every header)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdr_time = _newest_header() if only_changed else 0.0
    jobs, objs = [], []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ_DIR, s + ".o")
        objs.append(obj)
        if only_changed and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), hdr_time):
            continue
        jobs.append([HIPCC, *FLAGS, "-I", INCLUDE, "-I", CSRC, "-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    tmp = LIB + f".tmp{os.getpid()}"
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp], verbose)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, only_changed="--changed" in sys.argv))
