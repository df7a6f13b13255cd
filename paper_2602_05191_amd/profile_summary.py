"""Short text summary of rocprofv3 runs of bench.py (the files under profiles/ are its output).

Three runs of the same bench command are read, each from the result database rocprofv3 leaves in its -d folder:

    rocprofv3 --kernel-trace --stats -d <trace_dir> -o bench -- python3 bench.py <bench args>
    rocprofv3 --pmc FETCH_SIZE        -d <fetch_dir> -o f     -- python3 bench.py <counter-run args>
    rocprofv3 --pmc WRITE_SIZE        -d <write_dir> -o w     -- python3 bench.py <counter-run args>

usage:
    python3 -m paper_2602_05191_amd.profile_summary --title "<workload>" --bench-args "<bench args>" \
        --counter-args "<counter-run args>" --trace <trace_dir>/bench_results.db --fetch <fetch_dir>/f_results.db \
        --write <write_dir>/w_results.db [--kernel <name prefix> --alg-bytes <bytes per launch>] > profiles/<name>.txt

Optionally a fourth run with SQ counters (at most 8 in one run), reported for the kernel named by --kernel:

    rocprofv3 --pmc <SQ counters>     -d <sq_dir>    -o s     -- python3 bench.py <counter-run args>
    ... --sq <sq_dir>/s_results.db --sq-counters "<SQ counters>"

Durations are aggregated per kernel name; HBM traffic is the median per dispatch of the two counters, scaled by
what the same counters read for the largest device-to-device copy of the run (a K cache replica of known size).
"""
from __future__ import annotations

import argparse
import os
import re
import sqlite3
import statistics
from collections import defaultdict


def short(name: str) -> str:
    m = re.search(r"(\w+_kernel(<[^>]*>)?)", name)
    return m.group(1) if m else name[:48]


def kernel_rows(db: str):
    cur = sqlite3.connect(db).cursor()
    return cur.execute("select name,start,end from kernels order by start").fetchall()


def counter_medians(db: str):
    cur = sqlite3.connect(db).cursor()
    d = defaultdict(list)
    for name, _counter, val, grid in cur.execute(
            "select kernel_name,counter_name,value,grid_size from counters_collection"):
        d[(short(name), grid)].append(val)
    return d


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--title", required=True)
    ap.add_argument("--bench-args", required=True)
    ap.add_argument("--counter-args", default=None)
    ap.add_argument("--trace", required=True)
    ap.add_argument("--fetch", default=None)
    ap.add_argument("--write", default=None)
    ap.add_argument("--kernel", default=None, help="name prefix of the kernel to report the roofline figures for")
    ap.add_argument("--alg-bytes", type=float, default=None, help="algorithmic bytes per launch of that kernel")
    ap.add_argument("--in-step", default="score,select", help="prefixes of the kernels of one dp_decode_attention step, in order")
    ap.add_argument("--sq", default=None, help="result database of a run with SQ counters (one --pmc run)")
    ap.add_argument("--sq-counters", default="", help="the counters of that run, as given to --pmc")
    a = ap.parse_args()
    cargs = a.counter_args or a.bench_args
    out = []
    P = out.append
    P(f"Workload: {a.title}")
    P("Machine: one AMD Instinct MI355X (gfx950, 256 CUs, HBM3E), ROCm 7.2.0, rocprofv3; figures aggregated per kernel "
      "name from the tool's result database by paper_2602_05191_amd/profile_summary.py")
    P("")
    P("== kernel trace ==")
    P(f"command: rocprofv3 --kernel-trace --stats -d {os.path.dirname(a.trace)} -o bench -- python3 bench.py {a.bench_args}")
    rows = kernel_rows(a.trace)
    dur = defaultdict(list)
    for n, s, e in rows:
        dur[short(n)].append((e - s) / 1e3)
    P(f"{'kernel':44s} {'calls':>6s} {'avg_us':>8s} {'med_us':>8s} {'min_us':>8s} {'max_us':>8s} {'total_ms':>9s}")
    for n, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        P(f"{n[:44]:44s} {len(v):6d} {statistics.mean(v):8.2f} {statistics.median(v):8.2f} {min(v):8.2f} {max(v):8.2f} "
          f"{sum(v) / 1e3:9.3f}")
    P("(bench.py runs the step's kernels inside dp_decode_attention and alone in its per-stage loops, and the baselines, "
      "A/B variants, prefill build and k-means assignment in their own sections; __amd_rocclr_copyBuffer = the "
      "device-to-device copies that make the layer replicas)")
    # the kernels of one step: consecutive launches that match the given prefixes, followed by the first again
    seq = [p for p in a.in_step.split(",") if p]
    names = [short(r[0]) for r in rows]
    groups = []
    for i in range(len(rows) - len(seq)):
        if all(names[i + k].startswith(seq[k]) for k in range(len(seq))) and names[i + len(seq)].startswith(seq[0]):
            groups.append([(rows[i + k][2] - rows[i + k][1]) / 1e3 for k in range(len(seq))])
    med = None
    if len(groups) > 20:
        groups = groups[10:]
        med = [statistics.median(g[k] for g in groups) for k in range(len(seq))]
        P(f"inside dp_decode_attention (n={len(groups)} steps), median kernel duration: " +
          ", ".join(f"{seq[k]} {med[k]:.2f} us" for k in range(len(seq))))
        P("(gaps between kernels under the profiler are tool overhead; bench.py without the profiler reports the step time)")
    if a.fetch and a.write:
        P("")
        P("== HBM traffic (two counter runs) ==")
        P(f"command: rocprofv3 --pmc FETCH_SIZE -d {os.path.dirname(a.fetch)} -o f -- python3 bench.py {cargs}")
        P(f"command: rocprofv3 --pmc WRITE_SIZE -d {os.path.dirname(a.write)} -o w -- python3 bench.py {cargs}")
        f, w = counter_medians(a.fetch), counter_medians(a.write)
        P(f"{'kernel':30s} {'grid':>9s} {'n':>5s} {'FETCH_SIZE KiB (median)':>24s} {'WRITE_SIZE KiB (median)':>24s}")
        for k in sorted(set(f) | set(w)):
            if "Fill" in k[0]:
                continue
            fv = statistics.median(f[k]) if k in f else float("nan")
            wv = statistics.median(w[k]) if k in w else float("nan")
            P(f"{k[0][:30]:30s} {k[1]:9d} {len(f.get(k, [])):5d} {fv:24.2f} {wv:24.2f}")
        cp = [(k, max(v)) for k, v in f.items() if "copyBuffer" in k[0]]
        cw = [(k, max(v)) for k, v in w.items() if "copyBuffer" in k[0]]
        kf, kw = max(cp, key=lambda x: x[1]), max(cw, key=lambda x: x[1])
        sf = kw[1] / kf[1]
        P(f"calibration: the largest device-to-device copy (a K or V cache replica) writes WRITE_SIZE = {kw[1]:.0f} KiB = "
          f"its size, and reads FETCH_SIZE = {kf[1]:.0f} KiB,")
        P(f"  i.e. FETCH_SIZE reports {1 / sf:.3f} of the bytes read: FETCH_SIZE is scaled by {sf:.3f}, WRITE_SIZE by 1.000")
        if a.kernel:
            kk = [k for k in f if k[0].startswith(a.kernel)]
            k = max(kk, key=lambda k: len(f[k]))
            fv, wv = statistics.median(f[k]), statistics.median(w[k])
            tb = (fv * sf + wv) * 1024
            d = dur[k[0]]
            P("")
            P(f"== {k[0]} ==")
            P(f"duration (kernel trace above): average {statistics.mean(d):.2f} us, median {statistics.median(d):.2f} us over "
              f"{len(d)} launches")
            ref = statistics.mean(d)
            if med is not None:
                for j, pfx in enumerate(seq):
                    if k[0].startswith(pfx) and pfx != "score":
                        ref = med[j]
                        P(f"  (the launches include bench.py's other loops, which attend other row sets; inside "
                          f"dp_decode_attention the median is {med[j]:.2f} us)")
            P(f"HBM traffic per launch (medians of the two counter runs): read {fv * sf / 1024:.2f} MiB + written {wv / 1024:.2f} MiB")
            P(f"traffic_bytes_per_launch = {tb:.0f}")
            if a.alg_bytes:
                P(f"algorithmic_bytes_per_launch = {a.alg_bytes:.0f}   (traffic / algorithmic = {tb / a.alg_bytes:.3f})")
                P(f"achieved = algorithmic bytes / duration ({ref:.2f} us) = {a.alg_bytes / ref / 1e3:.0f} GB/s = "
                  f"{a.alg_bytes / ref / 1e3 / 8000:.3f} of the 8000 GB/s HBM peak")
    if a.sq and a.kernel:
        cur = sqlite3.connect(a.sq).cursor()
        per = defaultdict(lambda: defaultdict(list))
        for name, counter, val, grid in cur.execute(
                "select kernel_name,counter_name,value,grid_size from counters_collection"):
            if short(name).startswith(a.kernel):
                per[grid][counter].append(val)
        if per:
            grid = max(per, key=lambda g: sum(len(v) for v in per[g].values()))
            c = {k: statistics.median(v) for k, v in per[grid].items()}
            P("")
            P(f"== SQ counters of {a.kernel} (one counter run; median per launch, summed over the device) ==")
            P(f"command: rocprofv3 --pmc {a.sq_counters} -d {os.path.dirname(a.sq)} -o s -- python3 bench.py {cargs}")
            for k in sorted(c):
                P(f"{k:32s} n={len(per[grid][k]):5d} median {c[k]:16.0f}")
            wc = c.get("SQ_WAVE_CYCLES")
            if wc:
                parts = []
                for k, label in (("SQ_WAIT_INST_ANY", "waiting on an instruction's dependency"),
                                 ("SQ_WAIT_INST_LDS", "waiting on LDS"), ("SQ_ACTIVE_INST_VALU", "issuing vector ALU"),
                                 ("SQ_ACTIVE_INST_LDS", "issuing LDS"), ("SQ_ACTIVE_INST_SCA", "issuing scalar")):
                    if k in c:
                        parts.append(f"{100 * c[k] / wc:.0f} % {label}")
                if parts:
                    P("share of the cycles that waves were resident (waves that wait at a barrier or sleep count too): "
                      + ", ".join(parts))
            insts = [(k, c[k]) for k in ("SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_LDS", "SQ_INSTS_VMEM_RD",
                                         "SQ_INSTS_VMEM_WR", "SQ_INSTS_SMEM") if k in c]
            if insts:
                P("instructions per launch: " + ", ".join(f"{k[9:]} {v:.0f}" for k, v in insts))
    print("\n".join(out))


if __name__ == "__main__":
    main()
