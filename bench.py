#!/usr/bin/env python3
"""Benchmark of the CSR SpMM / SpMM-like hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--width N] [--op OP]

One "step" is one whole gespmm_csr call (row-initialisation kernel + chunk kernel) on a
seeded synthetic workload that is already resident in HBM.  Prints ONE JSON line:
throughput as the paper computes it (2 * nnz * N / time, Section V-A), the byte-model
bandwidth of the dominant kernel against the HBM peak ("roofline"), and the CPU oracle
timed on this box's host cores ("cpu_baseline").
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak

# HBM bytes per launch of the chunk kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs, scaled by a copy kernel of known size); see profiles/.  None = not measured.
MEASURED_TRAFFIC_BYTES = {}


def model_bytes(M, N, nnz, has_vals=True):
    """Algorithmic bytes of one SpMM: rowptr + colind + vals + one B-row gather per stored
    entry + C written once (fp32 / int32)."""
    return 4 * (M + 1) + 4 * nnz + (4 * nnz if has_vals else 0) + 4 * nnz * N + 4 * M * N


def compulsory_bytes(M, K, N, nnz, has_vals=True):
    """Same, but B counted once (what must cross HBM when caches keep every reuse)."""
    return 4 * (M + 1) + 4 * nnz + (4 * nnz if has_vals else 0) + 4 * K * N + 4 * M * N


def cpu_baseline(w, B, op, budget_s=10.0, max_passes=5):
    """The oracle as it stands, all rows of the same workload, repeated until ~budget_s."""
    import oracle
    times = []
    t_all = time.perf_counter()
    while len(times) < max_passes and (not times or time.perf_counter() - t_all < budget_s):
        t0 = time.perf_counter()
        oracle.spmm(w.rowptr, w.colind, w.vals, B, op)
        times.append(time.perf_counter() - t0)
    mean = sum(times) / len(times)
    return {"value": 2.0 * w.nnz * B.shape[1] / mean / 1e9, "unit": "GFLOP/s",
            "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"all {w.M} rows of the same workload, {len(times)} full pass(es), "
                      f"mean {mean:.3f} s per pass"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large_dense_degree")
    ap.add_argument("--width", type=int, default=0, help="feature width N (default: the workload's first)")
    ap.add_argument("--op", default="sum")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import graphgen
    import paper_2007_03179_amd as gs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    gs.lib()
    w = graphgen.workload(args.workload, args.scale)
    N = args.width or w.widths[0]
    op = args.op
    B = w.B(N)
    dev = torch.device("cuda:0")
    d_rp, d_ci = torch.from_numpy(w.rowptr).to(dev), torch.from_numpy(w.colind).to(dev)
    d_v, d_B = torch.from_numpy(w.vals).to(dev), torch.from_numpy(B).to(dev)
    C = torch.empty((w.M, N), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    for _ in range(args.warmup):
        gs.gespmm_csr(d_rp, d_ci, d_v, d_B, op, C=C, stream=stream)
    torch.cuda.synchronize()
    gs.gespmm_profile_begin(args.steps)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        gs.gespmm_csr(d_rp, d_ci, d_v, d_B, op, C=C, stream=stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    main_ms_sum, launches = gs.gespmm_profile_end()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flops = 2.0 * w.nnz * N
    mbytes = model_bytes(w.M, N, w.nnz)
    main_ms = main_ms_sum / max(launches, 1)
    achieved = mbytes / (main_ms * 1e-3) / 1e9
    plan = gs.gespmm_plan(w.M, N, w.nnz)
    key = f"{w.name}/N{N}/{op}"
    out = {
        "metric": "fp32 CSR SpMM GFLOP/s (2*nnz*N) and achieved HBM GB/s vs peak, 1 MI355X",
        "value": flops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: M=K={w.M}, nnz={w.nnz}, N={N}, reduce={op}, seed={w.seed}",
                   "csr_hash": w.describe()["csr_hash"], "max_row": int(w.describe()["max_row"]),
                   "kernel": f"spmm_chunks vec={plan['vec']} G={plan['lanes_per_row']} "
                             f"T={plan['tiles_per_lane']} S={plan['chunk_nnz']}"},
        "model_GBps_whole_step": mbytes / (ms_per_step * 1e-3) / 1e9,
        "frac_of_hbm_peak_whole_step": mbytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "compulsory_bytes": compulsory_bytes(w.M, w.K, N, w.nnz),
        "roofline": {"bound": "hbm", "kernel": "spmm_chunks", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(key),
                     "algorithmic_bytes_per_launch": mbytes, "avg_launch_ms": main_ms,
                     "launches_timed": launches},
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, B, op)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
