#!/usr/bin/env python3
"""Benchmark of the CSR SpMM / SpMM-like hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--width N] [--op OP]
    python bench.py --sweep            # every workload / width / op, table on stderr
    python bench.py --gradients        # also time the gradient-side entry points
    python bench.py --suite [--vendor] # shape suite at N = 128/256/512, geometric means
    python bench.py --tile-study       # every lanes-per-row x tiles-per-lane kernel shape
    python bench.py --copy-gib 1       # also launch the calibration copy kernel (for --pmc runs)

One "step" is one whole gespmm_csr call (row-initialisation kernel + chunk kernel) on a
seeded synthetic workload that is already resident in HBM.  Prints ONE JSON line on
stdout: throughput as the paper computes it (2 * nnz * N / time, Section V-A), the
byte-model bandwidth of the dominant kernel against the HBM peak ("roofline"), and the
CPU oracle timed on this box's host cores ("cpu_baseline").
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak

# HBM bytes per launch of the chunk kernel, measured with rocprofv3 --pmc (one FETCH_SIZE
# run and one WRITE_SIZE run, each scaled by the calibration copy kernel of known size;
# the summaries are under profiles/).  Key: "<workload>/N<width>/<op>".  Missing = null.
# Each entry: (bytes per CALL summed over the call's main-kernel launches, the launch shape it was measured
# with, the summary under profiles/).  A run whose shape matches none of a workload's entries reports traffic
# null: the number would describe another kernel.
MEASURED_TRAFFIC_BYTES = {
    "large_dense_degree/N64/sum": [
        (11.2728e9, "vec=4 G=16 T=1 S=1024 col_blocks=1 k_parts=8", "chunk_kernel_large_dense_degree_N64_sum.md"),
        (23.0278e9, "vec=4 G=8 T=1 S=512 col_blocks=2 k_parts=1", "chunk_kernel_large_dense_degree_N64_sum_plain_path.md")],
    "general_ops/N128/sum": [(1.05873e9, "vec=4 G=16 T=1 S=256 col_blocks=2 k_parts=1", "chunk_kernel_general_ops_N128_sum.md")],
    "skew_narrow/N8/sum": [(0.618235e9, "vec=4 G=2 T=1 S=1024 col_blocks=1 k_parts=1", "chunk_kernel_skew_narrow_N8_sum.md")],
    "skew_narrow/N32/sum": [(1.18322e9, "vec=4 G=8 T=1 S=256 col_blocks=1 k_parts=1", "chunk_kernel_skew_narrow_N32_sum.md")],
    "width_sweep/N512/sum": [(0.184119e9, "vec=4 G=16 T=1 S=256 col_blocks=8 k_parts=1 row_window=429", "chunk_kernel_width_sweep_N512_sum.md")],
    "uniform_512k_d4/N128/sum": [(1.37096e9, "vec=4 G=16 T=1 S=256 col_blocks=2 k_parts=1", "chunk_kernel_uniform_512k_d4_N128_sum.md")],
}
MEASURED_TRAFFIC_BYTES_BF16 = {
    "large_dense_degree/N64/sum": [
        (6.27652e9, "vec=4 G=16 T=1 S=1024 col_blocks=1 k_parts=4", "chunk_kernel_large_dense_degree_N64_bf16_sum.md")],
}


def plan_string(plan):
    return (f"vec={plan['vec']} G={plan['lanes_per_row']} T={plan['tiles_per_lane']} S={plan['chunk_nnz']} "
            f"col_blocks={plan['col_blocks']} k_parts={plan['k_parts']}"
            + (f" row_window={plan['row_window']}" if plan.get("row_window") else ""))


def measured_traffic(table, key, plan):
    """Bytes per call from the committed counter profile of this workload, or None when there is none or
    when it was measured with another launch shape than today's plan."""
    if key not in table:
        return None
    for nbytes, shape, _ in table[key]:
        if shape == plan_string(plan):
            return nbytes
    print(f"bench.py: the traffic profiles of {key} were measured with {[e[1] for e in table[key]]}, today's plan is "
          f"[{plan_string(plan)}]: traffic reported as null", file=sys.stderr)
    return None


B_ELEM_BYTES = 4                # 2 with --b-dtype bf16 / f16 (B stored in 16 bits; arithmetic and C stay fp32)


def model_bytes(M, N, nnz, has_vals=True):
    """Algorithmic bytes of one SpMM: rowptr + colind + vals + one B-row gather per stored
    entry + C written once (fp32 / int32)."""
    return 4 * (M + 1) + 4 * nnz + (4 * nnz if has_vals else 0) + B_ELEM_BYTES * nnz * N + 4 * M * N


def compulsory_bytes(M, K, N, nnz, has_vals=True):
    """Same, but B counted once (what must cross HBM when caches keep every reuse)."""
    return 4 * (M + 1) + 4 * nnz + (4 * nnz if has_vals else 0) + B_ELEM_BYTES * K * N + 4 * M * N


B_TORCH_DTYPE = None
B_DTYPE_NAME = "f32"
TUNING = None                   # --tuning: per-call overrides handed to every forward call
USE_WORKSPACE = True            # --no-workspace: never hand the forward call a workspace (no K-phased path)
ROW_BOUND = True                # --no-row-bound: do not tell the forward call how long the longest row of the matrix is

TUNING_FIELDS = ("lanes_per_row", "tiles_per_lane", "xcd_remap", "chunk_nnz", "short_len", "k_parts", "longest_row", "wide_addresses")


def case_tuning(w):
    """The --tuning overrides plus what a caller knows about its graph: the length of the longest row (a
    property GNN frameworks keep with the graph, like the degrees; it lets short-row matrices take the
    single-launch whole-row path)."""
    t = dict(zip(TUNING_FIELDS, TUNING)) if TUNING else {}
    if ROW_BOUND and t.get("longest_row", -1) < 0 and w.M:
        t["longest_row"] = int(np.diff(w.rowptr).max())
    return t or None


def forward(gs, tuning=None):
    """The forward call as benchmarked: gespmm_csr_ex with the case's workspace and tuning."""
    def call(rp, ci, v, B, op, C=None, stream=None, workspace=None, profiler=None):
        return gs.gespmm_csr_ex(rp, ci, v, B, op, C=C, workspace=workspace, tuning=tuning, profiler=profiler, stream=stream)
    return call


def cpu_baseline(w, B, op, C_gpu, budget_s=12.0, max_passes=60):
    """The oracle as it stands, all rows of the same workload, repeated for ~budget_s; its result is
    also what the output of the timed GPU run (C_gpu, a host array) is checked against, element by
    element.  Returns (cpu_baseline, parity)."""
    import oracle
    times = []
    t_all = time.perf_counter()
    while len(times) < max_passes and (not times or time.perf_counter() - t_all < budget_s):
        t0 = time.perf_counter()
        Cref, Sabs = oracle.spmm(w.rowptr, w.colind, w.vals, B, op)
        times.append(time.perf_counter() - t0)
    mean = sum(times) / len(times)
    ok, worst = oracle.compare(op, C_gpu, Cref, Sabs)
    parity = {"ok": bool(ok), "elements": int(C_gpu.size), "against": "oracle, every element of the timed run's output"}
    parity["worst_ratio" if op in ("sum", "mean") else "mismatches"] = worst
    return ({"value": 2.0 * w.nnz * B.shape[1] / mean / 1e9, "unit": "GFLOP/s",
             "cores": oracle.max_threads(), "kind": "oracle",
             "sample": f"all {w.M} rows of the same workload, {len(times)} full passes, "
                       f"mean {mean:.3f} s per pass"}, parity)


def time_graph_replay(gs, torch, case, op, steps, calls_per_graph=20):
    """Step time when `calls_per_graph` whole calls are captured into one HIP graph and replayed
    (the way a launch-bound inner loop would be run)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(calls_per_graph):
            forward(gs, case.tuning)(case.rp, case.ci, case.v, case.B, op, C=case.C, workspace=case.work)
    replays = max(1, steps // calls_per_graph)
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(replays):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / (replays * calls_per_graph)


class DeviceCase:
    """One workload at one width, resident on the GPU."""

    def __init__(self, w, N, torch, dev):
        self.w, self.N = w, N
        self.B_host = w.B(N)
        self.rp = torch.from_numpy(w.rowptr).to(dev)
        self.ci = torch.from_numpy(w.colind).to(dev)
        self.v = torch.from_numpy(w.vals).to(dev)
        self.B = torch.from_numpy(self.B_host).to(dev)
        if B_ELEM_BYTES == 2:                            # stored in 16 bits; the host copy keeps the rounded values
            self.B = self.B.to(B_TORCH_DTYPE)
            self.B_host = self.B.float().cpu().numpy()
        self.C = torch.empty((w.M, N), dtype=torch.float32, device=dev)
        self.work = None                                 # workspace of the K-phased path, when the plan wants one
        import paper_2007_03179_amd as gs
        self.tuning = gs.make_tuning(case_tuning(w))      # built once: the calls of the timed loop pass the structure
        need = gs.gespmm_csr_workspace_bytes(w.M, w.K, N, w.nnz, B_DTYPE_NAME, tuning=self.tuning) if USE_WORKSPACE else 0
        if need:
            self.work = torch.empty(need // 4 + 1, dtype=torch.int32, device=dev)
        self.plan = gs.gespmm_plan_ex(w.M, w.K, N, w.nnz, B_DTYPE_NAME, workspace_bytes=need, tuning=self.tuning)

    def time(self, gs, torch, op, steps, warmup, bracket_kernel=True):
        """Time `steps` whole calls.  With bracket_kernel the library also records a HIP event
        pair around every chunk-kernel launch inside the same timed region (needed for the
        roofline figure; the two extra event records per step cost a few microseconds, which
        only matters for microsecond-scale workloads)."""
        stream = torch.cuda.current_stream()
        # the same call of gespmm_csr_ex every step, its arguments marshalled once (the binding's prepared form)
        call = gs.gespmm_csr_prepared(self.rp, self.ci, self.v, self.B, op, C=self.C, workspace=self.work, tuning=self.tuning, stream=stream)
        for _ in range(warmup):
            call()
        torch.cuda.synchronize()
        launches_per_call = self.plan["k_parts"]         # main-kernel launches one call makes
        prof = gs.gespmm_profiler_create(steps * launches_per_call) if bracket_kernel else None
        t0 = time.perf_counter()
        for _ in range(steps):
            call(prof)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        main_ms_sum, launches = gs.gespmm_profiler_finish(prof) if bracket_kernel else (float("nan"), 0)
        w, N = self.w, self.N
        ms = (t1 - t0) * 1e3 / steps
        launch_ms = main_ms_sum / max(launches, 1)       # average duration of one main-kernel launch
        main_ms = launch_ms * launches_per_call          # main-kernel time of one call
        mb = model_bytes(w.M, N, w.nnz)
        return {"workload": w.name, "N": N, "op": op, "ms_per_step": ms, "main_kernel_ms": main_ms,
                "launch_ms": launch_ms, "launches_per_call": launches_per_call,
                "launches_timed": launches, "gflops": 2.0 * w.nnz * N / (ms * 1e-3) / 1e9,
                "model_bytes": mb, "model_GBps_step": mb / (ms * 1e-3) / 1e9,
                "model_GBps_kernel": mb / (main_ms * 1e-3) / 1e9,
                "compulsory_bytes": compulsory_bytes(w.M, w.K, N, w.nnz)}


class Evictor:
    """Pushes 2 GiB through the chip (the library's plain copy kernel, 1 GiB read + 1 GiB written)
    so that the next call starts with neither L2 nor the 256 MB Infinity Cache holding its
    operands; also yields the copy bandwidth this machine reaches, a practical ceiling next to the
    published peak."""

    def __init__(self, gs, torch, dev, gib=1.0):
        n = int(gib * (1 << 30)) // 16 * 4
        self.gs, self.torch, self.bytes = gs, torch, 8 * n
        self.src = torch.ones(n, dtype=torch.float32, device=dev)
        self.dst = torch.empty_like(self.src)

    def __call__(self):
        self.gs.gespmm_calibration_copy(self.src, self.dst)

    def copy_GBps(self, reps=10):
        torch = self.torch
        for _ in range(2):
            self()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(reps):
            self()
        ev[1].record()
        torch.cuda.synchronize()
        return self.bytes * reps / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9


def per_call_times(gs, torch, case, op, calls, before_each=None):
    """Milliseconds of `calls` single calls, each between its own event pair on torch's current
    stream (the one the calls are enqueued on); `before_each` runs outside the pair."""
    stream = torch.cuda.current_stream()
    pairs = []
    for _ in range(calls):
        if before_each is not None:
            before_each()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        forward(gs, case.tuning)(case.rp, case.ci, case.v, case.B, op, C=case.C, stream=stream, workspace=case.work)
        b.record(stream)
        pairs.append((a, b))
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in pairs]


def warm_and_cold(gs, torch, case, op, evictor, calls=30):
    """Per-call minimum and mean, back to back (warm) and after the caches were flushed (cold)."""
    per_call_times(gs, torch, case, op, 3)
    warm = per_call_times(gs, torch, case, op, calls)
    cold = per_call_times(gs, torch, case, op, calls, before_each=evictor)
    return {"warm_min_ms": min(warm), "warm_mean_ms": sum(warm) / len(warm),
            "cold_min_ms": min(cold), "cold_mean_ms": sum(cold) / len(cold), "calls": calls}


def gradient_bytes(kind, M, K, N, nnz):
    """Algorithmic bytes of the gradient-side calls (same counting rules as model_bytes)."""
    walk = 4 * (M + 1) + 8 * nnz                       # rowptr + colind + vals
    if kind == "arg":                                  # the forward bytes plus the positions written
        return model_bytes(M, N, nnz) + 4 * M * N
    if kind == "transposed":                           # zero dB + walk + read dC + one add of N floats per entry
        return 4 * K * N + walk + 4 * M * N + 4 * nnz * N
    if kind == "pool_backward":                        # zero dB + arg, dC, colind[arg], vals[arg], one add per element
        return 4 * K * N + 20 * M * N
    if kind == "csr_transpose_sorted":                 # row ids and weights written, two sort passes of 28 bytes, row starts
        return walk + 8 * nnz + 2 * 28 * nnz + 4 * nnz + 4 * (K + 1)
    if kind == "csr_transpose":                        # counts (read colind, add), scan, walk, write row ids + values
        return 4 * nnz + 4 * nnz + 16 * (K + 1) + walk + 8 * nnz
    if kind == "forward_on_transposed":                # a forward call with the roles of M and K swapped
        return model_bytes(K, N, nnz)
    raise ValueError(kind)


def time_gradients(args, gs, torch, graphgen, dev):
    """Gradient-side entry points on three workloads; table on stderr."""
    rows = []
    for name, N in (("general_ops", 128), ("skew_narrow", 32), ("large_dense_degree", 64)):
        w = graphgen.workload(name, args.scale)
        case = DeviceCase(w, N, torch, dev)
        dC = torch.from_numpy(graphgen.uniform_pm1((w.M, N), 99, stream=N)).to(dev)
        arg = torch.empty((w.M, N), dtype=torch.int32, device=dev)
        dB = torch.empty((w.K, N), dtype=torch.float32, device=dev)
        need_a = gs.gespmm_csr_workspace_bytes(w.M, w.K, N, w.nnz)
        work_a = torch.empty(need_a // 4 + 1, dtype=torch.int32, device=dev) if need_a else None
        calls = {
            # max with positions as the autograd wrapper issues it: with a workspace (the K-phased path where it applies)
            "arg": lambda: gs.gespmm_csr_arg_ex(case.rp, case.ci, case.v, case.B, "max", C=case.C, arg=arg, workspace=work_a),
            "transposed": lambda: gs.gespmm_csr_transposed(case.rp, case.ci, case.v, dC, "sum", w.K, dB=dB),
            "pool_backward": lambda: gs.gespmm_pool_backward(case.ci, case.v, arg, dC, w.K, dB=dB),
        }
        # (the sorted transpose keeps the columns of a transposed row in order, which the K-phased path wants)
        rpT, ciT, vT = gs.gespmm_csr_transpose_sorted(case.rp, case.ci, case.v, w.K)
        calls["csr_transpose"] = lambda: gs.gespmm_csr_transpose(case.rp, case.ci, case.v, w.K)
        calls["csr_transpose_sorted"] = lambda: gs.gespmm_csr_transpose_sorted(case.rp, case.ci, case.v, w.K)
        # the gradient of sum / mean as the autograd wrapper issues it: the forward call on the transposed arrays, with
        # a workspace (the K-phased path where it applies)
        need = gs.gespmm_csr_workspace_bytes(w.K, w.M, N, w.nnz)
        workT = torch.empty(need // 4 + 1, dtype=torch.int32, device=dev) if need else None
        calls["forward_on_transposed"] = lambda: gs.gespmm_csr_ex(rpT, ciT, vT, dC, "sum", C=dB, workspace=workT)
        for kind, call in calls.items():                # "arg" runs first and leaves valid positions behind
            steps = max(10, args.steps // (10 if w.nnz > 5e7 else 1))
            for _ in range(3):
                call()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                call()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
            gb = gradient_bytes(kind, w.M, w.K, N, w.nnz)
            rows.append({"workload": name, "N": N, "kind": kind, "ms_per_call": ms, "model_bytes": gb,
                         "model_GBps": gb / (ms * 1e-3) / 1e9})
            print(f"{name:20s} N={N:4d} {kind:14s} {ms*1e3:10.1f} us  model {gb/1e9:8.3f} GB  "
                  f"{gb/(ms*1e-3)/1e9:8.1f} GB/s ({gb/(ms*1e-3)/1e9/HBM_PEAK_GBPS*100:5.1f}% of HBM peak)",
                  file=sys.stderr, flush=True)
        del case, dC, arg, dB, rpT, ciT, vT
        torch.cuda.empty_cache()
    return rows


def gcn_share(args, gs, torch, graphgen, dev):
    """Share of the aggregation (forward and backward) in a 2-layer GCN and a 2-layer GraphSAGE-pool
    training step on the synthetic graphs, in the spirit of the paper's Table I (which profiles DGL's
    GCN example) and of its GraphSAGE-pool experiment (Section V-E)."""
    from paper_2007_03179_amd import autograd as ag
    rows = []
    for model, name, feats, hidden, classes in (("gcn", "tiny_citation", 1433, 16, 7), ("gcn", "width_sweep", 500, 16, 3),
                                                ("gcn", "general_ops", 128, 256, 40),
                                                ("sage-pool", "width_sweep", 500, 16, 3),
                                                ("sage-pool", "general_ops", 128, 256, 40)):
        w = graphgen.workload(name, args.scale)
        g = ag.CsrGraph(torch.from_numpy(w.rowptr).to(dev), torch.from_numpy(w.colind).to(dev),
                        torch.from_numpy(w.vals).to(dev) if model == "gcn" else None, w.K)
        X = torch.from_numpy(graphgen.uniform_pm1((w.M, feats), 7, stream=feats)).to(dev)
        y = torch.from_numpy((graphgen.uniform_01(w.M, 8) * classes).astype("int64") % classes).to(dev)
        torch.manual_seed(0)
        if model == "gcn":
            l1, l2 = ag.GraphConv(feats, hidden).to(dev), ag.GraphConv(hidden, classes).to(dev)
        else:
            l1, l2 = ag.SageConv(feats, hidden, "pool").to(dev), ag.SageConv(hidden, classes, "pool").to(dev)
        opt = torch.optim.Adam(list(l1.parameters()) + list(l2.parameters()), lr=0.01)

        def train_step():
            opt.zero_grad()
            loss = torch.nn.functional.cross_entropy(l2(g, torch.relu(l1(g, X))), y)
            loss.backward()
            opt.step()

        if model == "gcn":                           # aggregation after the dense layer: widths hidden, classes
            H1 = torch.randn(w.M, hidden, device=dev)
            H2 = torch.randn(w.M, classes, device=dev)
            t1 = g.transposed(False)

            def aggregation_only():                  # the four SpMM calls of one step, same shapes
                for H in (H1, H2):
                    gs.gespmm_csr(g.rowptr, g.colind, g.vals, H, "sum")
                    gs.gespmm_csr(t1[0], t1[1], t1[2], H, "sum")
        else:                                        # pooling over the layer's input width: feats, hidden
            H1 = torch.randn(w.M, feats, device=dev)
            H2 = torch.randn(w.M, hidden, device=dev)

            def aggregation_only():                  # max with positions forward, pooled gradient backward
                for H in (H1, H2):
                    _, arg = gs.gespmm_csr_arg(g.rowptr, g.colind, None, H, "max")
                    gs.gespmm_pool_backward(g.colind, None, arg, H, w.K)

        out = {}
        for label, fn in (("step", train_step), ("aggregation", aggregation_only)):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            n = max(20, args.steps)
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            out[label] = (time.perf_counter() - t0) * 1e3 / n
        rows.append({"model": model, "workload": name, "features": feats, "hidden": hidden, "classes": classes,
                     "train_step_ms": out["step"], "aggregation_ms": out["aggregation"],
                     "aggregation_share": out["aggregation"] / out["step"]})
        print(f"{name:20s} {model} {feats}-{hidden}-{classes}: step {out['step']*1e3:9.1f} us, aggregation (2 forward + 2 backward calls) "
              f"{out['aggregation']*1e3:8.1f} us = {out['aggregation']/out['step']*100:5.1f} % of the step",
              file=sys.stderr, flush=True)
    return rows


def sweep(args, gs, torch, graphgen, dev, evictor):
    """Every workload / width / op of the five configurations; table on stderr."""
    rows = []
    rocsparse = Rocsparse(torch) if args.rocsparse and B_ELEM_BYTES == 4 else None
    for name in graphgen.WORKLOAD_NAMES + graphgen.EXTRA_WORKLOAD_NAMES:
        w = graphgen.workload(name, args.scale)
        print(f"# {w.describe()}", file=sys.stderr, flush=True)
        for N in w.widths:
            case = DeviceCase(w, N, torch, dev)
            for op in w.ops:
                steps = args.steps if w.nnz * N > 5e8 else max(args.steps, 200)
                k = case.time(gs, torch, op, steps, args.warmup)                      # kernel bracketed
                r = case.time(gs, torch, op, steps, args.warmup, bracket_kernel=False)  # clean step time
                r["main_kernel_ms"], r["model_GBps_kernel"] = k["main_kernel_ms"], k["model_GBps_kernel"]
                r["graph_ms_per_step"] = time_graph_replay(gs, torch, case, op, steps) if w.nnz * N < 5e8 else None
                r.update(warm_and_cold(gs, torch, case, op, evictor, calls=20))
                r["rocsparse_ms"], r["rocsparse_alg"] = None, None
                if rocsparse is not None and op == "sum":          # the vendor library has the plain product only
                    case.time(gs, torch, op, 1, 0, bracket_kernel=False)          # case.C: this library's result, to check the vendor's call against
                    r["rocsparse_ms"], r["rocsparse_alg"] = rocsparse.best_time(case, min(steps, 200), case.C)
                rows.append(r)
                print(f"{r['workload']:20s} N={N:4d} {op:5s} step {r['ms_per_step']*1e3:9.1f} us  kernel "
                      f"{r['main_kernel_ms']*1e3:9.1f} us  {r['gflops']:8.1f} GFLOP/s  model "
                      f"{r['model_GBps_step']:8.1f} GB/s ({r['model_GBps_step']/HBM_PEAK_GBPS*100:5.1f}% of HBM peak)"
                      f"  single call min {r['warm_min_ms']*1e3:8.1f} us, caches flushed {r['cold_mean_ms']*1e3:8.1f} us"
                      + (f"  in a HIP graph {r['graph_ms_per_step']*1e3:7.1f} us" if r["graph_ms_per_step"] else "")
                      + (f"  rocsparse_spmm [{r['rocsparse_alg']}] {r['rocsparse_ms']*1e3:8.1f} us ({r['rocsparse_ms']/r['ms_per_step']:4.2f}x)"
                         if r["rocsparse_ms"] else ""), file=sys.stderr, flush=True)
            del case
            torch.cuda.empty_cache()
    return rows


def tile_study(args, gs, torch, graphgen, dev):
    """Lanes per row x column tiles per lane (the second is what the paper calls the coarsening
    factor, Table VI / Fig. 9) at fixed width, on a uniform random graph as in Section V-B and on
    two matrices of different locality; the automatic choice is marked."""
    rows = []
    cases = (("uniform_random_65k", 512), ("general_ops", 128), ("grid3d_64", 128), ("large_dense_degree", 64))
    for name, N in cases:
        w = graphgen.suite_matrix(name) if name in graphgen.SUITE_NAMES else graphgen.workload(name, args.scale)
        global TUNING, USE_WORKSPACE, ROW_BOUND
        saved = TUNING, USE_WORKSPACE, ROW_BOUND
        USE_WORKSPACE = ROW_BOUND = False                # the study is about the plain kernel's shape
        auto = gs.gespmm_plan(w.M, N, w.nnz)
        steps = max(20, min(args.steps, int(2e11 / (w.nnz * N))))
        try:
            for G in (4, 8, 16, 32, 64):
                for T in (1, 2, 4):
                    if 4 * G * T > max(N, 16) * 1 or 4 * G * T < 32:      # no wider than the row, no narrower than 128 bytes
                        continue
                    TUNING = (G, T)
                    try:
                        case = DeviceCase(w, N, torch, dev)
                        case.time(gs, torch, "sum", 5, 2)
                    except gs.GespmmError:                                # this shape is not instantiated
                        continue
                    r = case.time(gs, torch, "sum", steps, 3)
                    p = case.plan
                    is_auto = (G, T) == (auto["lanes_per_row"], auto["tiles_per_lane"])
                    rows.append({"workload": name, "N": N, "lanes_per_row": G, "tiles_per_lane": T,
                                 "col_blocks": p["col_blocks"], "kernel_ms": r["main_kernel_ms"],
                                 "gflops_kernel": 2.0 * w.nnz * N / (r["main_kernel_ms"] * 1e-3) / 1e9, "auto": is_auto})
                    print(f"{name:20s} N={N:4d} lanes/row {G:2d} tiles/lane {T}  column blocks {p['col_blocks']:2d}  kernel "
                          f"{r['main_kernel_ms']*1e3:9.1f} us {rows[-1]['gflops_kernel']:8.1f} GFLOP/s"
                          + ("   <- automatic" if is_auto else ""), file=sys.stderr, flush=True)
                    del case
        finally:
            TUNING, USE_WORKSPACE, ROW_BOUND = saved
        torch.cuda.empty_cache()
    return rows


def gather_ceiling(gs, torch, case, kernel_ms, plan, reps=10):
    """Rate of the plain gather yardstick on this workload's own index stream (colind, in storage order) with
    the kernel's own access shape (rows of one column block of B, the slot's lanes, 16 bytes per lane, eight
    in flight), next to the rows per second the chunk kernel itself gathers.  fp32 with the vector kernels only."""
    w = case.w
    if plan["vec"] != 4:
        return None
    lanes = plan["lanes_per_row"]
    row_bytes = 16 * lanes * plan["tiles_per_lane"]                      # one column block of a row of B
    lanes = min(lanes, 64)
    table = torch.empty((w.K, row_bytes // 4), dtype=torch.float32, device=case.B.device).uniform_(-1, 1)
    try:
        out = gs.gespmm_calibration_gather_shape(table, row_bytes, case.ci, lanes, 16, 8)
    except gs.GespmmError:                                               # no yardstick of that shape
        return None
    for _ in range(2):
        gs.gespmm_calibration_gather_shape(table, row_bytes, case.ci, lanes, 16, 8, out=out)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(reps):
        gs.gespmm_calibration_gather_shape(table, row_bytes, case.ci, lanes, 16, 8, out=out)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / reps
    rows = w.nnz * plan["col_blocks"]
    return {"row_bytes": row_bytes, "gather_only_G_rows_per_s": w.nnz / (ms * 1e-3) / 1e9,
            "chunk_kernel_G_rows_per_s": rows / (kernel_ms * 1e-3) / 1e9,
            "index_order": "colind as stored (the K-phased path visits it part by part; see profiles/gather_ceiling_sweep.md)",
            "table_MB": w.K * row_bytes / 1e6}


def gather_sweep(args, gs, torch, graphgen, dev):
    """What the chip delivers to a plain gather, as a function of the size of the table, the access shape
    (lanes per row x bytes per lane x rows in flight), the cache policy of the loads and the order of the
    index stream: uniform random indices, and the colind streams of workloads 4 and 5 in storage order and
    with the column range cut into parts that are visited one after the other (what the K-phased path does).
    Rates in G rows per second; table on stderr."""
    rows = []
    out = torch.empty(2048 * 256, dtype=torch.float32, device=dev)

    def rate(table, row_bytes, idx, lanes=8, load=16, flight=8, policy=0, reps=5):
        call = lambda: gs.gespmm_calibration_gather_shape(table, row_bytes, idx, lanes, load, flight, policy, out=out)
        call(); call()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(reps):
            call()
        ev[1].record()
        torch.cuda.synchronize()
        return idx.numel() / (ev[0].elapsed_time(ev[1]) / reps * 1e-3) / 1e9

    def note(stream, table_mb, row_bytes, lanes, load, flight, policy, g):
        rows.append({"stream": stream, "table_MB": table_mb, "row_bytes": row_bytes, "lanes": lanes, "load_bytes": load,
                     "in_flight": flight, "policy": ("plain", "bypass L1", "non-temporal")[policy], "G_rows_per_s": g})

    def table_of(nrows, row_bytes):
        return torch.empty(nrows * row_bytes // 4, dtype=torch.float32, device=dev).uniform_(-1, 1)

    def say(text):
        print(text, file=sys.stderr, flush=True)

    torch.manual_seed(0)
    n = 32 << 20
    say("== uniform random indices, rows of 128 bytes, 8 lanes x 16 bytes, 8 in flight: table size x cache policy (G rows/s)")
    for mb in (1, 2, 3, 4, 6, 8, 16, 32, 64, 128, 256, 512, 1024):
        nrows = (mb << 20) // 128
        t, idx = table_of(nrows, 128), torch.randint(0, nrows, (n,), dtype=torch.int32, device=dev)
        res = [rate(t, 128, idx, policy=p) for p in (0, 1, 2)]
        for p, g in enumerate(res):
            note("uniform", mb, 128, 8, 16, 8, p, g)
        say(f"table {mb:5d} MB: plain {res[0]:7.1f}   bypass L1 {res[1]:7.1f}   non-temporal {res[2]:7.1f}")
        del t, idx
    say("== uniform random indices, rows of 128 bytes: lanes x bytes per lane, in flight 2 / 4 / 8 / 16 (G rows/s)")
    for mb in (2, 32, 512):
        nrows = (mb << 20) // 128
        t, idx = table_of(nrows, 128), torch.randint(0, nrows, (n,), dtype=torch.int32, device=dev)
        for lanes, load in ((8, 16), (16, 8), (32, 4), (4, 16), (2, 16), (4, 8), (8, 4)):
            res = [rate(t, 128, idx, lanes, load, f) for f in (2, 4, 8, 16)]
            for f, g in zip((2, 4, 8, 16), res):
                note("uniform", mb, 128, lanes, load, f, 0, g)
            say(f"table {mb:4d} MB, {lanes:2d} lanes x {load:2d} B ({lanes*load:3d} B of the row): " + " ".join(f"{g:7.1f}" for g in res))
        del t, idx
    for row_bytes, lanes in ((256, 16), (512, 32), (1024, 64)):
        nrows = (32 << 20) // row_bytes
        t, idx = table_of(nrows, row_bytes), torch.randint(0, nrows, (n // 2,), dtype=torch.int32, device=dev)
        res = [rate(t, row_bytes, idx, lanes, 16, f) for f in (2, 4, 8)]
        for f, g in zip((2, 4, 8), res):
            note("uniform", 32, row_bytes, lanes, 16, f, 0, g)
        say(f"table   32 MB, rows of {row_bytes:4d} B, {lanes} lanes x 16 B, in flight 2 / 4 / 8: " + " ".join(f"{g:7.1f}" for g in res))
        del t, idx

    def cut(colind, K, parts):                          # the stream with part 0 of the column range first, then part 1, ...
        part = (colind.long() * parts // K).to(torch.int32)
        return colind[torch.sort(part, stable=True).indices].contiguous()

    w = graphgen.workload("large_dense_degree", args.scale)
    ci = torch.from_numpy(w.colind).to(dev)
    say(f"== colind of {w.name} (K = {w.K}, {w.nnz} entries) as the index stream")
    for row_bytes, lanes in ((128, 8), (256, 16)):
        t = table_of(w.K, row_bytes)
        mb = w.K * row_bytes / 1e6
        for policy in ((0, 1, 2) if row_bytes == 128 else (0,)):
            res = [rate(t, row_bytes, ci, lanes, 16, f, policy, reps=3) for f in (4, 8, 16)]
            for f, g in zip((4, 8, 16), res):
                note(f"{w.name} storage order", mb, row_bytes, lanes, 16, f, policy, g)
            say(f"rows of {row_bytes} B ({mb:.1f} MB), storage order, {('plain', 'bypass L1', 'non-temporal')[policy]:12s} in flight 4 / 8 / 16: "
                + " ".join(f"{g:7.1f}" for g in res))
        for parts in (2, 4, 8, 16, 32, 64):
            stream = cut(ci, w.K, parts)
            res = [rate(t, row_bytes, stream, lanes, 16, f, reps=3) for f in (8, 16)]
            for f, g in zip((8, 16), res):
                note(f"{w.name} cut in {parts} parts", mb, row_bytes, lanes, 16, f, 0, g)
            say(f"rows of {row_bytes} B, column range cut in {parts:2d} parts of {mb/parts:6.2f} MB, in flight 8 / 16: "
                + " ".join(f"{g:7.1f}" for g in res))
            del stream
        del t
    del ci
    w = graphgen.workload("skew_narrow", args.scale)
    ci = torch.from_numpy(w.colind).to(dev)
    say(f"== colind of {w.name} (K = {w.K}, {w.nnz} entries) as the index stream")
    for row_bytes, shapes in ((32, ((2, 16), (4, 8), (8, 4))), (128, ((8, 16),))):
        t = table_of(w.K, row_bytes)
        mb = w.K * row_bytes / 1e6
        for lanes, load in shapes:
            res = [rate(t, row_bytes, ci, lanes, load, f) for f in (4, 8, 16)]
            for f, g in zip((4, 8, 16), res):
                note(f"{w.name} storage order", mb, row_bytes, lanes, load, f, 0, g)
            say(f"rows of {row_bytes:3d} B ({mb:.0f} MB), storage order, {lanes} lanes x {load:2d} B, in flight 4 / 8 / 16: "
                + " ".join(f"{g:7.1f}" for g in res))
        for parts in (4, 16, 64):
            g = rate(t, row_bytes, cut(ci, w.K, parts), shapes[0][0], shapes[0][1], 8)
            note(f"{w.name} cut in {parts} parts", mb, row_bytes, shapes[0][0], shapes[0][1], 8, 0, g)
            say(f"rows of {row_bytes:3d} B, column range cut in {parts:2d} parts, in flight 8: {g:7.1f}")
        del t
    return rows


def geomean(xs):
    import math
    xs = [x for x in xs if x]
    return math.exp(sum(math.log(x) for x in xs) / len(xs)) if xs else None


class Rocsparse:
    """The vendor's own CSR x dense product (rocsparse_spmm on librocsparse.so, fp32, row-major B and C), called
    directly.  It plays the part cuSPARSE plays in the paper's Table VII; timed: the compute stage only (buffer
    query and the preprocess stage are done once, outside the timed region)."""
    ALGS = {"default": 0, "csr": 1, "csr_row_split": 4, "csr_nnz_split": 5, "csr_merge_path": 9}

    def __init__(self, torch):
        import ctypes
        self.ct, self.torch = ctypes, torch
        self.lib = ctypes.CDLL("librocsparse.so")
        self.handle = ctypes.c_void_p()
        self.check(self.lib.rocsparse_create_handle(ctypes.byref(self.handle)))
        self.check(self.lib.rocsparse_set_stream(self.handle, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)))
        self.one, self.zero = ctypes.c_float(1.0), ctypes.c_float(0.0)

    def check(self, status):
        if status != 0:
            raise RuntimeError(f"rocsparse status {status}")

    def prepare(self, case, alg):
        """Descriptors, buffer and preprocess stage for one case; returns a function that runs the compute stage."""
        ct, vp = self.ct, self.ct.c_void_p
        w, N = case.w, case.N
        A, B, C = vp(), vp(), vp()
        i32, f32, base0, row_major, csr_op = 2, 151, 0, 0, 111
        out = self.torch.empty((w.M, N), dtype=self.torch.float32, device=case.B.device)
        self.check(self.lib.rocsparse_create_csr_descr(ct.byref(A), ct.c_int64(w.M), ct.c_int64(w.K), ct.c_int64(w.nnz), vp(case.rp.data_ptr()),
                                                       vp(case.ci.data_ptr()), vp(case.v.data_ptr()), i32, i32, base0, f32))
        self.check(self.lib.rocsparse_create_dnmat_descr(ct.byref(B), ct.c_int64(w.K), ct.c_int64(N), ct.c_int64(N), vp(case.B.data_ptr()), f32, row_major))
        self.check(self.lib.rocsparse_create_dnmat_descr(ct.byref(C), ct.c_int64(w.M), ct.c_int64(N), ct.c_int64(N), vp(out.data_ptr()), f32, row_major))
        size = ct.c_size_t(0)

        def stage(which, buffer):
            return self.lib.rocsparse_spmm(self.handle, csr_op, csr_op, ct.byref(self.one), A, B, ct.byref(self.zero), C, f32,
                                           self.ALGS[alg], which, ct.byref(size), buffer)
        self.check(stage(1, None))
        work = self.torch.empty(max(int(size.value), 16), dtype=self.torch.uint8, device=case.B.device)
        self.check(stage(2, vp(work.data_ptr())))
        keep = (A, B, C, work)

        def compute():
            self.check(stage(3, vp(work.data_ptr())))
            return out
        def release():
            self.lib.rocsparse_destroy_spmat_descr(A)
            self.lib.rocsparse_destroy_dnmat_descr(B)
            self.lib.rocsparse_destroy_dnmat_descr(C)
        compute.keep = keep
        compute.release = release
        return compute

    def best_time(self, case, steps, reference):
        """Milliseconds per call of the fastest of the library's CSR algorithms on this case (each checked against
        `reference`, the result of this library, to make sure the call computes the same product)."""
        best, best_alg = None, None
        for alg in self.ALGS:
            try:
                run = self.prepare(case, alg)
                got = run()
                self.torch.cuda.synchronize()
            except RuntimeError:
                continue
            scale = float(reference.abs().max()) + 1e-30
            if float((got - reference).abs().max()) > 1e-3 * scale:
                print(f"# rocsparse {alg}: result differs from this library's, not counted", file=sys.stderr)
                run.release()
                continue
            t0 = time.perf_counter()
            for _ in range(steps):
                run()
            self.torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
            run.release()
            if best is None or ms < best:
                best, best_alg = ms, alg
        return best, best_alg


def shape_suite(args, gs, torch, graphgen, dev):
    """The shape suite at N = 128 / 256 / 512, geometric means per width as in the paper's
    Table VII.  With --vendor the same product through torch's CSR matmul (the vendor sparse
    library underneath) is timed beside it, as context."""
    rows = []
    rocsparse = Rocsparse(torch) if args.rocsparse and B_ELEM_BYTES == 4 else None
    for name in graphgen.SUITE_NAMES:
        w = graphgen.suite_matrix(name)
        d = w.describe()
        print(f"# {name}: M={w.M} nnz={w.nnz} mean row {d['mean_row']:.1f} longest {d['max_row']}",
              file=sys.stderr, flush=True)
        A = None
        if args.vendor:
            A = torch.sparse_csr_tensor(torch.from_numpy(w.rowptr).to(dev), torch.from_numpy(w.colind).to(dev),
                                        torch.from_numpy(w.vals).to(dev), size=(w.M, w.K))
        for N in w.widths:
            case = DeviceCase(w, N, torch, dev)
            steps = max(20, min(args.steps, int(2e11 / (w.nnz * N))))
            r = case.time(gs, torch, "sum", steps, 3, bracket_kernel=False)
            r["vendor_ms"] = None
            r["rocsparse_ms"], r["rocsparse_alg"] = None, None
            if rocsparse is not None:
                r["rocsparse_ms"], r["rocsparse_alg"] = rocsparse.best_time(case, steps, case.C)
            if A is not None:
                for _ in range(2):
                    torch.sparse.mm(A, case.B)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    torch.sparse.mm(A, case.B)
                torch.cuda.synchronize()
                r["vendor_ms"] = (time.perf_counter() - t0) * 1e3 / steps
            rows.append(r)
            print(f"{name:22s} N={N:4d} {r['ms_per_step']*1e3:9.1f} us {r['gflops']:8.1f} GFLOP/s  model "
                  f"{r['model_GBps_step']:8.1f} GB/s ({r['model_GBps_step']/HBM_PEAK_GBPS*100:5.1f}% of HBM peak)"
                  + (f"  vendor CSR matmul {r['vendor_ms']*1e3:9.1f} us ({r['vendor_ms']/r['ms_per_step']:5.2f}x)"
                     if r["vendor_ms"] else "")
                  + (f"  rocsparse_spmm [{r['rocsparse_alg']}] {r['rocsparse_ms']*1e3:9.1f} us ({r['rocsparse_ms']/r['ms_per_step']:5.2f}x)"
                     if r["rocsparse_ms"] else ""), file=sys.stderr, flush=True)
            del case
            torch.cuda.empty_cache()
    summary = []
    for N in (128, 256, 512):
        sel = [r for r in rows if r["N"] == N]
        g = {"N": N, "matrices": len(sel), "geomean_gflops": geomean([r["gflops"] for r in sel]),
             "geomean_model_GBps": geomean([r["model_GBps_step"] for r in sel]),
             "geomean_speedup_over_vendor": geomean([r["vendor_ms"] / r["ms_per_step"] for r in sel if r["vendor_ms"]]),
             "geomean_speedup_over_rocsparse": geomean([r["rocsparse_ms"] / r["ms_per_step"] for r in sel if r["rocsparse_ms"]])}
        summary.append(g)
        print(f"geometric mean N={N:4d}: {g['geomean_gflops']:8.1f} GFLOP/s, model {g['geomean_model_GBps']:8.1f} GB/s"
              + (f", {g['geomean_speedup_over_vendor']:.2f}x the vendor CSR matmul" if g["geomean_speedup_over_vendor"] else "")
              + (f", {g['geomean_speedup_over_rocsparse']:.2f}x rocsparse_spmm" if g["geomean_speedup_over_rocsparse"] else ""),
              file=sys.stderr, flush=True)
    return {"rows": [{k: r[k] for k in ("workload", "N", "ms_per_step", "gflops", "model_GBps_step", "vendor_ms", "rocsparse_ms", "rocsparse_alg")}
                     for r in rows], "summary": summary}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large_dense_degree")
    ap.add_argument("--width", type=int, default=0, help="feature width N (default: the workload's first)")
    ap.add_argument("--op", default="sum")
    ap.add_argument("--mtx", default="", help="benchmark a user-supplied Matrix Market file instead of --workload")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the single-call / flushed-cache / copy-bandwidth figures (used under counter runs)")
    ap.add_argument("--sweep", action="store_true", help="also time every workload/width/op")
    ap.add_argument("--sweep-out", default="", help="write the sweep rows to this JSON file")
    ap.add_argument("--gcn", action="store_true",
                    help="also time a 2-layer GCN training step and the share of the aggregation in it")
    ap.add_argument("--suite", action="store_true",
                    help="also run the shape suite at N = 128/256/512 and print geometric means (Table VII's layout)")
    ap.add_argument("--rocsparse", action="store_true",
                    help="with --suite or --sweep: time rocsparse_spmm (the fastest of its CSR algorithms per case) beside each case")
    ap.add_argument("--vendor", action="store_true",
                    help="with --suite: time torch's CSR matmul (vendor sparse library) beside each case")
    ap.add_argument("--tile-study", action="store_true",
                    help="also time every lanes-per-row x tiles-per-lane kernel shape on four matrices (Table VI's question)")
    ap.add_argument("--gather-sweep", action="store_true",
                    help="also map out the rate of plain gathers over table size, access shape, cache policy and index order")
    ap.add_argument("--gradients", action="store_true",
                    help="also time the gradient-side entry points (positions, transposed, pooling gradient)")
    ap.add_argument("--copy-gib", type=float, default=0.0,
                    help="launch the calibration copy kernel on this many GiB (traffic-counter yardstick)")
    ap.add_argument("--copy-reps", type=int, default=1,
                    help="with --copy-gib: launch the copy this many times on the same buffers (a small buffer copied "
                         "repeatedly stays in the Infinity Cache: tells cache hits from HBM accesses in the counters)")
    ap.add_argument("--b-dtype", default="f32", choices=("f32", "bf16", "f16"),
                    help="storage type of the dense input B (arithmetic and C stay fp32); f32 is the paper's setting")
    ap.add_argument("--tuning", default="",
                    help="lanes_per_row,tiles_per_lane,xcd_remap,chunk_nnz,short_len,k_parts,longest_row,wide_addresses override, e.g. "
                         "--tuning=-1,-1,0,512,16,8 (each -1 = automatic)")
    ap.add_argument("--no-workspace", action="store_true",
                    help="never hand the forward call a workspace: the K-phased path stays off")
    ap.add_argument("--no-row-bound", action="store_true",
                    help="do not pass the length of the matrix's longest row (tuning.longest_row): the whole-row "
                         "path stays off and every call is init_rows + chunk kernel")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import graphgen
    import paper_2007_03179_amd as gs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    global B_ELEM_BYTES, B_TORCH_DTYPE, B_DTYPE_NAME, TUNING, USE_WORKSPACE, ROW_BOUND
    if args.b_dtype != "f32":
        B_ELEM_BYTES, B_TORCH_DTYPE = 2, {"bf16": torch.bfloat16, "f16": torch.float16}[args.b_dtype]
        B_DTYPE_NAME = args.b_dtype
        assert not (args.gradients or args.gcn or args.tile_study or args.vendor), "--b-dtype applies to the forward call only"
    gs.lib()
    dev = torch.device("cuda:0")
    if args.tuning:
        TUNING = tuple(int(x) for x in args.tuning.split(","))
    USE_WORKSPACE = not args.no_workspace
    ROW_BOUND = not args.no_row_bound

    if args.copy_gib > 0:
        n = int(args.copy_gib * (1 << 30)) // 16 * 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(max(1, args.copy_reps)):
            gs.gespmm_calibration_copy(src, dst)
        torch.cuda.synchronize()
        print(f"# calibration copy: {n * 4} bytes read, {n * 4} bytes written, {max(1, args.copy_reps)} time(s)", file=sys.stderr)
        del src, dst

    evictor = None if args.no_cold else Evictor(gs, torch, dev)
    if args.sweep and evictor is None:
        evictor = Evictor(gs, torch, dev)
    sweep_rows = sweep(args, gs, torch, graphgen, dev, evictor) if args.sweep else None
    if sweep_rows is not None and args.sweep_out:
        with open(args.sweep_out, "w") as f:
            json.dump(sweep_rows, f, indent=1)

    grad_rows = time_gradients(args, gs, torch, graphgen, dev) if args.gradients else None
    gcn_rows = gcn_share(args, gs, torch, graphgen, dev) if args.gcn else None
    suite_out = shape_suite(args, gs, torch, graphgen, dev) if args.suite else None
    tile_rows = tile_study(args, gs, torch, graphgen, dev) if args.tile_study else None
    gather_rows = gather_sweep(args, gs, torch, graphgen, dev) if args.gather_sweep else None

    if args.mtx:
        w = graphgen.workload_from_matrix_market(args.mtx)
    elif args.workload in graphgen.SUITE_NAMES:
        w = graphgen.suite_matrix(args.workload)
    else:
        w = graphgen.workload(args.workload, args.scale)
    N = args.width or w.widths[0]
    op = args.op
    case = DeviceCase(w, N, torch, dev)
    # the timed region: K whole calls, nothing else on the stream (this is ms_per_step and value) ...
    clean = case.time(gs, torch, op, args.steps, args.warmup, bracket_kernel=False)
    C_timed = case.C.cpu().numpy()                       # what the last timed step left in C
    # ... then the same K calls again with an event pair around every main-kernel launch, for the roofline
    r = case.time(gs, torch, op, args.steps, 0)
    r["bracketed_ms_per_step"] = r["ms_per_step"]
    for key in ("ms_per_step", "gflops", "model_GBps_step"):
        r[key] = clean[key]
    plan = case.plan
    desc = w.describe()
    achieved = r["model_GBps_kernel"]
    launches = r["launches_per_call"]
    table = MEASURED_TRAFFIC_BYTES if args.b_dtype == "f32" else MEASURED_TRAFFIC_BYTES_BF16 if args.b_dtype == "bf16" else {}
    traffic_call = measured_traffic(table, f"{w.name}/N{N}/{op}", plan)
    out = {
        "metric": "fp32 CSR SpMM GFLOP/s (2*nnz*N) and achieved HBM GB/s vs peak, 1 MI355X",
        "value": r["gflops"], "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: M=K={w.M}, nnz={w.nnz}, N={N}, reduce={op}, seed={w.seed}"
                               + ("" if args.b_dtype == "f32" else f", B stored as {args.b_dtype}"),
                   "csr_hash": desc["csr_hash"], "max_row": desc["max_row"],
                   "kernel": f"chunk_kernel<FoldRows> {plan_string(plan)}"
                             + (f" (K-phased path: {launches} launches per call, workspace "
                                f"{plan['workspace_bytes']} bytes)" if launches > 1 else "")},
        "model_GBps_whole_step": r["model_GBps_step"],
        "frac_of_hbm_peak_whole_step": r["model_GBps_step"] / HBM_PEAK_GBPS,
        "compulsory_bytes": r["compulsory_bytes"],
        # achieved = algorithmic bytes of one launch / average duration of one launch of the dominant kernel.
        # The byte model bills every gathered row of B as memory traffic although the caches serve most of
        # them, so the fraction can exceed 1; frac_compulsory counts B once and is a lower bound on what
        # must cross HBM.  What actually bounds the kernel is the rate at which L2 and fabric deliver
        # 128-byte lines (gather_ceiling below gives the rate of a plain gather of the same rows).
        "roofline": {"bound": "hbm", "bound_note": "byte model; B is served from L2 / Infinity Cache, not HBM",
                     "kernel": "chunk_kernel<FoldRows>", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic_call / launches if traffic_call else None,
                     "algorithmic_bytes_per_launch": r["model_bytes"] / launches,
                     "avg_launch_ms": r["launch_ms"], "launches_timed": r["launches_timed"],
                     "launches_per_call": launches,
                     "frac_compulsory": r["compulsory_bytes"] / (r["main_kernel_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS},
    }
    if traffic_call:
        # what actually crossed the L2 / fabric boundary per second (Infinity Cache hits included)
        out["roofline"]["traffic_GBps"] = traffic_call / (r["main_kernel_ms"] * 1e-3) / 1e9
        out["roofline"]["traffic_over_algorithmic"] = traffic_call / r["model_bytes"]
        out["roofline"]["traffic_over_compulsory"] = traffic_call / r["compulsory_bytes"]
    if args.b_dtype == "f32" and not args.no_cold:
        # a plain gather of the same lines in the same order: the ceiling for the kernel's inner loop
        out["roofline"]["gather_ceiling"] = gather_ceiling(gs, torch, case, r["main_kernel_ms"], plan)
    if evictor is not None:
        # outside the timed region: one call at a time, back to back and with L2 and Infinity Cache
        # flushed before each call, and the plain-copy bandwidth of this machine as a practical ceiling
        out["single_call"] = warm_and_cold(gs, torch, case, op, evictor)
        copy = evictor.copy_GBps()
        out["measured_copy_GBps"] = copy
        out["roofline"]["frac_of_measured_copy"] = achieved / copy
        out["single_call"]["cold_model_GBps"] = r["model_bytes"] / (out["single_call"]["cold_mean_ms"] * 1e-3) / 1e9
        # the same calls captured into one HIP graph and replayed (what a launch-bound inner loop would do)
        out["single_call"]["hip_graph_ms_per_step"] = time_graph_replay(gs, torch, case, op, min(args.steps, 200))
    if evictor is not None and args.b_dtype == "f32" and op == "sum":
        # context, outside the timed region: the vendor library's CSR x dense product on the same operands
        try:
            ms, alg = Rocsparse(torch).best_time(case, min(args.steps, 50), case.C)
            if ms:
                out["vendor_baseline"] = {"library": "rocsparse_spmm", "algorithm": alg, "ms_per_call": ms,
                                          "this_library_speedup": ms / r["ms_per_step"],
                                          "note": "fastest of rocSPARSE's CSR algorithms, compute stage only, result checked against this library's"}
        except (OSError, RuntimeError, AttributeError) as exc:
            print(f"bench.py: no rocSPARSE baseline ({exc})", file=sys.stderr)
    if not args.no_cpu:
        out["cpu_baseline"], out["parity"] = cpu_baseline(w, case.B_host, op, C_timed)
    if sweep_rows is not None:
        out["sweep"] = [{k: row[k] for k in ("workload", "N", "op", "ms_per_step", "gflops", "model_GBps_step",
                                             "warm_min_ms", "cold_mean_ms", "graph_ms_per_step", "rocsparse_ms", "rocsparse_alg")}
                        for row in sweep_rows]
    if grad_rows is not None:
        out["gradients"] = grad_rows
    if gcn_rows is not None:
        out["gcn"] = gcn_rows
    if suite_out is not None:
        out["suite"] = suite_out
    if tile_rows is not None:
        out["tile_study"] = tile_rows
    if gather_rows is not None:
        out["gather_sweep"] = gather_rows
    print(json.dumps(out), flush=True)
    if "parity" in out and not out["parity"]["ok"]:
        print("bench.py: the timed run's output does NOT match the oracle", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
