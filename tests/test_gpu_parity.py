"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

sum / mean: |C - Cref| <= 1e-5 * Sabs + 1e-6 per element (Sabs = sum |a||b|, divided by the
row length for mean); max / min: bit-for-bit equal to the oracle rounded once to fp32.
"""
import ctypes
import sys

import numpy as np
import pytest

import graphgen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

OPS = ("sum", "mean", "max", "min")
KERNEL_SHAPES = [(1, 1), (2, 1), (4, 1), (8, 1), (16, 1), (32, 1), (64, 1),
                 (4, 2), (8, 2), (16, 2), (32, 2), (64, 2),
                 (8, 4), (16, 4), (32, 4), (64, 4)]
# (xcd_remap, chunk_nnz, short_len): smallest and largest chunks, slot-per-row mode off / default / always
LAUNCH_VARIANTS = [(0, 16, 0), (1, 64, -1), (1, 256, 16), (1, 1024, 1024), (0, 128, 3)]


@pytest.fixture(scope="module")
def gs():
    import paper_2007_03179_amd as gs
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    gs.lib()                                   # raises if the HIP library was not built
    return gs


# largest error / bound seen for sum and mean in this session: over all cases, and over the
# five workloads at full size only
WORST = {"ratio": 0.0, "case": "", "workload_ratio": 0.0, "workload_case": ""}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(x):
    return None if x is None else torch.from_numpy(np.ascontiguousarray(x)).cuda()


def check(gs, rowptr, colind, vals, B, op, rows=None, label="", entry="gespmm_csr", dB=None, dA=None, tuning=None,
          workspace=None):
    """Run one call on the GPU and compare with the oracle (all rows, or the sampled rows).  With tuning
    overrides or a workspace the call goes through gespmm_csr_ex."""
    say(f"  case {label} op={op} M={len(rowptr) - 1} K={B.shape[0]} N={B.shape[1]} nnz={len(colind)}")
    d_rp, d_ci, d_v = dA if dA is not None else (dev(rowptr), dev(colind), dev(vals))
    d_B = dB if dB is not None else dev(B)
    if tuning is not None or workspace is not None:
        C = gs.gespmm_csr_ex(d_rp, d_ci, d_v, d_B, op, tuning=tuning, workspace=workspace)
    else:
        C = getattr(gs, entry)(d_rp, d_ci, d_v, d_B, op)
    torch.cuda.synchronize()
    C = C.cpu().numpy()
    Cref, Sabs = oracle.spmm(rowptr, colind, vals, B, op, rows=rows)
    got = C if rows is None else C[rows]
    ok, worst = oracle.compare(op, got, Cref, Sabs)
    assert ok, f"{label} {op}: worst={worst}"
    if op in ("sum", "mean") and worst > WORST["ratio"]:
        WORST.update(ratio=worst, case=f"{label} {op} N={B.shape[1]}")
    if op in ("sum", "mean") and label.split(" ")[0] in graphgen.WORKLOAD_NAMES and worst > WORST["workload_ratio"]:
        WORST.update(workload_ratio=worst, workload_case=f"{label} {op} N={B.shape[1]}")
    return C


# ----------------------------------------------------------------------------
@pytest.mark.parametrize("N", [1, 3, 4, 7, 8, 16, 32, 33, 64, 100, 128, 256, 512, 520])
def test_widths_all_ops(gs, N):
    # several chunks, ragged tails, empty rows, one row spanning ~12 chunks, M != K
    rp, ci, v = graphgen.random_csr(700, 500, 9.0, 100 + N, empty_frac=0.1, long_rows=((350, 3000),),
                                    duplicates=True)
    B = graphgen.random_dense(500, N, N)
    for op in OPS:
        check(gs, rp, ci, v, B, op, label=f"widths N={N}")


def test_unsorted_duplicate_columns_and_null_vals(gs):
    rp, ci, v = graphgen.random_csr(400, 300, 12.0, 7, empty_frac=0.2, duplicates=True, sort_cols=False)
    B = graphgen.random_dense(300, 32, 7)
    for op in OPS:
        check(gs, rp, ci, v, B, op, label="unsorted+dups")
        check(gs, rp, ci, None, B, op, label="vals=NULL")


def test_degenerate_shapes(gs):
    B = graphgen.random_dense(5, 8, 1)
    # all rows empty (nnz == 0): C must be all zeros for every op
    rp = np.zeros(4, dtype=np.int32)
    ci = np.zeros(0, dtype=np.int32)
    v = np.zeros(0, dtype=np.float32)
    for op in OPS:
        C = check(gs, rp, ci, v, B, op, label="nnz=0")
        assert not C.any()
    # one row, one entry
    rp, ci, v = np.array([0, 1], np.int32), np.array([4], np.int32), np.array([-2.5], np.float32)
    for op in OPS:
        check(gs, rp, ci, v, B, op, label="1x1")
    # leading and trailing empty rows around a single dense row longer than several chunks
    n = 1000
    rp = np.array([0, 0, 0, n, n, n], dtype=np.int32)
    rng = np.random.default_rng(3)
    ci = rng.integers(0, 5, size=n).astype(np.int32)
    v = (rng.random(n) - 0.5).astype(np.float32)
    for op in OPS:
        check(gs, rp, ci, v, B, op, label="empty-around-long")
    # a chunk border that falls exactly on a row border (256 entries per chunk)
    rp = np.array([0, 256, 512, 700], dtype=np.int32)
    ci = rng.integers(0, 5, size=700).astype(np.int32)
    v = (rng.random(700) - 0.5).astype(np.float32)
    for op in OPS:
        check(gs, rp, ci, v, B, op, label="row-border==chunk-border")
    # many more rows than entries: long runs of empty rows inside and after the last chunk
    rp, ci, v = graphgen.random_csr(5000, 64, 1.0, 17, empty_frac=0.97)
    B = graphgen.random_dense(64, 16, 17)
    for op in OPS:
        check(gs, rp, ci, v, B, op, label="mostly-empty")


def test_signed_zero_rule_on_gpu(gs):
    # +0 must win max and lose min, whichever comes first and wherever the row is split
    for n in (2, 600):
        ci = np.tile(np.array([0, 1], dtype=np.int32), n // 2)
        rp = np.array([0, n, 2 * n], dtype=np.int32)
        ci = np.concatenate([ci, ci[::-1]]).astype(np.int32)
        v = np.ones(2 * n, dtype=np.float32)
        B = np.array([[-0.0] * 4, [0.0] * 4], dtype=np.float32)
        hi = check(gs, rp, ci, v, B, "max", label=f"signed-zero n={n}")
        lo = check(gs, rp, ci, v, B, "min", label=f"signed-zero n={n}")
        assert not np.signbit(hi).any() and np.signbit(lo).all()


def test_closed_form_long_row(gs):
    # one row of 100000 ones against B[k, j] = k * (j + 1): hundreds of chunks combined by atomics
    n, N = 100_000, 8
    rp = np.array([0, n, n], dtype=np.int32)
    ci = np.arange(n, dtype=np.int32)
    B = (np.arange(n, dtype=np.float64)[:, None] * (np.arange(N) + 1.0)[None, :]).astype(np.float32)
    for op in OPS:
        C = check(gs, rp, ci, None, B, op, label="closed-form")
        if op == "max":
            assert np.array_equal(C[0], (n - 1) * (np.arange(N) + 1.0).astype(np.float32))
        if op == "min":
            assert not C[0].any()
        assert not C[1].any()


@pytest.mark.parametrize("vec_n", [(4, 72), (1, 37)])
def test_every_kernel_shape(gs, vec_n):
    vec, N = vec_n
    rp, ci, v = graphgen.random_csr(300, 260, 7.0, 55, empty_frac=0.1, long_rows=((11, 900), (12, 300)))
    B = graphgen.random_dense(260, N, 55)
    dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
    for G, T in KERNEL_SHAPES:
        for remap, chunk, short in LAUNCH_VARIANTS:
            tuning = (G, T, remap, chunk, short)
            plan = gs.gespmm_plan_ex(300, 260, N, len(ci), tuning=tuning)
            assert plan["vec"] == vec and plan["lanes_per_row"] == G and plan["tiles_per_lane"] == T
            assert plan["chunk_nnz"] == chunk and plan["xcd_remap"] == remap
            for op in ("sum", "mean", "max", "min"):
                check(gs, rp, ci, v, B, op, dA=dA, dB=dB, tuning=tuning,
                      label=f"G={G} T={T} remap={remap} S={chunk} short={short}")


@pytest.mark.parametrize("whole_rows", [False, True])
def test_xcd_runs_cover_every_chunk(gs, whole_rows):
    """Workgroups are dealt to the XCDs in runs (plan.xcd_remap > 1): every run length, on grids that are a multiple
    of eight runs, one short of it, one beyond it and shorter than one period, must still visit every chunk once."""
    rp, ci, v = graphgen.random_csr(4000, 900, 9.0, 61, empty_frac=0.05, long_rows=((17, 700),))
    B = graphgen.random_dense(900, 32, 61)
    dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
    longest = int(np.diff(rp).max())
    for chunk in (16, 64, 256):                       # about 2500, 630 and 160 workgroups
        for runs in (2, 3, 5, 16, 32, 79, 4096):
            tuning = dict(xcd_remap=runs, chunk_nnz=chunk, longest_row=longest if whole_rows else -1)
            plan = gs.gespmm_plan_ex(4000, 900, 32, len(ci), tuning=tuning)
            assert plan["xcd_remap"] == runs and (plan["row_window"] > 0) == (whole_rows and chunk + longest <= 1984)
            for op in ("sum", "max"):
                check(gs, rp, ci, v, B, op, dA=dA, dB=dB, tuning=tuning, label=f"runs={runs} S={chunk} whole={whole_rows}")


def test_unaligned_buffers(gs):
    """B (and, below, C) at addresses that are only 4-byte aligned take one column per lane; guard values around C."""
    rp, ci, v = graphgen.random_csr(200, 150, 8.0, 9, empty_frac=0.1, long_rows=((5, 700),))
    B = graphgen.random_dense(150, 64, 9)
    d_rp, d_ci, d_v = dev(rp), dev(ci), dev(v)
    raw = torch.empty(150 * 64 + 1, dtype=torch.float32, device="cuda")
    d_B = raw[1:].view(150, 64)
    d_B.copy_(torch.from_numpy(B))
    assert d_B.data_ptr() % 16 != 0
    for op in OPS:
        say(f"  case unaligned op={op}")
        C = gs.gespmm_csr(d_rp, d_ci, d_v, d_B, op)
        torch.cuda.synchronize()
        ok, worst = oracle.compare(op, C.cpu().numpy(), *oracle.spmm(rp, ci, v, B, op))
        assert ok, worst
        raw_c = torch.full((200 * 64 + 3,), 7.0, dtype=torch.float32, device="cuda")      # C two floats off, guards around it
        d_C = raw_c[2:-1].view(200, 64)
        for tuning in (None, dict(longest_row=700, chunk_nnz=1024), dict(chunk_nnz=16)):
            gs.gespmm_csr_ex(d_rp, d_ci, d_v, d_B, op, C=d_C, tuning=tuning)
            torch.cuda.synchronize()
            ok, worst = oracle.compare(op, d_C.cpu().numpy(), *oracle.spmm(rp, ci, v, B, op))
            assert ok, worst
            assert raw_c[0].item() == 7.0 and raw_c[1].item() == 7.0 and raw_c[-1].item() == 7.0


@pytest.mark.parametrize("N", [5, 6, 7, 9, 33, 65, 127, 130, 250, 1001])
def test_widths_that_are_no_multiple_of_four(gs, N):
    """One column per lane: all four reductions, rows split among chunks, the whole-row path, forced shapes (a forced
    number of parts is ignored: no phased kernel for these widths), guard values around an unaligned C."""
    rp, ci, v = graphgen.random_csr(700, 500, 12.0, 400 + N, empty_frac=0.1, long_rows=((3, 3000), (699, 1500), (350, 0)),
                                    duplicates=True, sort_cols=False)
    B = graphgen.random_dense(500, N, 400 + N)
    dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
    raw_c = torch.full((700 * N + 8,), -3.0, dtype=torch.float32, device="cuda")
    d_C = raw_c[3:-5].view(700, N)                    # (and only 4-byte aligned)
    ws = torch.empty(1 << 20, dtype=torch.int32, device="cuda")
    variants = [dict(), dict(chunk_nnz=16), dict(chunk_nnz=1024, short_len=0), dict(longest_row=100, chunk_nnz=256),
                dict(k_parts=3), dict(k_parts=2, lanes_per_row=8, tiles_per_lane=2), dict(k_parts=5, lanes_per_row=16, tiles_per_lane=2, chunk_nnz=64),
                dict(lanes_per_row=4, tiles_per_lane=2), dict(lanes_per_row=64, tiles_per_lane=4)]
    for tuning in variants:
        for op in OPS:
            say(f"  case ragged N={N} {tuning} op={op}")
            gs.gespmm_csr_ex(*dA, dB, op, C=d_C, tuning=tuning, workspace=ws if "k_parts" in tuning else None)
            torch.cuda.synchronize()
            ok, worst = oracle.compare(op, d_C.cpu().numpy(), *oracle.spmm(rp, ci, v, B, op))
            assert ok, (tuning, op, worst)
            assert (raw_c[:3] == -3.0).all().item() and (raw_c[-5:] == -3.0).all().item()
            if op in ("max", "min"):
                assert np.array_equal(d_C.cpu().numpy().view(np.uint32), oracle.spmm(rp, ci, v, B, op)[0].astype(np.float32).view(np.uint32))


def test_simple_entry_point_and_side_stream(gs):
    rp, ci, v = graphgen.random_csr(500, 400, 10.0, 21, empty_frac=0.05, long_rows=((0, 2000),))
    B = graphgen.random_dense(400, 64, 21)
    for op in OPS:
        check(gs, rp, ci, v, B, op, label="simple", entry="gespmm_csr_simple")
    d_rp, d_ci, d_v, d_B = dev(rp), dev(ci), dev(v), dev(B)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    say("  case side-stream")
    with torch.cuda.stream(side):
        C = gs.gespmm_csr(d_rp, d_ci, d_v, d_B, "sum", stream=side)
    side.synchronize()
    ok, worst = oracle.compare("sum", C.cpu().numpy(), *oracle.spmm(rp, ci, v, B, "sum"))
    assert ok, worst


@pytest.mark.parametrize("seed", range(12))
def test_seeded_random_shapes(gs, seed):
    """Five random problems per seed: sizes, widths (odd ones too), row-length mix, empty rows, duplicates,
    hub rows and NULL values all drawn from the seed; forward call and value+position call."""
    rng = np.random.default_rng(1000 + seed)
    for _ in range(5):
        M, K = int(rng.integers(1, 3000)), int(rng.integers(1, 3000))
        N = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 20, 31, 32, 36, 64, 96, 100, 128, 130, 200, 256, 260, 384, 512, 640]))
        mean_len = float(rng.choice([0.3, 1.0, 3.0, 10.0, 40.0]))
        long_rows = tuple((int(rng.integers(0, M)), int(rng.integers(300, 5000))) for _ in range(int(rng.integers(0, 3))))
        rp, ci, v = graphgen.random_csr(M, K, mean_len, int(rng.integers(1 << 30)), empty_frac=float(rng.choice([0, 0.2, 0.7])),
                                        duplicates=True, sort_cols=bool(rng.integers(2)), long_rows=long_rows)
        if rng.integers(4) == 0:
            v = None
        B = graphgen.random_dense(K, N, int(rng.integers(1 << 30)))
        op = str(rng.choice(OPS))
        C_narrow = check(gs, rp, ci, v, B, op, label=f"random seed={seed}")
        # the same call with 64-bit addresses for its gathers instead of buffer offsets: max / min the same bits
        C_wide = check(gs, rp, ci, v, B, op, label=f"random seed={seed} wide", tuning=dict(wide_addresses=1))
        if op in ("max", "min"):
            assert np.array_equal(C_narrow.view(np.uint32), C_wide.view(np.uint32))
        if op in ("max", "min"):
            C, arg = gs.gespmm_csr_arg(dev(rp), dev(ci), dev(v), dev(B), op)
            torch.cuda.synchronize()
            Cref, aref = oracle.spmm_arg(rp, ci, v, B, op)
            assert np.array_equal(C.cpu().numpy().view(np.uint32), Cref.astype(np.float32).view(np.uint32))
            assert np.array_equal(arg.cpu().numpy(), aref)


def test_prepared_call_is_the_same_call(gs):
    """gespmm_csr_prepared marshals the arguments of gespmm_csr_ex once; every call of the object is that C call."""
    rp, ci, v = graphgen.random_csr(800, 600, 9.0, 12, empty_frac=0.1, long_rows=((3, 900),))
    B = graphgen.random_dense(600, 40, 12)
    d = dev(rp), dev(ci), dev(v), dev(B)
    for op in OPS:
        for tuning in (None, dict(longest_row=int(np.diff(rp).max())), gs.make_tuning(dict(chunk_nnz=64))):
            C = torch.full((800, 40), float("nan"), dtype=torch.float32, device="cuda")
            call = gs.gespmm_csr_prepared(*d, op, C=C, tuning=tuning)
            for _ in range(3):
                out = call()
            torch.cuda.synchronize()
            assert out is C
            ok, worst = oracle.compare(op, C.cpu().numpy(), *oracle.spmm(rp, ci, v, B, op))
            assert ok, (op, worst)
    prof = gs.gespmm_profiler_create(2)
    call = gs.gespmm_csr_prepared(*d, "sum")
    call(prof)
    call(prof)
    ms, launches = gs.gespmm_profiler_finish(prof)
    assert launches == 2 and ms > 0


def test_calls_on_two_streams_at_once_do_not_disturb_each_other(gs):
    """The library keeps no state between calls and owns no scratch memory: calls in flight on two streams
    (different matrices, different ops, enqueued alternately) both give the oracle's result."""
    cases = []
    for seed, (M, K, N), op in ((31, (3000, 2500, 64), "sum"), (32, (2000, 3500, 128), "max")):
        rp, ci, v = graphgen.random_csr(M, K, 12.0, seed, empty_frac=0.05, long_rows=((7, 4000),))
        B = graphgen.random_dense(K, N, seed)
        cases.append((rp, ci, v, B, op, (dev(rp), dev(ci), dev(v), dev(B)),
                      torch.empty((M, N), dtype=torch.float32, device="cuda"), torch.cuda.Stream()))
    torch.cuda.synchronize()
    say("  case two-streams")
    for _ in range(20):
        for rp, ci, v, B, op, d, C, stream in cases:
            gs.gespmm_csr(*d, op, C=C, stream=stream)
    torch.cuda.synchronize()
    for rp, ci, v, B, op, d, C, stream in cases:
        ok, worst = oracle.compare(op, C.cpu().numpy(), *oracle.spmm(rp, ci, v, B, op))
        assert ok, (op, worst)


def test_results_do_not_depend_on_what_C_held(gs):
    rp, ci, v = graphgen.random_csr(300, 200, 5.0, 33, empty_frac=0.3, long_rows=((5, 800),))
    B = graphgen.random_dense(200, 16, 33)
    d = dev(rp), dev(ci), dev(v), dev(B)
    for op in OPS:
        say(f"  case dirty-C op={op}")
        C = torch.full((300, 16), float("nan"), dtype=torch.float32, device="cuda")
        for fill in (float("nan"), 1e30, -1e30):
            C.fill_(fill)
            gs.gespmm_csr(*d, op, C=C)
            torch.cuda.synchronize()
            ok, worst = oracle.compare(op, C.cpu().numpy(), *oracle.spmm(rp, ci, v, B, op))
            assert ok, (op, fill, worst)


def test_profile_brackets_main_kernel(gs):
    rp, ci, v = graphgen.random_csr(2000, 2000, 20.0, 2)
    d = dev(rp), dev(ci), dev(v), dev(graphgen.random_dense(2000, 64, 2))
    prof = gs.gespmm_profiler_create(3)
    for _ in range(5):
        gs.gespmm_csr_ex(*d, "sum", profiler=prof)
    ms, n = gs.gespmm_profiler_finish(prof)
    assert n == 3 and 0 < ms < 1000
    # the K-phased path brackets every one of its launches
    prof = gs.gespmm_profiler_create(10)
    work = torch.empty(gs.gespmm_csr_workspace_bytes(2000, 2000, 64, len(ci), tuning={"k_parts": 4}) // 4,
                       dtype=torch.int32, device="cuda")
    gs.gespmm_csr_ex(*d, "sum", workspace=work, tuning={"k_parts": 4}, profiler=prof)
    ms, n = gs.gespmm_profiler_finish(prof)
    assert n == 4 and 0 < ms < 1000


@pytest.mark.parametrize("floats", [4, 1020, 4 * 256 * 8192 * 4 + 4 * 77, 4 * 256 * 8192 * 9 + 4])
def test_calibration_copy_is_a_copy(gs, floats):
    src = torch.arange(floats, dtype=torch.int32, device="cuda").view(torch.float32)
    dst = torch.full((floats + 8,), -1.0, device="cuda")
    gs.gespmm_calibration_copy(src, dst[4:4 + floats])
    torch.cuda.synchronize()
    assert torch.equal(dst[4:4 + floats].view(torch.int32), src.view(torch.int32))
    assert bool((dst[:4] == -1).all()) and bool((dst[-4:] == -1).all())


def test_calibration_gather_reads_every_requested_line(gs):
    lines, n = 5000, 123_457
    table = torch.arange(lines, dtype=torch.float32, device="cuda").repeat_interleave(32).view(lines, 32).contiguous()
    idx = torch.from_numpy(np.random.default_rng(5).integers(0, lines, n).astype(np.int32)).cuda()
    out = gs.gespmm_calibration_gather(table, idx)
    torch.cuda.synchronize()
    assert abs(float(out.double().sum()) - 32.0 * float(idx.double().sum())) <= 1e-6 * 32.0 * float(idx.double().sum())
    with pytest.raises(gs.GespmmError):                       # scratch output too small
        gs.gespmm_calibration_gather(table, idx, out=torch.empty(16, device="cuda"))


def _workspace(gs, M, K, N, nnz, tuning, dtype="f32"):
    need = gs.gespmm_csr_workspace_bytes(M, K, N, nnz, dtype, tuning=tuning)
    assert need > 0
    return torch.full((need // 4 + 1,), -12345, dtype=torch.int32, device="cuda")


@pytest.mark.parametrize("N", [4, 32, 64, 72, 128, 260])
def test_k_phased_path_forced_on_small_matrices(gs, N):
    """The path that runs the operation once per part of the column range, forced on matrices of a few
    chunks: sorted columns (what it is made for), unsorted columns with repeats (the pieces still
    partition every row), NULL values, empty rows, rows much longer than a chunk, M != K, parts that hold
    no entry at all, more parts than columns per row; every op, every slot width it has kernels for."""
    cases = (graphgen.random_csr(700, 500, 9.0, 300 + N, empty_frac=0.1, long_rows=((350, 3000),)),
             graphgen.random_csr(400, 900, 40.0, 301 + N, empty_frac=0.05, duplicates=True, sort_cols=False,
                                 long_rows=((7, 2000), (8, 1))),
             graphgen.random_csr(50, 30, 2.0, 302 + N, empty_frac=0.5))
    for which, (rp, ci, v) in enumerate(cases):
        M, K = len(rp) - 1, (500, 900, 30)[which]
        if which == 0:                                           # entries only in the lower half of the columns
            ci = (ci // 2).astype(np.int32)
        B = graphgen.random_dense(K, N, N + which)
        dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
        for parts, G, chunk in ((2, -1, -1), (3, 8, 64), (7, 16, 256), (64, 32, 16), (5, 16, 1024)):
            if G > 0 and 4 * G > max(N, 32) * 2:
                G = -1
            tuning = dict(k_parts=parts, lanes_per_row=G, chunk_nnz=chunk)
            plan = gs.gespmm_plan_ex(M, K, N, len(ci), workspace_bytes=1 << 30, tuning=tuning)
            assert plan["k_parts"] == min(parts, K) and plan["workspace_bytes"] > 0
            work = _workspace(gs, M, K, N, len(ci), tuning)
            for op in OPS:
                check(gs, rp, ci, v, B, op, dA=dA, dB=dB, tuning=tuning, workspace=work,
                      label=f"phased case={which} parts={parts} G={G} S={chunk}")
            check(gs, rp, ci, None, B, "sum", dA=(dA[0], dA[1], None), dB=dB, tuning=tuning, workspace=work,
                  label=f"phased vals=NULL case={which} parts={parts}")


def test_k_phased_path_arguments(gs):
    rp, ci, v = graphgen.random_csr(300, 200, 20.0, 5)
    d = dev(rp), dev(ci), dev(v), dev(graphgen.random_dense(200, 64, 5))
    with pytest.raises(gs.GespmmError) as e:                     # phases forced, nowhere to put their row starts
        gs.gespmm_csr_ex(*d, "sum", tuning={"k_parts": 4})
    assert e.value.status == 4
    small = torch.empty(16, dtype=torch.int32, device="cuda")
    with pytest.raises(gs.GespmmError) as e:
        gs.gespmm_csr_ex(*d, "sum", tuning={"k_parts": 4}, workspace=small)
    assert e.value.status == 4
    # automatic choice on a small problem: the workspace is ignored, the plain path runs
    assert gs.gespmm_plan_ex(300, 200, 64, len(ci), workspace_bytes=1 << 30)["k_parts"] == 1
    C = gs.gespmm_csr_ex(*d, "sum", workspace=small)
    torch.cuda.synchronize()
    ok, worst = oracle.compare("sum", C.cpu().numpy(), *oracle.spmm(rp, ci, v, graphgen.random_dense(200, 64, 5), "sum"))
    assert ok, worst
    # N not a multiple of 4: no phased kernel, the plain path runs whatever is forced
    assert gs.gespmm_plan_ex(300, 200, 30, len(ci), workspace_bytes=1 << 30, tuning={"k_parts": 4})["k_parts"] == 1


def test_non_finite_features_reach_exactly_the_rows_that_use_them(gs):
    """Algorithm 1 in IEEE arithmetic: an infinite element of B makes the outputs of the rows that store an
    entry for it infinite (NaN where +inf and -inf meet or a stored zero multiplies it), and no other."""
    rp, ci, v = graphgen.random_csr(600, 400, 9.0, 88, empty_frac=0.1, long_rows=((30, 2500),))
    v = np.abs(v) + 0.5                                           # positive weights: inf stays inf
    B = graphgen.random_dense(400, 40, 88)
    B[17, :] = np.inf
    B[200, 3] = -np.inf
    B[399, 39] = np.inf
    for op in OPS:
        C = check(gs, rp, ci, v, B, op, label="inf in B")
        touched = np.zeros(600, dtype=bool)
        touched[np.repeat(np.arange(600), np.diff(rp))[np.isin(ci, (17, 200, 399))]] = True
        assert np.isfinite(C[~touched]).all()
        assert not np.isfinite(C[touched]).all()
    v2 = v.copy()
    v2[rp[30]:rp[30] + 5] = 0.0                                   # stored zeros: 0 * inf = NaN where they meet row 17 of B
    ci2 = ci.copy()
    ci2[rp[30]] = 17
    check(gs, rp, ci2, v2, B, "sum", label="0 * inf")


# --------------------------------------------------------- whole-row path --
@pytest.mark.parametrize("N", [1, 4, 7, 16, 32, 64, 72, 128, 256, 260, 512])
def test_whole_row_path_on_small_matrices(gs, N):
    """The single-launch path chosen through tuning.longest_row: every row is written once by the chunk that
    owns its first item.  True bounds and bounds that understate the longest row (then the row is walked in
    windows), runs of empty rows inside, before and after the entries, rows far longer than a chunk, unsorted
    repeated columns, NULL values, every op, every chunk size and slot width, and a C that held garbage."""
    cases = (graphgen.random_csr(700, 500, 9.0, 500 + N, empty_frac=0.1, long_rows=((350, 900),)),
             graphgen.random_csr(400, 900, 40.0, 501 + N, empty_frac=0.05, duplicates=True, sort_cols=False,
                                 long_rows=((7, 3000), (8, 1), (399, 1500))),
             graphgen.random_csr(3000, 64, 1.0, 502 + N, empty_frac=0.9),
             graphgen.random_csr(300, 300, 5.0, 503 + N))
    for which, (rp, ci, v) in enumerate(cases):
        M, K = len(rp) - 1, (500, 900, 64, 300)[which]
        longest = int(np.diff(rp).max())
        B = graphgen.random_dense(K, N, N + which)
        dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
        for hint, G, chunk, short_len in ((longest, -1, -1, -1), (1, -1, 16, 0), (longest, 64, 64, -1), (70, 4, 256, 1024),
                                          (3, 1, 1024, 3), (200, 32, 128, -1), (1024, 16, 512, -1)):
            tuning = dict(longest_row=hint, lanes_per_row=G, chunk_nnz=chunk, short_len=short_len)
            plan = gs.gespmm_plan_ex(M, K, N, len(ci), tuning=tuning)
            if hint == longest and longest > 1024:
                assert plan["row_window"] == 0                  # too long for the path: the two-launch path runs
            else:
                assert plan["row_window"] >= plan["chunk_nnz"] + hint, plan
            for op in OPS:
                check(gs, rp, ci, v, B, op, dA=dA, dB=dB, tuning=tuning,
                      label=f"whole-row case={which} hint={hint} longest={longest} G={G} S={chunk}")
            check(gs, rp, ci, None, B, "mean", dA=(dA[0], dA[1], None), dB=dB, tuning=tuning,
                  label=f"whole-row vals=NULL case={which} hint={hint}")


def test_whole_row_path_degenerate_and_deterministic(gs):
    B = graphgen.random_dense(5, 8, 1)
    hint = dict(longest_row=1000)
    rp = np.zeros(4, dtype=np.int32)                                # no entries at all: zeros from the one launch
    for op in OPS:
        C = check(gs, rp, np.zeros(0, np.int32), np.zeros(0, np.float32), B, op, tuning=hint, label="whole-row nnz=0")
        assert not C.any()
    rp = np.array([0, 0, 0, 1000, 1000, 1000], dtype=np.int32)      # empty rows around one long row
    rng = np.random.default_rng(3)
    ci = rng.integers(0, 5, size=1000).astype(np.int32)
    v = (rng.random(1000) - 0.5).astype(np.float32)
    for op in OPS:
        check(gs, rp, ci, v, B, op, tuning=hint, label="whole-row empty-around-long")
        check(gs, rp, ci, v, B, op, tuning=dict(longest_row=5, chunk_nnz=64), label="whole-row windows")
    # nothing is combined by atomics: two runs give the same bits, also for sum, whatever C held before
    rp, ci, v = graphgen.random_csr(5000, 4000, 12.0, 9, empty_frac=0.05, long_rows=((77, 800),))
    Bn = graphgen.random_dense(4000, 64, 9)
    d = dev(rp), dev(ci), dev(v), dev(Bn)
    tuning = dict(longest_row=int(np.diff(rp).max()))
    assert gs.gespmm_plan_ex(5000, 4000, 64, len(ci), tuning=tuning)["row_window"] > 0
    first = gs.gespmm_csr_ex(*d, "sum", tuning=tuning, C=torch.full((5000, 64), float("nan"), device="cuda"))
    second = gs.gespmm_csr_ex(*d, "sum", tuning=tuning, C=torch.full((5000, 64), 7.0, device="cuda"))
    torch.cuda.synchronize()
    assert torch.equal(first, second)
    ok, worst = oracle.compare("sum", first.cpu().numpy(), *oracle.spmm(rp, ci, v, Bn, "sum"))
    assert ok, worst


@pytest.mark.parametrize("which", [0, 1, 2, "uniform_random_65k"])
def test_whole_row_path_on_workloads(gs, which):
    """The workloads whose longest row is short enough, full size, every element, with the true bound."""
    w = graphgen.workload(which)
    longest = int(np.diff(w.rowptr).max())
    tuning = dict(longest_row=longest)
    dA = dev(w.rowptr), dev(w.colind), dev(w.vals)
    for N in w.widths:
        plan = gs.gespmm_plan_ex(w.M, w.K, N, w.nnz, tuning=tuning)
        say(f"  {w.name} N={N} longest row {longest}: row_window {plan['row_window']} S {plan['chunk_nnz']}")
        B = w.B(N)
        dB = dev(B)
        for op in w.ops:
            check(gs, w.rowptr, w.colind, w.vals, B, op, label=w.name + " whole-row", dA=dA, dB=dB, tuning=tuning)


# ------------------------------------------------------------ the workloads --
@pytest.mark.parametrize("which", [0, 1, 2, "uniform_random_65k"])
def test_workload_full_size_every_element(gs, which):
    w = graphgen.workload(which)
    say(" ", w.describe())
    dA = dev(w.rowptr), dev(w.colind), dev(w.vals)
    for N in w.widths:
        B = w.B(N)
        dB = dev(B)
        for op in w.ops:
            check(gs, w.rowptr, w.colind, w.vals, B, op, label=w.name, dA=dA, dB=dB)
        if which == 2:   # the unweighted graph is also run with vals == NULL
            check(gs, w.rowptr, w.colind, None, B, "sum", label=w.name + " vals=NULL",
                  dA=(dA[0], dA[1], None), dB=dB)


def _sample_rows(rowptr, count, seed):
    lens = np.diff(rowptr)
    rng = np.random.default_rng(seed)
    longest = np.argsort(lens)[-24:]
    empties = np.flatnonzero(lens == 0)[:8]
    rand = rng.integers(0, len(lens), size=count)
    edges = np.array([0, 1, len(lens) - 2, len(lens) - 1])
    return np.unique(np.concatenate([longest, empties, rand, edges])).astype(np.int64)


@pytest.mark.parametrize("which", [3, 4])
def test_large_workloads_full_size_every_element_and_properties(gs, which):
    """Workloads 4 and 5 at full size: EVERY element of every op and width against the oracle (one full
    oracle pass per case), plus properties that hold at any size."""
    w = graphgen.workload(which)
    say(" ", w.describe())
    dA = dev(w.rowptr), dev(w.colind), dev(w.vals)
    lens = np.diff(w.rowptr).astype(np.float64)[:, None]
    for N in w.widths:
        B = w.B(N)
        dB = dev(B)
        out = {}
        for op in w.ops:
            out[op] = check(gs, w.rowptr, w.colind, w.vals, B, op, label=w.name, dA=dA, dB=dB)
            assert np.isfinite(out[op]).all()
            assert not out[op][lens[:, 0] == 0].any()            # every empty row is exactly zero
        # column independence: the left half computed alone must equal the left half of the
        # full run (bit-for-bit for max; every element of the half-width run is checked against the oracle)
        half = N // 2
        Bh = np.ascontiguousarray(B[:, :half])
        for op in w.ops:
            Ch = check(gs, w.rowptr, w.colind, w.vals, Bh, op, label=w.name + " half-width", dA=dA)
            if op in ("max", "min"):
                assert np.array_equal(Ch.view(np.uint32), out[op][:, :half].view(np.uint32))
        if "mean" in out:                                        # mean * len == sum
            _, Sabs = oracle.spmm(w.rowptr, w.colind, w.vals, B, "sum")
            err = np.abs(out["mean"].astype(np.float64) * lens - out["sum"])
            assert (err <= 2e-5 * Sabs + 2e-6 * np.maximum(lens, 1)).all()


@pytest.mark.parametrize("name", graphgen.SUITE_NAMES)
def test_shape_suite_matrices(gs, name):
    """Every matrix of the benchmark's shape suite (banded equal rows, R-MAT skew, many empty rows, long
    rows ...) at the suite's widths, sum and max, every element against the oracle."""
    w = graphgen.suite_matrix(name)
    say(" ", w.describe())
    dA = dev(w.rowptr), dev(w.colind), dev(w.vals)
    for N in ((128, 512) if w.nnz < 1_000_000 else (128,) if w.nnz > 10_000_000 else (128, 256)):
        B = w.B(N)
        for op in ("sum", "max"):
            check(gs, w.rowptr, w.colind, w.vals, B, op, label=name, dA=dA)


def test_invariants_on_the_gpu_at_workload_size(gs):
    """Properties that hold at any size, on workload 3 at full size: permuting the rows of A permutes the
    rows of C (bit for bit for max / min, within twice the bound for sum), min <= mean <= max for unit
    values, and sum is linear in B up to rounding."""
    w = graphgen.workload(2)
    rng = np.random.default_rng(11)
    N = 128
    B = w.B(N)
    order = rng.permutation(w.M)
    lens = np.diff(w.rowptr)
    rp2 = np.zeros(w.M + 1, dtype=np.int32)
    np.cumsum(lens[order], out=rp2[1:])
    starts = w.rowptr[:-1][order]
    src = (np.repeat(starts - rp2[:-1], lens[order]) + np.arange(w.nnz)).astype(np.int64)
    ci2 = w.colind[src]
    dB = dev(B)
    out, moved = {}, {}
    for op in OPS:
        say(f"  case invariants {op}")
        out[op] = gs.gespmm_csr(dev(w.rowptr), dev(w.colind), None, dB, op).cpu().numpy()
        moved[op] = gs.gespmm_csr(dev(rp2), dev(ci2), None, dB, op).cpu().numpy()
    for op in ("max", "min"):
        assert np.array_equal(moved[op].view(np.uint32), out[op][order].view(np.uint32))
    rows = _sample_rows(w.rowptr, 1500, 3)
    _, Sabs = oracle.spmm(w.rowptr, w.colind, None, B, "sum", rows=rows)
    inv = np.empty(w.M, dtype=np.int64)
    inv[order] = np.arange(w.M)
    assert (np.abs(moved["sum"][inv[rows]].astype(np.float64) - out["sum"][rows]) <= 2e-5 * Sabs + 2e-6).all()
    nonempty = lens > 0
    assert (out["min"][nonempty] <= out["mean"][nonempty] + 1e-6).all()
    assert (out["mean"][nonempty] <= out["max"][nonempty] + 1e-6).all()
    B2 = w.B(N + 1)[:, :N].copy()
    both = gs.gespmm_csr(dev(w.rowptr), dev(w.colind), None, dev(B + B2), "sum").cpu().numpy()
    two = gs.gespmm_csr(dev(w.rowptr), dev(w.colind), None, dev(B2), "sum").cpu().numpy()
    _, Sabs2 = oracle.spmm(w.rowptr, w.colind, None, B2, "sum", rows=rows)
    err = np.abs(both[rows].astype(np.float64) - (out["sum"][rows].astype(np.float64) + two[rows]))
    assert (err <= 4e-5 * (Sabs + Sabs2) + 4e-6).all()      # B + B2 is itself rounded to fp32 (relative 6e-8)


def test_wide_feature_matrix_many_column_blocks(gs):
    rp, ci, v = graphgen.random_csr(64, 50, 6.0, 77, empty_frac=0.1, long_rows=((5, 400),), duplicates=True)
    B = graphgen.random_dense(50, 4100, 77)           # 4100 columns: 65 column blocks, ragged last one
    for op in OPS:
        check(gs, rp, ci, v, B, op, label="N=4100")


def test_entry_count_near_the_32_bit_limit(gs):
    """nnz = 2^31 - 2048 (the largest the library accepts is 2^31 - 1025): chunk offsets, the row search
    and the atomics of split rows at the top of the int32 range.  Inputs are built on the device and
    chosen so that the results are exact: 1024 equal rows of ones against an all-ones / ramp B."""
    nnz = 2**31 - 2048
    M, K, N = 1024, 1000, 4
    per_row = nnz // M                                  # 2,097,150: row sums stay below 2^24, exact in fp32
    assert per_row * M == nnz
    say(f"  case near-limit nnz={nnz}")
    colind = torch.arange(nnz, dtype=torch.int32, device="cuda").remainder_(K)
    rowptr = (torch.arange(M + 1, dtype=torch.int64, device="cuda") * per_row).to(torch.int32)
    ones = torch.ones((K, N), dtype=torch.float32, device="cuda")
    ramp = torch.arange(K, dtype=torch.float32, device="cuda")[:, None].repeat(1, N).contiguous()
    C = gs.gespmm_csr(rowptr, colind, None, ones, "sum")
    torch.cuda.synchronize()
    assert bool((C == float(per_row)).all())
    C = gs.gespmm_csr(rowptr, colind, None, ones, "mean")
    torch.cuda.synchronize()
    assert bool(((C - 1.0).abs() <= 1e-5).all())
    C = gs.gespmm_csr(rowptr, colind, None, ramp, "max")
    torch.cuda.synchronize()
    assert bool((C == float(K - 1)).all())
    C = gs.gespmm_csr(rowptr, colind, None, ramp, "min")
    torch.cuda.synchronize()
    assert bool((C == 0.0).all())
    p = ctypes.c_void_p(0x1000)                         # beyond the limit: rejected on the host, nothing runs
    assert gs.lib().gespmm_csr(M, K, N, 2**31 - 1, p, p, None, p, p, 0, None) == 3


@pytest.mark.parametrize("K", [670_000, 671_200])
def test_feature_matrix_at_the_2_gib_border_of_the_buffer_offsets(gs, K):
    """B of 800 columns: 670,000 rows are 2,144,000,000 bytes, just inside what the gathers address with 32-bit
    buffer offsets (byte offsets up to the top of the signed range); 671,200 rows are beyond the border, where the
    kernels compute 64-bit addresses.  Few rows of A, entries spread over all of B including its last row."""
    N, M = 800, 300
    say(f"  case 2 GiB border K={K} bytes={K * N * 4}")
    rng = np.random.default_rng(K)
    B = rng.standard_normal((K, N), dtype=np.float32)
    rp, ci, v = graphgen.random_csr(M, K, 20.0, 77, empty_frac=0.1, long_rows=((5, 1500),))
    ci[-1] = K - 1
    ci[rp[5]:rp[5] + 3] = (0, K - 1, K - 2)
    dB = dev(B)
    for op in ("sum", "max"):
        check(gs, rp, ci, v, B, op, dB=dB, label=f"2 GiB border K={K}")
    del dB
    torch.cuda.empty_cache()


def test_zz_report_worst_error_ratio(gs):
    """Not a check of its own: prints how close sum/mean came to the tolerance in this session."""
    say(f"  worst |C - Cref| / (1e-5 * Sabs + 1e-6) over all sum/mean cases: {WORST['ratio']:.3f} ({WORST['case']})")
    say(f"  ... over the five workloads at full size: {WORST['workload_ratio']:.3f} ({WORST['workload_case']})")
    assert WORST["ratio"] <= 1.0
