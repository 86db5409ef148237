"""GPU parity of the gradient-side entry points against the CPU oracle, through the C ABI.

positions (arg): the value is bit-exact and the position is unique by definition (smallest entry
index among the entries whose product has the bits of the result), so both are compared exactly;
transposed sum/mean and the routed pooling gradient: |dB - dBref| <= 1e-5 * Sabs + 1e-6.
"""
import sys

import numpy as np
import pytest

import graphgen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gs():
    import paper_2007_03179_amd as gs
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    gs.lib()
    return gs


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(x):
    return None if x is None else torch.from_numpy(np.ascontiguousarray(x)).cuda()


def check_arg(gs, rp, ci, v, B, op, rows=None, label="", dA=None, dB=None, tuning=None, workspace=None):
    say(f"  case arg {label} op={op} M={len(rp) - 1} N={B.shape[1]} nnz={len(ci)}")
    d_rp, d_ci, d_v = dA if dA is not None else (dev(rp), dev(ci), dev(v))
    if tuning is None and workspace is None:
        C, arg = gs.gespmm_csr_arg(d_rp, d_ci, d_v, dB if dB is not None else dev(B), op)
    else:
        C, arg = gs.gespmm_csr_arg_ex(d_rp, d_ci, d_v, dB if dB is not None else dev(B), op, tuning=tuning,
                                      workspace=workspace)
    torch.cuda.synchronize()
    C, arg = C.cpu().numpy(), arg.cpu().numpy()
    Cref, aref = oracle.spmm_arg(rp, ci, v, B, op, rows=rows)
    got_c, got_a = (C, arg) if rows is None else (C[rows], arg[rows])
    assert np.array_equal(got_c.view(np.uint32), Cref.astype(np.float32).view(np.uint32)), f"{label}: value bits"
    bad = np.flatnonzero(got_a != aref)
    assert bad.size == 0, f"{label}: {bad.size} positions differ, first at flat index {bad[:1]}"
    return C, arg


def check_transposed(gs, rp, ci, v, dC, op, K, label="", dA=None):
    say(f"  case transposed {label} op={op} M={len(rp) - 1} K={K} N={dC.shape[1]} nnz={len(ci)}")
    d_rp, d_ci, d_v = dA if dA is not None else (dev(rp), dev(ci), dev(v))
    out = gs.gespmm_csr_transposed(d_rp, d_ci, d_v, dev(dC), op, K)
    torch.cuda.synchronize()
    ref, sabs = oracle.spmm_transposed(rp, ci, v, dC, op, K)
    ok, worst = oracle.compare("sum", out.cpu().numpy(), ref, sabs)
    assert ok, f"{label} transposed {op}: worst={worst}"
    return out


def check_pool_backward(gs, ci, v, arg, dC, K, label=""):
    say(f"  case pool-backward {label} M={dC.shape[0]} K={K} N={dC.shape[1]}")
    out = gs.gespmm_pool_backward(dev(ci), dev(v), dev(arg), dev(dC), K)
    torch.cuda.synchronize()
    ref, sabs = oracle.pool_backward(ci, v, arg, dC, K)
    ok, worst = oracle.compare("sum", out.cpu().numpy(), ref, sabs)
    assert ok, f"{label} pool backward: worst={worst}"
    return out


# ---------------------------------------------------------------------------
@pytest.mark.parametrize("N", [1, 4, 7, 8, 32, 33, 64, 128, 520, 1024, 1028])
def test_positions_widths_ties_and_split_rows(gs, N):
    # few distinct values -> many ties; a row spanning many chunks; duplicates; empty rows; M != K
    rp, ci, v = graphgen.random_csr(600, 400, 8.0, 300 + N, empty_frac=0.1, long_rows=((77, 2500),),
                                    duplicates=True, sort_cols=False)
    B = np.round(graphgen.random_dense(400, N, N) * 4.0).astype(np.float32)
    v = np.round(v * 2.0).astype(np.float32)
    v[v == 0] = 1.0
    B[5] = -0.0
    B[6] = 0.0
    for op in ("max", "min"):
        for vv in (v, None):
            check_arg(gs, rp, ci, vv, B, op, label=f"ties N={N}")


@pytest.mark.parametrize("N", [1, 4, 7, 32, 72, 128, 520])
def test_positions_whole_row_path(gs, N):
    """Value and position from the single-launch path (tuning.longest_row): ties, repeated and unsorted columns, empty
    rows at both ends, true and understated bounds (the long row is then walked in windows), every slot width."""
    rp, ci, v = graphgen.random_csr(600, 400, 8.0, 700 + N, empty_frac=0.15, long_rows=((77, 900), (599, 0), (0, 0)),
                                    duplicates=True, sort_cols=False)
    B = np.round(graphgen.random_dense(400, N, N) * 4.0).astype(np.float32)
    v = np.round(v * 2.0).astype(np.float32)
    dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
    longest = int(np.diff(rp).max())
    for hint, G, chunk in ((longest, -1, -1), (5, -1, 64), (longest, 64, 128), (100, 1, 1024), (longest, 4, 16)):
        tuning = dict(longest_row=hint, lanes_per_row=G, chunk_nnz=chunk)
        for op in ("max", "min"):
            check_arg(gs, rp, ci, v, B, op, dA=dA, dB=dB, tuning=tuning, label=f"whole-row hint={hint} G={G} S={chunk}")
    rp0 = np.zeros(5, dtype=np.int32)                               # nothing stored: zeros and -1 from the one launch
    C, arg = check_arg(gs, rp0, np.zeros(0, np.int32), np.zeros(0, np.float32), B, "max", tuning=dict(longest_row=3),
                       label="whole-row nnz=0")
    assert not C.any() and (arg == -1).all()


@pytest.mark.parametrize("N", [4, 12, 64, 128, 520, 1024])
def test_positions_k_phased_path(gs, N):
    """Value and position through the phases of the column range (gespmm_csr_arg_ws with forced parts): ties within and
    across parts, repeated and unsorted columns, empty rows, rows split among chunks, every kernel shape of the path."""
    rp, ci, v = graphgen.random_csr(500, 400, 30.0, 900 + N, empty_frac=0.1, long_rows=((77, 2500), (499, 0), (0, 700)),
                                    duplicates=True, sort_cols=False)
    B = np.round(graphgen.random_dense(400, N, N) * 4.0).astype(np.float32)
    v = np.round(v * 2.0).astype(np.float32)
    v[v == 0] = 1.0
    B[5] = -0.0
    B[6] = 0.0
    dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
    sorted_rows = graphgen.random_csr(500, 400, 30.0, 901 + N, empty_frac=0.1, long_rows=((3, 1500),))
    shapes = ((-1, -1, -1), (8, 1, 64), (16, 1, 512), (32, 1, 128), (8, 2, 256), (16, 2, 1024))
    for parts in (2, 3, 8):
        for G, T, chunk in shapes:
            if G > 0 and G * T * 4 > max(N, 32) * 2:
                continue                                       # (shapes far wider than the matrix add nothing)
            tuning = dict(k_parts=parts, lanes_per_row=G, tiles_per_lane=T, chunk_nnz=chunk)
            need = gs.gespmm_csr_workspace_bytes(len(rp) - 1, 400, N, len(ci), "f32", tuning=tuning)
            assert need > 0
            ws = torch.empty(need // 4 + 1, dtype=torch.int32, device="cuda")
            for op in ("max", "min"):
                check_arg(gs, rp, ci, v, B, op, dA=dA, dB=dB, tuning=tuning, workspace=ws,
                          label=f"phased parts={parts} G={G} T={T} S={chunk}")
        check_arg(gs, *sorted_rows, B, "max", tuning=dict(k_parts=parts), workspace=ws, label=f"phased sorted parts={parts}")
    # all-ones weights (vals == NULL) and nothing stored at all
    check_arg(gs, rp, ci, None, B, "min", tuning=dict(k_parts=3), workspace=ws, label="phased no vals")
    rp0 = np.zeros(6, dtype=np.int32)
    C, arg = check_arg(gs, rp0, np.zeros(0, np.int32), np.zeros(0, np.float32), B, "max", tuning=dict(k_parts=2),
                       workspace=ws, label="phased nnz=0")
    assert not C.any() and (arg == -1).all()


def test_positions_k_phased_path_chosen_by_the_rule(gs):
    """Long rows and a B that is many times an L2: with a workspace the call takes the phases by itself (and says so
    in the plan); values and positions equal the oracle's and the plain call's."""
    M, K, N = 1500, 90000, 64
    rp, ci, v = graphgen.random_csr(M, K, 150.0, 77, empty_frac=0.02, long_rows=((9, 6000),))
    B = np.round(graphgen.random_dense(K, N, 78) * 16.0).astype(np.float32)
    plan = gs.gespmm_plan_ex(M, K, N, len(ci), workspace_bytes=1 << 30)
    assert plan["k_parts"] > 1, plan
    need = gs.gespmm_csr_workspace_bytes(M, K, N, len(ci))
    ws = torch.empty(need // 4 + 1, dtype=torch.int32, device="cuda")
    dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
    for op in ("max", "min"):
        C, arg = check_arg(gs, rp, ci, v, B, op, dA=dA, dB=dB, workspace=ws, label="phased by rule")
        C0, arg0 = gs.gespmm_csr_arg(*dA, dB, op)
        assert np.array_equal(C0.cpu().numpy().view(np.uint32), C.view(np.uint32)) and np.array_equal(arg0.cpu().numpy(), arg)


def test_positions_k_phased_argument_errors(gs):
    rp, ci, v = graphgen.random_csr(64, 64, 5.0, 5)
    B = graphgen.random_dense(64, 8, 6)
    dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
    ws = torch.empty(1 << 16, dtype=torch.int32, device="cuda")
    gs.gespmm_csr_arg_ex(*dA, dB, "max", tuning=dict(k_parts=2))   # the call without a workspace ignores k_parts
    with pytest.raises(gs.GespmmError) as e:                    # too small a workspace
        gs.gespmm_csr_arg_ex(*dA, dB, "max", tuning=dict(k_parts=2), workspace=ws[:4])
    assert e.value.status == 4
    with pytest.raises(gs.GespmmError) as e:                    # 16-bit features have no phased kernels with positions
        gs.gespmm_csr_arg_ex(*dA, dB.to(torch.bfloat16), "max", tuning=dict(k_parts=2), workspace=ws)
    assert e.value.status == 1
    with pytest.raises(gs.GespmmError) as e:                    # nor do widths that are not a multiple of four
        gs.gespmm_csr_arg_ex(*dA, dev(graphgen.random_dense(64, 7, 6)), "max", tuning=dict(k_parts=2), workspace=ws)
    assert e.value.status == 1


def test_positions_every_launch_shape(gs):
    rp, ci, v = graphgen.random_csr(300, 260, 7.0, 56, empty_frac=0.1, long_rows=((11, 900), (12, 300)))
    B = np.round(graphgen.random_dense(260, 72, 56) * 8.0).astype(np.float32)
    dA, dB = (dev(rp), dev(ci), dev(v)), dev(B)
    shapes = [(1, 1), (2, 1), (8, 1), (16, 1), (64, 1), (4, 2), (16, 2), (64, 2), (8, 4), (64, 4)]
    for G, T in shapes:
        for remap, chunk, short in ((0, 16, 0), (1, 256, -1), (1, 1024, 1024)):
            for op in ("max", "min"):
                check_arg(gs, rp, ci, v, B, op, label=f"G={G} T={T} S={chunk} short={short}", dA=dA, dB=dB,
                          tuning=(G, T, remap, chunk, short))


def test_positions_unaligned_outputs_take_the_two_pass_route(gs):
    """C or arg off a 16-byte boundary: scalar kernels, split rows finished by the second pass."""
    rp, ci, v = graphgen.random_csr(300, 200, 6.0, 61, empty_frac=0.1, long_rows=((40, 1500),), duplicates=True)
    B = np.round(graphgen.random_dense(200, 64, 61) * 4.0).astype(np.float32)
    d = dev(rp), dev(ci), dev(v), dev(B)
    for op in ("max", "min"):
        Cref, aref = oracle.spmm_arg(rp, ci, v, B, op)
        for off_c, off_a in ((1, 0), (0, 1), (2, 2)):
            say(f"  case arg unaligned op={op} C+{off_c} arg+{off_a}")
            rawc = torch.full((300 * 64 + 4,), 7.0, device="cuda")
            rawa = torch.full((300 * 64 + 4,), 7, dtype=torch.int32, device="cuda")
            C = rawc[off_c:off_c + 300 * 64].view(300, 64)
            arg = rawa[off_a:off_a + 300 * 64].view(300, 64)
            gs.gespmm_csr_arg(*d, op, C=C, arg=arg)
            torch.cuda.synchronize()
            assert np.array_equal(C.cpu().numpy().view(np.uint32), Cref.astype(np.float32).view(np.uint32))
            assert np.array_equal(arg.cpu().numpy(), aref)
            assert float(rawc[-1]) == 7.0 and int(rawa[-1]) == 7 and float(rawc[0]) in (7.0, float(C[0, 0]))


def test_positions_degenerate(gs):
    B = graphgen.random_dense(5, 8, 1)
    rp, ci, v = np.zeros(4, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32)
    C, arg = check_arg(gs, rp, ci, v, B, "max", label="nnz=0")
    assert (arg == -1).all() and not C.any()
    n = 1000                                        # one long row between empty rows, all products equal
    rp = np.array([0, 0, n, n], dtype=np.int32)
    ci = np.full(n, 3, dtype=np.int32)
    v = np.ones(n, dtype=np.float32)
    C, arg = check_arg(gs, rp, ci, v, B, "min", label="all-equal long row")
    assert (arg[1] == 0).all() and (arg[0] == -1).all() and (arg[2] == -1).all()


@pytest.mark.parametrize("N", [1, 4, 7, 16, 64, 100, 256])
def test_transposed_widths(gs, N):
    rp, ci, v = graphgen.random_csr(500, 350, 9.0, 400 + N, empty_frac=0.1, long_rows=((9, 2000),),
                                    duplicates=True, sort_cols=False)
    dC = graphgen.random_dense(500, N, N + 1)
    for op in ("sum", "mean"):
        check_transposed(gs, rp, ci, v, dC, op, 350, label=f"N={N}")
        check_transposed(gs, rp, ci, None, dC, op, 350, label=f"N={N} vals=NULL")


def test_transposed_degenerate_and_adjoint(gs):
    dC = graphgen.random_dense(3, 8, 2)
    out = check_transposed(gs, np.zeros(4, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32), dC, "sum", 6,
                           label="nnz=0")
    assert not out.cpu().numpy().any()
    # <A (x) B, dC> == <B, A^T (x) dC> with both sides from the GPU
    rp, ci, v = graphgen.random_csr(800, 700, 10.0, 5, empty_frac=0.05, long_rows=((3, 3000),))
    B, dC = graphgen.random_dense(700, 32, 5), graphgen.random_dense(800, 32, 6)
    dA = dev(rp), dev(ci), dev(v)
    for op in ("sum", "mean"):
        C = gs.gespmm_csr(*dA, dev(B), op).double().cpu().numpy()
        dBt = gs.gespmm_csr_transposed(*dA, dev(dC), op, 700).double().cpu().numpy()
        lhs, rhs = float((C * dC).sum()), float((B * dBt).sum())
        scale = float((np.abs(C) * np.abs(dC)).sum())
        assert abs(lhs - rhs) <= 1e-4 * scale, (op, lhs, rhs)


def test_pool_backward_matches_oracle_and_forward_positions(gs):
    rp, ci, v = graphgen.random_csr(700, 500, 9.0, 8, empty_frac=0.1, long_rows=((350, 3000),), duplicates=True)
    for N in (4, 7, 64):
        B = graphgen.random_dense(500, N, N)
        dC = graphgen.random_dense(700, N, N + 9)
        for op in ("max", "min"):
            _, arg = check_arg(gs, rp, ci, v, B, op, label="for pool backward")
            check_pool_backward(gs, ci, v, arg, dC, 500, label=f"{op} N={N}")
            check_pool_backward(gs, ci, None, arg, dC, 500, label=f"{op} N={N} vals=NULL")
    # nothing routed: all rows empty
    arg = np.full((5, 8), -1, dtype=np.int32)
    out = check_pool_backward(gs, np.zeros(1, np.int32), np.ones(1, np.float32), arg, graphgen.random_dense(5, 8, 1), 3)
    assert not out.cpu().numpy().any()


def check_transpose(gs, rp, ci, v, K, scale, label=""):
    """Transposed CSR: row starts exact; inside a row the order is free, so rows are compared as sorted
    lists of (row index of A, value bits)."""
    say(f"  case transpose {label} M={len(rp) - 1} K={K} nnz={len(ci)} scale={scale}")
    rpT, ciT, vT = gs.gespmm_csr_transpose(dev(rp), dev(ci), dev(v), K, scale_by_row_length=scale)
    torch.cuda.synchronize()
    rpT, ciT, vT = rpT.cpu().numpy(), ciT.cpu().numpy(), vT.cpu().numpy()
    rpR, ciR, vR = oracle.csr_transpose(rp, ci, v, K, scale_by_row_length=scale)
    assert np.array_equal(rpT, rpR), f"{label}: row starts"
    rowsT = np.repeat(np.arange(K, dtype=np.int64), np.diff(rpR))
    key_g = np.lexsort((vT.view(np.uint32), ciT, rowsT))
    key_r = np.lexsort((vR.view(np.uint32), ciR, rowsT))
    assert np.array_equal(ciT[key_g], ciR[key_r]), f"{label}: row indices"
    assert np.array_equal(vT.view(np.uint32)[key_g], vR.view(np.uint32)[key_r]), f"{label}: values"
    return rpT, ciT, vT


def check_transpose_sorted(gs, rp, ci, v, K, scale, label=""):
    """The radix-sort transpose is stable, so all three arrays equal the oracle's bit for bit."""
    say(f"  case transpose-sorted {label} M={len(rp) - 1} K={K} nnz={len(ci)} scale={scale}")
    rpT, ciT, vT = gs.gespmm_csr_transpose_sorted(dev(rp), dev(ci), dev(v), K, scale_by_row_length=scale)
    torch.cuda.synchronize()
    rpR, ciR, vR = oracle.csr_transpose(rp, ci, v, K, scale_by_row_length=scale)
    assert np.array_equal(rpT.cpu().numpy(), rpR), f"{label}: row starts"
    assert np.array_equal(ciT.cpu().numpy(), ciR), f"{label}: row indices"
    assert np.array_equal(vT.cpu().numpy().view(np.uint32), vR.view(np.uint32)), f"{label}: values"


@pytest.mark.parametrize("shape", [(500, 350, 9.0), (3000, 5000, 2.0), (1, 1, 1.0), (40, 3, 30.0), (4097, 1025, 1.0),
                                   (200, 70_000, 25.0), (50, 1_100_000, 90.0), (9000, 2, 3.0)])
def test_transpose_sorted_small_and_degenerate(gs, shape):
    # 1, 2 and 3 sort passes (K up to 2^10, 2^20, beyond), tiles that end exactly at 4096, hub columns, empty rows
    M, K, mean_len = shape
    rp, ci, v = graphgen.random_csr(M, K, mean_len, M + K, empty_frac=0.2, duplicates=True, sort_cols=False,
                                    long_rows=((M // 2, 5000),) if M > 100 else ())
    if len(ci) > 300:
        ci[100:300] = ci[0]                                   # a hub column
    for scale in (False, True):
        check_transpose_sorted(gs, rp, ci, v, K, scale, label=f"M={M} K={K}")
    check_transpose_sorted(gs, rp, ci, None, K, True, label=f"M={M} K={K} vals=NULL")


def test_transpose_sorted_nothing_stored_and_exact_tile(gs):
    rpT, ciT, vT = gs.gespmm_csr_transpose_sorted(dev(np.zeros(4, np.int32)), dev(np.zeros(0, np.int32)), None, 7)
    assert rpT.shape == (8,) and not rpT.cpu().numpy().any() and ciT.numel() == 0
    rp = np.arange(0, 4096 * 2 + 1, 2, dtype=np.int32)          # exactly two full tiles
    ci = np.tile(np.array([5, 0], dtype=np.int32), 4096)
    check_transpose_sorted(gs, rp, ci, None, 6, False, label="two full tiles")


def test_transpose_structure_small_and_degenerate(gs):
    for M, K, mean_len, seed, kw in ((500, 350, 9.0, 1, dict(empty_frac=0.1, duplicates=True, sort_cols=False,
                                                              long_rows=((9, 2000),))),
                                     (3000, 5000, 2.0, 2, dict(empty_frac=0.5)),          # several scan tiles
                                     (1, 1, 1.0, 3, {}), (40, 3, 30.0, 4, dict(duplicates=True))):
        rp, ci, v = graphgen.random_csr(M, K, mean_len, seed, **kw)
        for scale in (False, True):
            check_transpose(gs, rp, ci, v, K, scale, label=f"M={M}")
        check_transpose(gs, rp, ci, None, K, False, label=f"M={M} vals=NULL")
    rpT, ciT, vT = check_transpose(gs, np.zeros(4, np.int32), np.zeros(0, np.int32), None, 7, False, label="nnz=0")
    assert not rpT.any()


def test_gradient_of_sum_and_mean_through_the_transposed_arrays(gs):
    rp, ci, v = graphgen.random_csr(900, 700, 10.0, 6, empty_frac=0.05, long_rows=((3, 3000),), duplicates=True)
    dC = graphgen.random_dense(900, 64, 7)
    for scale, op in ((False, "sum"), (True, "mean")):
        rpT, ciT, vT = gs.gespmm_csr_transpose(dev(rp), dev(ci), dev(v), 700, scale_by_row_length=scale)
        out = gs.gespmm_csr(rpT, ciT, vT, dev(dC), "sum")
        torch.cuda.synchronize()
        ref, sabs = oracle.spmm_transposed(rp, ci, v, dC, op, 700)
        ok, worst = oracle.compare("sum", out.cpu().numpy(), ref, sabs)
        assert ok, (op, worst)


@pytest.mark.parametrize("which", [2, 4, 3])
def test_gradient_side_on_workloads(gs, which):
    w = graphgen.workload(which)
    say(" ", w.describe())
    N = w.widths[-1]
    B = w.B(N)
    dC = graphgen.uniform_pm1((w.M, N), 99, stream=N)
    vals = graphgen.uniform_pm1(w.nnz, 98)              # signed weights: max and min both non-trivial
    dA = dev(w.rowptr), dev(w.colind), dev(vals)
    lens = np.diff(w.rowptr)
    for op in ("max", "min"):                           # every value and every position against the oracle
        C, arg = check_arg(gs, w.rowptr, w.colind, vals, B, op, label=w.name, dA=dA)
        # properties at full size: the position lies in its row and reproduces the value bit for bit
        i, j = np.nonzero(arg >= 0)
        p = arg[i, j]
        assert (arg[lens == 0] == -1).all() and (arg[lens > 0] >= 0).all()
        assert (p >= w.rowptr[i]).all() and (p < w.rowptr[i + 1]).all()
        prod = vals[p] * B[w.colind[p], j]              # one fp32 product, as the kernel forms it
        assert np.array_equal(prod.view(np.uint32), C[i, j].view(np.uint32))
        if op == "max":
            check_pool_backward(gs, w.colind, vals, arg, dC, w.K, label=w.name)
    if which == 3:          # the long-row workload: positions and pooled gradient only (every row is split)
        return
    for op in ("sum", "mean"):
        check_transposed(gs, w.rowptr, w.colind, vals, dC, op, w.K, label=w.name, dA=dA)
    check_transpose(gs, w.rowptr, w.colind, vals, w.K, True, label=w.name)
    check_transpose_sorted(gs, w.rowptr, w.colind, vals, w.K, True, label=w.name)
