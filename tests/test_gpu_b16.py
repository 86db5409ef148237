"""GPU parity of gespmm_csr_b16 (B stored as bfloat16 / float16, fp32 arithmetic and result).

The oracle is unchanged: it receives B widened back to fp32 (exact), so the bar is the same as for
fp32 inputs: sum / mean within 1e-5 * Sabs + 1e-6, max / min bit-for-bit.
"""
import sys

import numpy as np
import pytest

import graphgen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

OPS = ("sum", "mean", "max", "min")
DTYPES = {"bf16": torch.bfloat16, "f16": torch.float16}


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


def narrow(B, dt):
    """(B rounded to the 16-bit type as a torch CPU tensor, the same values widened to fp32 numpy)."""
    Bn = torch.from_numpy(B).to(DTYPES[dt])
    return Bn, Bn.float().numpy()


def check(gs, rp, ci, v, B, dt, op, rows=None, label="", dA=None, dB=None, tuning=None, workspace=None):
    say(f"  case {label} {dt} op={op} M={len(rp) - 1} K={B.shape[0]} N={B.shape[1]} nnz={len(ci)}")
    Bn, Bw = narrow(B, dt)
    d_rp, d_ci, d_v = dA if dA is not None else (dev(rp), dev(ci), dev(v))
    if tuning is None and workspace is None:
        C = gs.gespmm_csr_b16(d_rp, d_ci, d_v, dB if dB is not None else Bn.cuda(), op)
    else:
        C = gs.gespmm_csr_ex(d_rp, d_ci, d_v, dB if dB is not None else Bn.cuda(), op, tuning=tuning, workspace=workspace)
    torch.cuda.synchronize()
    C = C.cpu().numpy()
    Cref, Sabs = oracle.spmm(rp, ci, v, Bw, op, rows=rows)
    ok, worst = oracle.compare(op, C if rows is None else C[rows], Cref, Sabs)
    assert ok, f"{label} {dt} {op}: worst={worst}"
    return C


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("N", [1, 3, 4, 8, 12, 16, 32, 64, 72, 100, 128, 256, 512, 520])
def test_widths_all_ops(gs, N, dt):
    rp, ci, v = graphgen.random_csr(700, 500, 9.0, 200 + N, empty_frac=0.1, long_rows=((350, 3000),), duplicates=True)
    B = graphgen.random_dense(500, N, N)
    for op in OPS:
        check(gs, rp, ci, v, B, dt, op, label=f"widths N={N}")


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_every_kernel_shape(gs, dt):
    rp, ci, v = graphgen.random_csr(300, 260, 7.0, 56, empty_frac=0.1, long_rows=((11, 900), (12, 300)))
    dA = dev(rp), dev(ci), dev(v)
    for N, vec, shapes in ((136, 4, (1, 2, 4, 8, 16, 32)), (37, 1, (1, 2, 4, 8, 16, 32, 64))):
        B = graphgen.random_dense(260, N, 56)
        dB = narrow(B, dt)[0].cuda()
        for G in shapes:
            for chunk, short in ((16, 0), (256, -1), (1024, 1024)):
                tuning = (G, 1, -1, chunk, short)
                plan = gs.gespmm_plan_ex(300, 260, N, len(ci), dt, tuning=tuning)
                assert (plan["vec"], plan["lanes_per_row"], plan["chunk_nnz"]) == (vec, G, chunk)
                for op in OPS:
                    check(gs, rp, ci, v, B, dt, op, dA=dA, dB=dB, tuning=tuning, label=f"G={G} S={chunk} short={short}")


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_k_phased_path_with_16_bit_features(gs, dt):
    rp, ci, v = graphgen.random_csr(500, 700, 30.0, 57, empty_frac=0.1, long_rows=((11, 2500),))
    dA = dev(rp), dev(ci), dev(v)
    for N in (64, 136):
        B = graphgen.random_dense(700, N, 57)
        dB = narrow(B, dt)[0].cuda()
        for parts, G in ((3, 8), (16, 16), (5, 32)):
            tuning = dict(k_parts=parts, lanes_per_row=G)
            need = gs.gespmm_csr_workspace_bytes(500, 700, N, len(ci), dt, tuning=tuning)
            assert need > 0
            work = torch.empty(need // 4, dtype=torch.int32, device="cuda")
            for op in OPS:
                check(gs, rp, ci, v, B, dt, op, dA=dA, dB=dB, tuning=tuning, workspace=work, label=f"phased parts={parts} G={G}")


def test_unaligned_and_special_values(gs):
    rp, ci, v = graphgen.random_csr(200, 150, 8.0, 9, empty_frac=0.2)
    B = graphgen.random_dense(150, 64, 9)
    B[3, :8] = [0.0, -0.0, 65504.0, -65504.0, 6.1035e-05, 5.96e-08, 1.0, -1.0]    # fp16 extremes and subnormals
    for dt in ("bf16", "f16"):
        Bn, Bw = narrow(B, dt)
        raw = torch.empty(150 * 64 + 1, dtype=DTYPES[dt], device="cuda")
        d_B = raw[1:].view(150, 64)                       # 2 bytes off a 16-byte boundary: one column per lane
        d_B.copy_(Bn)
        for op in OPS:
            C = gs.gespmm_csr_b16(dev(rp), dev(ci), dev(v), d_B, op)
            torch.cuda.synchronize()
            ok, worst = oracle.compare(op, C.cpu().numpy(), *oracle.spmm(rp, ci, v, Bw, op))
            assert ok, (dt, op, worst)
            check(gs, rp, ci, None, B, dt, op, label="vals=NULL")


def test_fp32_dtype_code_is_the_plain_call(gs):
    rp, ci, v = graphgen.random_csr(300, 200, 6.0, 4)
    B = dev(graphgen.random_dense(200, 32, 4))
    for op in ("sum", "max"):
        a = gs.gespmm_csr_b16(dev(rp), dev(ci), dev(v), B, op)
        b = gs.gespmm_csr(dev(rp), dev(ci), dev(v), B, op)
        torch.cuda.synchronize()
        if op == "max":
            assert torch.equal(a, b)
        else:
            assert torch.allclose(a, b, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("which,N,dt", [(2, 128, "bf16"), (2, 128, "f16"), (4, 32, "bf16"), (3, 64, "bf16")])
def test_workloads_at_full_size(gs, which, N, dt):
    w = graphgen.workload(which)
    say(" ", w.describe())
    dA = dev(w.rowptr), dev(w.colind), dev(w.vals)
    B = w.B(N)
    for op in w.ops:                                    # every element against the oracle
        C = check(gs, w.rowptr, w.colind, w.vals, B, dt, op, label=w.name, dA=dA)
        assert np.isfinite(C).all()


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("N", [1, 4, 7, 12, 32, 64, 100, 128, 520, 1028])
def test_value_and_position_with_16_bit_features(gs, N, dt):
    """gespmm_csr_arg_b16: value bits and positions equal the oracle's on the stored (widened) values; few
    distinct values so that ties are common; a row spanning many chunks; widths on both routes for split rows."""
    rp, ci, v = graphgen.random_csr(600, 400, 8.0, 500 + N, empty_frac=0.1, long_rows=((77, 2500),),
                                    duplicates=True, sort_cols=False)
    B = np.round(graphgen.random_dense(400, N, N) * 4.0).astype(np.float32)
    v = np.round(v * 2.0).astype(np.float32)
    v[v == 0] = 1.0
    B[5] = -0.0
    Bn, Bw = narrow(B, dt)
    for op in ("max", "min"):
        for vv in (v, None):
            say(f"  case arg-b16 {dt} N={N} op={op} vals={'yes' if vv is not None else 'NULL'}")
            C, arg = gs.gespmm_csr_arg_b16(dev(rp), dev(ci), dev(vv), Bn.cuda(), op)
            torch.cuda.synchronize()
            Cref, aref = oracle.spmm_arg(rp, ci, vv, Bw, op)
            assert np.array_equal(C.cpu().numpy().view(np.uint32), Cref.astype(np.float32).view(np.uint32))
            assert np.array_equal(arg.cpu().numpy(), aref)


def test_value_and_position_b16_on_a_workload(gs):
    w = graphgen.workload(2)
    N = 128
    Bn, Bw = narrow(w.B(N), "bf16")
    vals = graphgen.uniform_pm1(w.nnz, 98)
    for op in ("max", "min"):                           # every value and position
        say(f"  case arg-b16 workload op={op}")
        C, arg = gs.gespmm_csr_arg_b16(dev(w.rowptr), dev(w.colind), dev(vals), Bn.cuda(), op)
        torch.cuda.synchronize()
        Cref, aref = oracle.spmm_arg(w.rowptr, w.colind, vals, Bw, op)
        assert np.array_equal(C.cpu().numpy().view(np.uint32), Cref.astype(np.float32).view(np.uint32))
        assert np.array_equal(arg.cpu().numpy(), aref)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("N", [1, 4, 8, 37, 64, 136, 512])
def test_whole_row_path_on_16_bit_features(gs, N, dt):
    """The single-launch path (tuning.longest_row) with B stored in 16 bits: true and understated bounds, empty rows,
    rows longer than a chunk, every slot width the kernels exist for."""
    rp, ci, v = graphgen.random_csr(600, 400, 9.0, 900 + N, empty_frac=0.15, long_rows=((77, 900), (599, 0), (0, 0)))
    B = graphgen.random_dense(400, N, N)
    dA, dB = (dev(rp), dev(ci), dev(v)), narrow(B, dt)[0].cuda()
    longest = int(np.diff(rp).max())
    for hint, G, chunk in ((longest, -1, -1), (4, -1, 64), (longest, 32, 128), (100, 1, 1024), (longest, 2, 16)):
        tuning = dict(longest_row=hint, lanes_per_row=G, chunk_nnz=chunk)
        if G < 0:                                   # (a forced narrow slot can make the problem too large for a long bound)
            assert gs.gespmm_plan_ex(600, 400, N, len(ci), dt, tuning=tuning)["row_window"] > 0
        for op in OPS:
            check(gs, rp, ci, v, B, dt, op, dA=dA, dB=dB, tuning=tuning, label=f"whole-row hint={hint} G={G} S={chunk}")
