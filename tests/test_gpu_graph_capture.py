"""The entry points under HIP graph capture: no call allocates, synchronises or uses a memset node,
so a captured call must replay with the same results as eager calls (checked on every replay, with
eager work and synchronisations in between)."""
import numpy as np
import pytest

import graphgen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_captured_calls_replay_like_eager_calls():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2007_03179_amd as gs
    gs.lib()
    rp, ci, v = graphgen.random_csr(3000, 2000, 9.0, 41, empty_frac=0.1, long_rows=((7, 5000),), duplicates=True)
    d = lambda x: torch.from_numpy(x).cuda()
    d_rp, d_ci, d_v = d(rp), d(ci), d(v)
    N = 64
    B = torch.empty((2000, N), dtype=torch.float32, device="cuda")
    dC = torch.empty((3000, N), dtype=torch.float32, device="cuda")
    C_sum = torch.empty((3000, N), dtype=torch.float32, device="cuda")
    C_max = torch.empty_like(C_sum)
    arg = torch.empty((3000, N), dtype=torch.int32, device="cuda")
    dB_t = torch.empty((2000, N), dtype=torch.float32, device="cuda")
    dB_p = torch.empty_like(dB_t)

    def fill(seed):
        B.copy_(d(graphgen.random_dense(2000, N, seed)))
        dC.copy_(d(graphgen.random_dense(3000, N, seed + 100)))

    def calls():
        gs.gespmm_csr(d_rp, d_ci, d_v, B, "sum", C=C_sum)
        gs.gespmm_csr_arg(d_rp, d_ci, d_v, B, "max", C=C_max, arg=arg)
        gs.gespmm_csr_transposed(d_rp, d_ci, d_v, dC, "mean", 2000, dB=dB_t)
        gs.gespmm_pool_backward(d_ci, d_v, arg, dC, 2000, dB=dB_p)

    fill(0)
    calls()                                   # warm-up outside capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
    for replay in range(4):
        print(f"  case graph replay {replay}", flush=True)
        fill(10 + replay)                     # eager work between replays
        for t in (C_sum, C_max, dB_t, dB_p):
            t.fill_(float("nan"))
        arg.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (C_sum, C_max, arg, dB_t, dB_p)]
        calls()                               # the same work eagerly
        torch.cuda.synchronize()
        Bh, dCh = B.cpu().numpy(), dC.cpu().numpy()
        ok, worst = oracle.compare("sum", got[0].cpu().numpy(), *oracle.spmm(rp, ci, v, Bh, "sum"))
        assert ok, (replay, worst)
        assert torch.equal(got[1], C_max) and torch.equal(got[2], arg), replay      # exact ops: bit-identical
        cref, aref = oracle.spmm_arg(rp, ci, v, Bh, "max")
        assert np.array_equal(got[2].cpu().numpy(), aref)
        ok, worst = oracle.compare("sum", got[3].cpu().numpy(), *oracle.spmm_transposed(rp, ci, v, dCh, "mean", 2000))
        assert ok, (replay, worst)
        ok, worst = oracle.compare("sum", got[4].cpu().numpy(), *oracle.pool_backward(ci, v, aref, dCh, 2000))
        assert ok, (replay, worst)


def test_captured_phased_and_whole_row_calls_replay_like_eager_calls():
    """The K-phased path (workspace, several launches that fold into C, scan kernels) and the whole-row path
    (one launch) of gespmm_csr_ex, and a reduce compiled at run time, captured into one graph."""
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2007_03179_amd as gs
    gs.lib()
    rp, ci, v = graphgen.random_csr(2500, 1800, 30.0, 43, empty_frac=0.05, long_rows=((9, 900),))
    d = lambda x: torch.from_numpy(x).cuda()
    d_rp, d_ci, d_v = d(rp), d(ci), d(v)
    N = 64
    B = torch.empty((1800, N), dtype=torch.float32, device="cuda")
    C_phased, C_whole, C_custom = (torch.empty((2500, N), dtype=torch.float32, device="cuda") for _ in range(3))
    phased = dict(k_parts=5)
    whole = dict(longest_row=int(np.diff(rp).max()))
    assert gs.gespmm_plan_ex(2500, 1800, N, len(ci), tuning=whole)["row_window"] > 0
    work = torch.empty(gs.gespmm_csr_workspace_bytes(2500, 1800, N, len(ci), tuning=phased) // 4 + 1, dtype=torch.int32, device="cuda")
    op = gs.gespmm_custom_op_create("""struct SumAbs {
        static __device__ float identity() { return 0.0f; }
        static __device__ float step(float acc, float a, float b) { return acc + __builtin_fabsf(a * b); }
        static __device__ float merge(float x, float y) { return x + y; } };""", "SumAbs")

    def calls():
        gs.gespmm_csr_ex(d_rp, d_ci, d_v, B, "mean", C=C_phased, workspace=work, tuning=phased)
        gs.gespmm_csr_ex(d_rp, d_ci, d_v, B, "sum", C=C_whole, tuning=whole)
        gs.gespmm_csr_custom(op, d_rp, d_ci, d_v, B, C=C_custom)

    B.copy_(d(graphgen.random_dense(1800, N, 1)))
    calls()                                   # warm-up outside capture (also compiles the run-time kernel)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
    for replay in range(3):
        print(f"  case graph replay (phased, whole-row, run-time reduce) {replay}", flush=True)
        B.copy_(d(graphgen.random_dense(1800, N, 20 + replay)))
        for t in (C_phased, C_whole, C_custom):
            t.fill_(float("nan"))
        work.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        Bh = B.cpu().numpy()
        ok, worst = oracle.compare("mean", C_phased.cpu().numpy(), *oracle.spmm(rp, ci, v, Bh, "mean"))
        assert ok, (replay, worst)
        ok, worst = oracle.compare("sum", C_whole.cpu().numpy(), *oracle.spmm(rp, ci, v, Bh, "sum"))
        assert ok, (replay, worst)
        ref = oracle.spmm_custom(rp, ci, v, Bh[:, :4].copy(), 0.0, lambda acc, a, b: acc + abs(a * b))
        got = C_custom.cpu().numpy()[:, :4]
        assert np.all(np.abs(got - ref) <= 1e-5 * ref + 1e-6), replay
    gs.gespmm_custom_op_destroy(op)
