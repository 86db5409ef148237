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
