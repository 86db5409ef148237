"""The autograd wrapper on the GPU: gradients against the CPU oracle and against dense PyTorch."""
import numpy as np
import pytest

import graphgen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ag():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2007_03179_amd as gs
    from paper_2007_03179_amd import autograd as ag
    gs.lib()
    return ag


def _graph(ag, rp, ci, v, K):
    d = lambda x: torch.from_numpy(x).cuda()
    return ag.CsrGraph(d(rp), d(ci), None if v is None else d(v), K)


@pytest.mark.parametrize("op", ["sum", "mean", "max", "min"])
def test_gradient_matches_oracle(ag, op):
    rp, ci, v = graphgen.random_csr(600, 450, 8.0, 21, empty_frac=0.1, long_rows=((5, 2500),), duplicates=True)
    Bh, dCh = graphgen.random_dense(450, 32, 3), graphgen.random_dense(600, 32, 4)
    print(f"  case autograd {op}", flush=True)
    g = _graph(ag, rp, ci, v, 450)
    B = torch.from_numpy(Bh).cuda().requires_grad_(True)
    C = ag.spmm(g, B, op)
    C.backward(torch.from_numpy(dCh).cuda())
    torch.cuda.synchronize()
    ok, worst = oracle.compare(op, C.detach().cpu().numpy(), *oracle.spmm(rp, ci, v, Bh, op))
    assert ok, worst
    if op in ("sum", "mean"):
        ref, sabs = oracle.spmm_transposed(rp, ci, v, dCh, op, 450)
    else:
        _, arg = oracle.spmm_arg(rp, ci, v, Bh, op)
        ref, sabs = oracle.pool_backward(ci, v, arg, dCh, 450)
    ok, worst = oracle.compare("sum", B.grad.cpu().numpy(), ref, sabs)
    assert ok, worst
    # a second backward through the cached transposed arrays gives the same gradient
    B.grad = None
    ag.spmm(g, B, op).backward(torch.from_numpy(dCh).cuda())
    ok, worst = oracle.compare("sum", B.grad.cpu().numpy(), ref, sabs)
    assert ok, worst


def test_gradient_matches_dense_pytorch(ag):
    rp, ci, v = graphgen.random_csr(40, 30, 5.0, 31, empty_frac=0.1)
    A = np.zeros((40, 30), dtype=np.float32)
    rows = np.repeat(np.arange(40), np.diff(rp))
    A[rows, ci] = v
    mask = np.zeros((40, 30), dtype=bool)
    mask[rows, ci] = True
    g = _graph(ag, rp, ci, v, 30)
    Bh, dCh = graphgen.random_dense(30, 8, 5), graphgen.random_dense(40, 8, 6)
    Ad, maskd, dC = torch.from_numpy(A).cuda(), torch.from_numpy(mask).cuda(), torch.from_numpy(dCh).cuda()
    for op in ("sum", "max"):
        print(f"  case dense-reference {op}", flush=True)
        B1 = torch.from_numpy(Bh).cuda().requires_grad_(True)
        B2 = torch.from_numpy(Bh).cuda().requires_grad_(True)
        ag.spmm(g, B1, op).backward(dC)
        if op == "sum":
            ref = Ad @ B2
        else:
            prod = Ad[:, :, None] * B2[None, :, :]
            prod = torch.where(maskd[:, :, None], prod, torch.full_like(prod, -float("inf")))
            ref = prod.max(dim=1).values
            ref = torch.where(torch.isinf(ref), torch.zeros_like(ref), ref)
        ref.backward(dC)
        torch.cuda.synchronize()
        assert torch.allclose(B1.grad, B2.grad, rtol=1e-5, atol=1e-5)


def test_two_layer_gcn_trains(ag):
    """GCN layer (sum, normalised weights) + pooling layer (max): the loss on labels produced by a
    teacher of the same shape must fall, i.e. the gradients point the right way end to end."""
    w = graphgen.workload(0)
    g = _graph(ag, w.rowptr, w.colind, w.vals, w.K)
    X = torch.from_numpy(graphgen.uniform_pm1((w.M, 32), 1)).cuda()
    torch.manual_seed(1)
    t1, t2 = ag.GraphConv(32, 16).cuda(), ag.GraphConv(16, 7, op="max").cuda()
    with torch.no_grad():
        y = t2(g, torch.relu(t1(g, X))).argmax(dim=1)
    torch.manual_seed(2)
    l1, l2 = ag.GraphConv(32, 16).cuda(), ag.GraphConv(16, 7, op="max").cuda()
    opt = torch.optim.Adam(list(l1.parameters()) + list(l2.parameters()), lr=0.02)
    losses = []
    for _ in range(60):
        opt.zero_grad()
        loss = torch.nn.functional.cross_entropy(l2(g, torch.relu(l1(g, X))), y)
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    print("  gcn losses", losses[0], losses[-1], flush=True)
    assert np.isfinite(losses).all() and losses[-1] < losses[0] * 0.8


@pytest.mark.parametrize("aggregator", ["mean", "pool"])
def test_sage_layer_matches_dense_pytorch(ag, aggregator):
    """Output and every gradient of a GraphSAGE layer against the same layer written with dense tensors."""
    rp, ci, _ = graphgen.random_csr(50, 50, 4.0, 41, empty_frac=0.1)
    print(f"  case sage {aggregator}", flush=True)
    g = _graph(ag, rp, ci, None, 50)
    rows = np.repeat(np.arange(50), np.diff(rp))
    mask = np.zeros((50, 50), dtype=bool)
    mask[rows, ci] = True
    maskd = torch.from_numpy(mask).cuda()
    lens = torch.from_numpy(np.diff(rp).astype(np.float32)).cuda()
    torch.manual_seed(3)
    layer = ag.SageConv(12, 8, aggregator).cuda()
    X1 = torch.from_numpy(graphgen.random_dense(50, 12, 8)).cuda().requires_grad_(True)
    X2 = X1.detach().clone().requires_grad_(True)
    dOut = torch.from_numpy(graphgen.random_dense(50, 8, 9)).cuda()
    out = layer(g, X1)
    out.backward(dOut)
    got = [X1.grad.clone()] + [p.grad.clone() for p in layer.parameters()]
    layer.zero_grad()
    if aggregator == "mean":
        agg = (maskd.float() @ X2) / lens.clamp(min=1)[:, None]
    else:
        m = torch.relu(layer.w_pool(X2))
        prod = torch.where(maskd[:, :, None], m[None, :, :], torch.full((50, 50, 12), -float("inf"), device="cuda"))
        agg = prod.max(dim=1).values
        agg = torch.where(torch.isinf(agg), torch.zeros_like(agg), agg)
    ref = layer.w_self(X2) + layer.w_neigh(agg)
    ref.backward(dOut)
    want = [X2.grad] + [p.grad for p in layer.parameters()]
    torch.cuda.synchronize()
    assert torch.allclose(out, ref, rtol=1e-5, atol=1e-5)
    for a, b in zip(got, want):
        assert torch.allclose(a, b, rtol=1e-4, atol=1e-5)


@pytest.mark.parametrize("op", ["sum", "max"])
def test_features_stored_in_16_bits(ag, op):
    """B as bfloat16: forward equals the oracle on the stored values; the gradient (computed in fp32, rounded
    to bfloat16 at the end) is within one bfloat16 rounding of the oracle's."""
    rp, ci, v = graphgen.random_csr(500, 400, 8.0, 71, empty_frac=0.1, long_rows=((5, 2000),), duplicates=True)
    Bn = torch.from_numpy(graphgen.random_dense(400, 32, 7)).to(torch.bfloat16)
    Bw, dCh = Bn.float().numpy(), graphgen.random_dense(500, 32, 8)
    print(f"  case autograd bf16 {op}", flush=True)
    g = _graph(ag, rp, ci, v, 400)
    B = Bn.cuda().requires_grad_(True)
    C = ag.spmm(g, B, op)
    assert C.dtype == torch.float32
    C.backward(torch.from_numpy(dCh).cuda())
    torch.cuda.synchronize()
    ok, worst = oracle.compare(op, C.detach().cpu().numpy(), *oracle.spmm(rp, ci, v, Bw, op))
    assert ok, worst
    if op == "sum":
        ref, sabs = oracle.spmm_transposed(rp, ci, v, dCh, op, 400)
    else:
        _, arg = oracle.spmm_arg(rp, ci, v, Bw, op)
        ref, sabs = oracle.pool_backward(ci, v, arg, dCh, 400)
    assert B.grad.dtype == torch.bfloat16
    err = np.abs(B.grad.float().cpu().numpy().astype(np.float64) - ref)
    assert (err <= 2.0 ** -8 * np.abs(ref) + 1e-5 * sabs + 1e-6).all()
