"""The SpMM-like operation as a PyTorch autograd function: the paper embeds its kernel in the framework
as an operator that carries its own gradient definition and is used as the aggregation step of a GNN layer
(Section IV-B).

Thin glue over the C ABI: the forward pass is gespmm_csr_ex (sum, mean) or gespmm_csr_arg (max, min);
the backward pass with respect to the dense features is gespmm_csr_ex on the transposed arrays
(built once per graph by gespmm_csr_transpose_sorted and cached) or gespmm_pool_backward.  The edge
values are treated as constants (no gradient), as in the paper's operator.  The graph object keeps what a
framework knows about its graph anyway and the library can use: the length of the longest row of either
orientation (read back once; it selects the single-launch whole-row path on graphs of short rows) and a
workspace per feature width (it enables the K-phased path on graphs of long rows and wide feature tables).
"""
from __future__ import annotations

import torch

from . import binding as _b


class CsrGraph:
    """A sparse matrix A (M x K) in CSR on the GPU, plus lazily built transposed arrays."""

    def __init__(self, rowptr, colind, vals, K):
        assert rowptr.is_cuda and rowptr.dtype == torch.int32
        assert colind.is_cuda and colind.dtype == torch.int32
        assert vals is None or (vals.is_cuda and vals.dtype == torch.float32)
        self.rowptr, self.colind, self.vals = rowptr.contiguous(), colind.contiguous(), vals
        self.M, self.K = rowptr.numel() - 1, int(K)
        self._transposed = {}
        self._longest = {}
        self._workspaces = {}

    def transposed(self, mean: bool):
        """(rowptrT, colindT, valsT); with mean weights val / row length when `mean`."""
        if mean not in self._transposed:
            self._transposed[mean] = _b.gespmm_csr_transpose_sorted(self.rowptr, self.colind, self.vals, self.K,
                                                                    scale_by_row_length=mean)
        return self._transposed[mean]

    def aggregate(self, B, op, transposed=False):
        """The forward call on A (or, for the gradient of sum / mean, on the transposed arrays) with the hints
        and the workspace this graph keeps; for max / min it returns (C, positions).  The workspace of one
        (orientation, width, type) is reused by every call: calls on one graph are assumed to be issued on one
        stream, as autograd issues them."""
        rowptr, colind, vals = self.transposed(op == "mean") if transposed else (self.rowptr, self.colind, self.vals)
        rows, cols = (self.K, self.M) if transposed else (self.M, self.K)
        if transposed not in self._longest:            # one read-back per orientation
            self._longest[transposed] = int((rowptr[1:] - rowptr[:-1]).max().item()) if rows else 0
        if ("tuning", transposed) not in self._longest:
            self._longest[("tuning", transposed)] = _b.make_tuning({"longest_row": self._longest[transposed]})
        tuning = self._longest[("tuning", transposed)]
        dtype = {torch.float32: "f32", torch.bfloat16: "bf16", torch.float16: "f16"}[B.dtype]
        key = (transposed, B.shape[1], dtype)
        if key not in self._workspaces:
            need = _b.gespmm_csr_workspace_bytes(rows, cols, B.shape[1], colind.numel(), dtype, tuning=tuning)
            self._workspaces[key] = torch.empty(need // 4 + 1, dtype=torch.int32, device=B.device) if need else None
        if op in ("max", "min"):                       # value and position (forward pass of the pooling aggregation)
            return _b.gespmm_csr_arg_ex(rowptr, colind, vals, B, op, tuning=tuning, workspace=self._workspaces[key])
        return _b.gespmm_csr_ex(rowptr, colind, vals, B, "sum" if transposed else op, workspace=self._workspaces[key],
                                tuning=tuning)


class _SpMM(torch.autograd.Function):
    @staticmethod
    def forward(ctx, B, graph, op):
        B = B.contiguous()
        ctx.graph, ctx.op, ctx.b_dtype = graph, op, B.dtype
        if op in ("max", "min"):          # (the *_b16 calls take fp32 as well)
            C, arg = graph.aggregate(B, op)
            ctx.save_for_backward(arg)
            ctx.mark_non_differentiable(arg)
            return C
        return graph.aggregate(B, op)

    @staticmethod
    def backward(ctx, dC):
        graph, op = ctx.graph, ctx.op
        dC = dC.contiguous()
        if op in ("max", "min"):
            (arg,) = ctx.saved_tensors
            dB = _b.gespmm_pool_backward(graph.colind, graph.vals, arg, dC, graph.K)
        else:
            dB = graph.aggregate(dC, op, transposed=True)
        return dB.to(ctx.b_dtype), None, None


def spmm(graph: CsrGraph, B: torch.Tensor, op: str = "sum") -> torch.Tensor:
    """C = A (x) B with gradient with respect to B.  B: (K, N) CUDA tensor, float32, or bfloat16 / float16
    (stored features only: the arithmetic, C and the gradient computation are float32; the gradient is
    rounded to B's type at the end)."""
    assert op in _b.OPS and B.is_cuda and B.shape[0] == graph.K
    assert B.dtype in (torch.float32, torch.bfloat16, torch.float16)
    return _SpMM.apply(B, graph, op)


class GraphConv(torch.nn.Module):
    """One graph-convolution layer: aggregate(A, X W) + b, the layer both GCN (op='sum' with
    normalised edge values) and GraphSAGE-pool (op='max') are built from (Section V-E)."""

    def __init__(self, in_features, out_features, op="sum", bias=True):
        super().__init__()
        self.op = op
        self.weight = torch.nn.Parameter(torch.empty(in_features, out_features))
        self.bias = torch.nn.Parameter(torch.zeros(out_features)) if bias else None
        torch.nn.init.xavier_uniform_(self.weight)

    def forward(self, graph: CsrGraph, X):
        out = spmm(graph, X @ self.weight, self.op)
        return out if self.bias is None else out + self.bias


class SageConv(torch.nn.Module):
    """One GraphSAGE layer, h_v = W_self x_v + W_neigh agg_{u in N(v)} m_u (+ b).  aggregator 'mean'
    takes m_u = x_u with the mean over the stored entries of row v (an SpMM); aggregator 'pool' takes
    m_u = relu(W_pool x_u + b_pool) with the element-wise maximum (the SpMM-like operation the paper
    singles out, Section V-E).  Use a graph with vals = None (or all ones) for the textbook layer."""

    def __init__(self, in_features, out_features, aggregator="mean", bias=True):
        super().__init__()
        assert aggregator in ("mean", "pool")
        self.aggregator = aggregator
        self.w_self = torch.nn.Linear(in_features, out_features, bias=bias)
        self.w_neigh = torch.nn.Linear(in_features, out_features, bias=False)
        self.w_pool = torch.nn.Linear(in_features, in_features) if aggregator == "pool" else None

    def forward(self, graph: CsrGraph, X):
        if self.aggregator == "mean":
            agg = spmm(graph, X, "mean")
        else:
            agg = spmm(graph, torch.relu(self.w_pool(X)), "max")
        return self.w_self(X) + self.w_neigh(agg)
