"""Use from a GNN framework: the integration the paper's conclusion names as its goal.

A `Graph` owns the plan of a sparse matrix A and the plan of its transpose and offers the two
operations a message-passing layer is made of, both differentiable:

    aggregate(B, vals)      C = A.B                          (SpMM, the paper's operation)
    edge_scores(X, Y)       out[p] = <X[i_p], Y[j_p]>        (SDDMM on the same tile format)

Their gradients are the same two operations again: dB = A^T.dC, d(vals) = sddmm(dC, B),
dX = (A with values d(out)).Y, dY = (A^T with values d(out)).X.  Mixed precision as in the
forward pass: 16-bit operands (gradients are rounded to the operand type before they enter a
kernel), fp32 accumulation; results are fp32, except the gradients of 16-bit operands, which
the kernel rounds to that type as it stores them (acc_spmm_execute_c16).

torch supplies tensors, the current stream, the autograd tape and the index bookkeeping of the
transpose (a stable sort of the column ids); every product runs in the library's kernels.  There
is no fallback: without the shared library or a GPU, constructing a `Graph` raises.
"""
from __future__ import annotations

import numpy as np
import torch

from . import (ACC_SPMM_BF16, ACC_SPMM_FP16, acc_spmm_destroy, acc_spmm_execute, acc_spmm_execute_c16, acc_spmm_plan_device,
               acc_spmm_plan_stats, acc_spmm_sddmm, acc_spmm_update_values, make_options)

_VALUE_TYPES = {torch.float16: ACC_SPMM_FP16, torch.bfloat16: ACC_SPMM_BF16}


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _as_device(a, dtype, device):
    if isinstance(a, np.ndarray):
        a = torch.from_numpy(np.ascontiguousarray(a))
    return a.to(device=device, dtype=dtype).contiguous()


class Graph:
    """A sparse M x K matrix in CSR (sorted, distinct columns per row) prepared for SpMM and SDDMM.

    rowptr, colidx: int32 arrays (numpy or torch, any device).  vals: float16 or bfloat16 tensor of
    nnz values in CSR order; its dtype fixes the operand type of every later call.  `options` are
    fields of acc_spmm_options (reorder, load_balance, column_order, ...), applied to both plans.
    With transpose=False only the forward operations and d(vals) are available.
    """

    def __init__(self, M, K, rowptr, colidx, vals, transpose=True, device="cuda:0", **options):
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2501_09251_amd.gnn needs a GPU (there is no CPU path)")
        if not isinstance(vals, torch.Tensor) or vals.dtype not in _VALUE_TYPES:
            raise TypeError("vals must be a float16 or bfloat16 tensor")
        self.device = torch.device(device)
        self.M, self.K = int(M), int(K)
        self.dtype = vals.dtype
        self.rowptr = _as_device(rowptr, torch.int32, self.device)
        self.colidx = _as_device(colidx, torch.int32, self.device)
        self.nnz = int(self.colidx.numel())
        if self.rowptr.numel() != self.M + 1 or vals.numel() != self.nnz:
            raise ValueError("CSR array lengths do not match M / nnz")
        self.vals = vals.detach().to(self.device).contiguous()
        opt = make_options(keep_entry_map=1, value_type=_VALUE_TYPES[self.dtype], **options)
        self._plan = self._plan_t = None
        self._resident = self._resident_t = None    # (tensor, version) whose values each plan holds
        with torch.cuda.device(self.device):
            self._plan = acc_spmm_plan_device(self.M, self.K, self.nnz, self.rowptr, self.colidx, self.vals, opt)
            self._resident = (self.vals, self.vals._version)
            self.t_order = None
            if transpose:
                t_rowptr, t_colidx, self.t_order = self._transposed()
                t_vals = self.vals[self.t_order]
                self._plan_t = acc_spmm_plan_device(self.K, self.M, self.nnz, t_rowptr, t_colidx, t_vals, opt)
                self._resident_t = self._resident
            torch.cuda.synchronize()

    def _transposed(self):
        """CSR of A^T and, per entry of A^T, its position in A.  A stable sort by column keeps the
        entries of one column in row order, so the rows of A^T come out sorted."""
        counts = (self.rowptr[1:] - self.rowptr[:-1]).long()
        row_of = torch.repeat_interleave(torch.arange(self.M, device=self.device, dtype=torch.int32), counts)
        order = torch.argsort(self.colidx, stable=True)
        t_colidx = row_of[order].contiguous()
        t_rowptr = torch.zeros(self.K + 1, dtype=torch.int32, device=self.device)
        if self.nnz:
            t_rowptr[1:] = torch.cumsum(torch.bincount(self.colidx.long(), minlength=self.K), 0).int()
        return t_rowptr, t_colidx, order

    # ------------------------------------------------------------------ values held by the plans
    def _load(self, vals):
        if self._resident is None or self._resident[0] is not vals or self._resident[1] != vals._version:
            acc_spmm_update_values(self._plan, vals, _stream())
            self._resident = (vals, vals._version)

    def _load_t(self, vals):
        if self._plan_t is None:
            raise RuntimeError("this Graph was built with transpose=False")
        if self._resident_t is None or self._resident_t[0] is not vals or self._resident_t[1] != vals._version:
            acc_spmm_update_values(self._plan_t, vals[self.t_order], _stream())
            self._resident_t = (vals, vals._version)

    def _check_operand(self, name, T, rows):
        if T.dtype != self.dtype or T.dim() != 2 or T.shape[0] != rows or T.device != self.device:
            raise ValueError(f"{name} must be a {rows} x N {self.dtype} tensor on {self.device}")
        return T.contiguous()

    def _values(self, vals):
        if vals is None:
            return self.vals
        if vals.dtype != self.dtype or vals.numel() != self.nnz or vals.device != self.device:
            raise ValueError(f"vals must hold {self.nnz} {self.dtype} values on {self.device}")
        return vals.contiguous()

    # ------------------------------------------------------------------ raw products (no tape)
    def _spmm(self, vals, B, transposed=False, narrow=False):
        if transposed:
            self._load_t(vals)
            plan, rows = self._plan_t, self.K
        else:
            self._load(vals)
            plan, rows = self._plan, self.M
        C = torch.empty((rows, B.shape[1]), dtype=self.dtype if narrow else torch.float32, device=self.device)
        (acc_spmm_execute_c16 if narrow else acc_spmm_execute)(plan, B, B.shape[1], C, _stream())
        return C

    def _sddmm(self, X, Y):
        out = torch.empty(self.nnz, dtype=torch.float32, device=self.device)
        acc_spmm_sddmm(self._plan, X, Y, X.shape[1], out, 0, _stream())
        return out

    # ------------------------------------------------------------------ the two operations
    def aggregate(self, B, vals=None, narrow=False):
        """C = A.B as an fp32 M x N tensor (narrow=True: in the Graph's 16-bit dtype, rounded once from
        the fp32 accumulators, which halves the bytes written); B is K x N in the Graph's dtype.
        `vals` (nnz values in CSR order, e.g. attention weights) replaces the values of A for this
        call and may require a gradient; N must then be a width acc_spmm_sddmm accepts."""
        return _Aggregate.apply(self, self._values(vals), self._check_operand("B", B, self.K), bool(narrow))

    def edge_scores(self, X, Y):
        """out[p] = <X[i_p], Y[j_p]> for every stored entry p = (i_p, j_p), fp32, CSR order.
        X is M x N, Y is K x N, N a width acc_spmm_sddmm accepts."""
        X = self._check_operand("X", X, self.M)
        Y = self._check_operand("Y", Y, self.K)
        if X.shape[1] != Y.shape[1]:
            raise ValueError("X and Y must have the same number of columns")
        return _EdgeScores.apply(self, X, Y)

    def stats(self):
        return acc_spmm_plan_stats(self._plan)

    def close(self):
        for name in ("_plan", "_plan_t"):
            if getattr(self, name, None):
                acc_spmm_destroy(getattr(self, name))
                setattr(self, name, None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class _Aggregate(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, vals, B, narrow):
        ctx.graph = graph
        ctx.save_for_backward(vals, B)
        return graph._spmm(vals, B, narrow=narrow)

    @staticmethod
    def backward(ctx, dC):
        graph = ctx.graph
        vals, B = ctx.saved_tensors
        d16 = dC.to(graph.dtype).contiguous()
        d_vals = d_B = None
        if ctx.needs_input_grad[2]:
            d_B = graph._spmm(vals, d16, transposed=True, narrow=True)   # a gradient in B's own type
        if ctx.needs_input_grad[1]:
            d_vals = graph._sddmm(d16, B).to(graph.dtype)
        return None, d_vals, d_B, None


class _EdgeScores(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, X, Y):
        ctx.graph = graph
        ctx.save_for_backward(X, Y)
        return graph._sddmm(X, Y)

    @staticmethod
    def backward(ctx, d_out):
        graph = ctx.graph
        X, Y = ctx.saved_tensors
        g16 = d_out.to(graph.dtype).contiguous()
        d_X = d_Y = None
        if ctx.needs_input_grad[1]:
            d_X = graph._spmm(g16, Y, narrow=True)
        if ctx.needs_input_grad[2]:
            d_Y = graph._spmm(g16, X, transposed=True, narrow=True)
        return None, d_X, d_Y


class GraphConv(torch.nn.Module):
    """One graph-convolution layer, H' = A.(H W) + b: the dense product is torch's, the
    aggregation is `Graph.aggregate`.  H and W are in the Graph's 16-bit type; H' is fp32."""

    def __init__(self, graph, in_features, out_features, bias=True):
        super().__init__()
        self.graph = graph
        self.linear = torch.nn.Linear(in_features, out_features, bias=False, device=graph.device, dtype=graph.dtype)
        self.bias = torch.nn.Parameter(torch.zeros(out_features, device=graph.device)) if bias else None

    def forward(self, H, vals=None):
        out = self.graph.aggregate(self.linear(H), vals)   # fp32: the bias is added in fp32
        return out if self.bias is None else out + self.bias
