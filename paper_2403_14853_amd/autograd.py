"""Thin ``torch.autograd.Function`` wrappers over the C ABI, so the sparse operations can sit
inside an ordinary PyTorch training step (the role of the paper's C++ wrapper that connects
forward and backward propagation to the kernels, Section 3.1).  Everything numerical still runs
in the library's HIP kernels; these classes only route tensors and remember what backward needs.

``SparseGraph`` owns the handle; its transpose is built on the first backward and cached in the
handle for all later epochs (Section 3.3).
"""
from __future__ import annotations

import torch

from . import binding as _b


class SparseGraph:
    """A CSR matrix on the GPU plus its library handle.  ``values`` may be a leaf tensor that
    requires grad; its gradient is the SDDMM of (dY, X)."""

    def __init__(self, indptr, indices, values=None, n_cols=None):
        self.indptr, self.indices, self.values = indptr, indices, values
        self.handle = _b.csr_build(indptr, indices, None if values is None else values.detach(), n_cols=n_cols)
        self.n_rows, self.n_cols, self.nnz = self.handle.n_rows, self.handle.n_cols, self.handle.nnz
        self._values_version = None if values is None else values._version

    def sync_values(self):
        """The handle reads ``values``' storage directly.  When an optimizer step has rewritten it in place
        since the last call, the cached transpose has to pick the new values up (its structure, permutation
        and partition stay cached)."""
        if self.values is not None and self.values._version != self._values_version:
            _b.csr_values_changed(self.handle)
            self._values_version = self.values._version

    def transpose(self):
        self.sync_values()
        return _b.csr_transpose_cached(self.handle)[0]


class _SpMM(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, values, X):
        X = X.contiguous()
        Y = torch.empty(graph.n_rows, X.shape[1], device=X.device, dtype=torch.float32)
        _b.spmm(graph.handle, X, Y)
        ctx.graph = graph
        ctx.save_for_backward(X)
        ctx.need_dA = values is not None and values.requires_grad
        return Y

    @staticmethod
    def backward(ctx, dY):
        (X,) = ctx.saved_tensors
        graph = ctx.graph
        dY = dY.contiguous()
        dX = dA = None
        if ctx.needs_input_grad[2]:
            dX = torch.empty(graph.n_cols, dY.shape[1], device=dY.device, dtype=torch.float32)
            _b.spmm(graph.transpose(), dY, dX)  # cached after the first call
        if ctx.need_dA:
            dA = torch.empty(graph.nnz, device=dY.device, dtype=torch.float32)
            _b.sddmm(graph.handle, dY, X, dA)
        return None, dA, dX


def spmm(graph: SparseGraph, X):
    """Differentiable Y = A X (with respect to X and, if ``graph.values`` requires grad, to the values)."""
    return _SpMM.apply(graph, graph.values, X)


class _SpMMReduce(torch.autograd.Function):
    """Y = reduce over each row's stored entries of a_p X[col_p] for 'mean', 'min', 'max' (Sections 3.4, 3.5);
    min / max remember the position of the winning entry per output element for the backward."""

    @staticmethod
    def forward(ctx, graph, X, reduce):
        X = X.contiguous()
        d = X.shape[1]
        Y = torch.empty(graph.n_rows, d, device=X.device, dtype=torch.float32)
        arg = None if reduce == "mean" else torch.empty(graph.n_rows, d, device=X.device, dtype=torch.int32)
        _b.spmm_reduce(graph.handle, X, Y, reduce, arg)
        ctx.graph, ctx.reduce, ctx.arg = graph, reduce, arg
        return Y

    @staticmethod
    def backward(ctx, dY):
        graph = ctx.graph
        graph.transpose()  # built on the first backward, cached afterwards
        dY = dY.contiguous()
        dX = torch.empty(graph.n_cols, dY.shape[1], device=dY.device, dtype=torch.float32)
        _b.spmm_reduce_backward(graph.handle, dY, dX, ctx.reduce, ctx.arg)
        return None, dX, None


def matmul(graph: SparseGraph, X, reduce: str = "sum"):
    """The paper's matmul(sparse, dense, reduce) (Section 3.5): reduce in 'sum' | 'mean' | 'min' | 'max'.
    Differentiable with respect to X; with respect to the edge values for 'sum' only."""
    if reduce == "sum":
        return spmm(graph, X)
    if reduce not in ("mean", "min", "max"):
        raise ValueError("reduce must be 'sum', 'mean', 'min' or 'max'")
    if graph.values is not None and graph.values.requires_grad:
        raise NotImplementedError("gradients with respect to the edge values exist for reduce='sum' only")
    return _SpMMReduce.apply(graph, X, reduce)


class _FusedMM(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, X):
        X = X.contiguous()
        Y = torch.empty_like(X)
        _b.fusedmm(graph.handle, X, Y)
        ctx.graph = graph
        ctx.save_for_backward(X)
        return Y

    @staticmethod
    def backward(ctx, dY):
        (X,) = ctx.saved_tensors
        graph = ctx.graph
        graph.transpose()
        dX = torch.empty_like(X)
        _b.fusedmm_backward(graph.handle, X, dY.contiguous(), dX)
        return None, dX


def fusedmm(graph: SparseGraph, X):
    """Differentiable sigmoid FusedMM: y_i = sum_j a_ij sigmoid(<x_i, x_j>) x_j (with respect to X only)."""
    if graph.values is not None and graph.values.requires_grad:
        raise NotImplementedError("FusedMM has no gradient with respect to the edge values")
    return _FusedMM.apply(graph, X)
