"""The autograd wrappers route gradients to the right kernels: dX through the cached transpose,
dA through SDDMM, FusedMM through its two backward passes.  Checked against the CPU oracle."""
import numpy as np
import pytest
import torch

import graphgen
import oracle
from gpu_util import assert_close, dev

pytestmark = pytest.mark.gpu


def test_spmm_autograd_matches_oracle_gradients():
    from paper_2403_14853_amd import autograd as ag
    w = graphgen.make_config(1, shrink=32)
    values = dev(w.values).requires_grad_(True)
    g = ag.SparseGraph(dev(w.indptr), dev(w.indices), values)
    X = dev(w.X).requires_grad_(True)
    W = dev(w.dY)
    for epoch in range(2):  # the second epoch reuses the cached transpose
        X.grad = values.grad = None
        Y = ag.spmm(g, X)
        (Y * W).sum().backward()
        assert g.handle.info()["has_cached_transpose"] == 1
        ti, tj, perm, tv = oracle.transpose(w.n, w.n, w.indptr, w.indices, w.values)
        assert_close(X.grad, *oracle.spmm(ti, tj, tv, w.dY), "dX epoch %d" % epoch)
        assert_close(values.grad, *oracle.sddmm(w.indptr, w.indices, w.values, w.dY, w.X), "dA epoch %d" % epoch)
        assert_close(Y.detach(), *oracle.spmm(w.indptr, w.indices, w.values, w.X), "Y epoch %d" % epoch)


def test_two_layer_gcn_step_runs_and_matches_dense_torch():
    """A 2-layer GCN step with real GEMMs: the sparse path against torch's dense autograd."""
    from paper_2403_14853_amd import autograd as ag
    w = graphgen.make_config(1, shrink=128)
    n, d, h, c = w.n, 32, 16, 7
    torch.manual_seed(0)
    X = torch.randn(n, d, device="cuda")
    W1 = torch.randn(d, h, device="cuda", requires_grad=True)
    W2 = torch.randn(h, c, device="cuda", requires_grad=True)
    g = ag.SparseGraph(dev(w.indptr), dev(w.indices), dev(w.values))
    out = ag.spmm(g, torch.relu(ag.spmm(g, X @ W1)) @ W2)
    out.square().mean().backward()
    g1, g2 = W1.grad.clone(), W2.grad.clone()
    # dense reference (fp64) built from the same CSR
    A = torch.zeros(n, n, dtype=torch.float64, device="cuda")
    rows = torch.from_numpy(np.repeat(np.arange(n), np.diff(w.indptr))).cuda()
    A.index_put_((rows, dev(w.indices).long()), dev(w.values).double(), accumulate=True)
    V1 = W1.detach().double().requires_grad_(True)
    V2 = W2.detach().double().requires_grad_(True)
    ref = A @ (torch.relu(A @ (X.double() @ V1)) @ V2)
    ref.square().mean().backward()
    assert torch.allclose(out.detach().double(), ref.detach(), rtol=1e-4, atol=1e-4)
    assert torch.allclose(g1.double(), V1.grad, rtol=1e-3, atol=1e-4)
    assert torch.allclose(g2.double(), V2.grad, rtol=1e-3, atol=1e-4)


def test_fusedmm_autograd():
    from paper_2403_14853_amd import autograd as ag
    w = graphgen.make_config(4, shrink=64)
    g = ag.SparseGraph(dev(w.indptr), dev(w.indices), None)
    X = dev(w.X).requires_grad_(True)
    Y = ag.fusedmm(g, X)
    (Y * dev(w.dY)).sum().backward()
    assert_close(Y.detach(), *oracle.fusedmm(w.indptr, w.indices, None, w.X), "fusedmm")
    assert_close(X.grad, *oracle.fusedmm_backward(w.indptr, w.indices, None, w.X, w.dY), "fusedmm dX")


def test_trained_edge_values_reach_the_cached_transpose():
    """Edge values as a trainable leaf: an in-place update between epochs must show up in the next
    epoch's forward (the handle reads the tensor's storage) and backward (the cached transpose's values are
    gathered again; structure and permutation stay cached)."""
    from paper_2403_14853_amd import autograd as ag
    w = graphgen.make_config(1, shrink=32)
    values = dev(w.values).requires_grad_(True)
    g = ag.SparseGraph(dev(w.indptr), dev(w.indices), values)
    X = dev(w.X).requires_grad_(True)
    W = dev(w.dY)
    cur = w.values.copy()
    for epoch in range(3):
        values.grad = None
        X.grad = None
        Y = ag.spmm(g, X)
        (Y * W).sum().backward()
        ti, tj, perm, tv = oracle.transpose(w.n, w.n, w.indptr, w.indices, cur)
        assert_close(Y.detach(), *oracle.spmm(w.indptr, w.indices, cur, w.X), "Y epoch %d" % epoch)
        assert_close(X.grad, *oracle.spmm(ti, tj, tv, w.dY), "dX epoch %d" % epoch)
        dA, mag = oracle.sddmm(w.indptr, w.indices, cur, w.dY, w.X)
        assert_close(values.grad, dA, mag, "dA epoch %d" % epoch)
        # the gradient step, taken from the oracle's gradient (no expected value may depend on the GPU path)
        # and written into the leaf tensor in place, as an optimizer would
        cur = (cur - 1e-3 * dA).astype(np.float32)
        with torch.no_grad():
            values.copy_(dev(cur))
    assert g.handle.info()["has_cached_transpose"] == 1


@pytest.mark.parametrize("reduce", ["mean", "min", "max"])
def test_matmul_with_the_other_reductions(reduce):
    """matmul(graph, X, reduce) as the paper's interface offers it: forward against the oracle (min / max bit
    for bit), and the gradient with respect to X through the cached transpose."""
    from paper_2403_14853_amd import autograd as ag
    w = graphgen.make_config(1, shrink=32)
    g = ag.SparseGraph(dev(w.indptr), dev(w.indices), dev(w.values))
    X = dev(w.X).requires_grad_(True)
    W = dev(w.dY)
    ref, ref_arg, mag = oracle.spmm_reduce(w.indptr, w.indices, w.values, w.X, reduce)
    for epoch in range(2):
        X.grad = None
        Y = ag.matmul(g, X, reduce)
        (Y * W).sum().backward()
        if reduce == "mean":
            assert_close(Y.detach(), ref, mag, "mean forward")
        else:
            assert np.array_equal(Y.detach().cpu().numpy().astype(np.float64), ref)
        assert_close(X.grad, *oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, w.values, w.dY, reduce, ref_arg),
                     "%s dX epoch %d" % (reduce, epoch))
    assert torch.equal(ag.matmul(g, X.detach(), "sum"), ag.spmm(g, X.detach()))
    with pytest.raises(ValueError):
        ag.matmul(g, X, "prod")
    trainable = ag.SparseGraph(dev(w.indptr), dev(w.indices), dev(w.values).requires_grad_(True))
    with pytest.raises(NotImplementedError):
        ag.matmul(trainable, X, reduce)
