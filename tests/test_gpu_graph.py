"""The compute entry points only enqueue kernels on the given stream (no allocation, no memset,
no synchronisation), so they can be captured in a HIP graph.  Every replay is checked against the
eager result, with eager work and synchronisation between replays."""
import numpy as np
import pytest
import torch

import graphgen
import oracle
import paper_2403_14853_amd as isp
from gpu_util import assert_close, build, dev

pytestmark = pytest.mark.gpu


def test_graph_capture_and_replay_of_a_training_step():
    w = graphgen.make_config(1, shrink=8)
    A = build(w.indptr, w.indices, w.values)
    At, _ = isp.csr_transpose_cached(A)  # built before capture: a cache miss synchronises the stream
    X, dY = dev(w.X), dev(w.dY)
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    dA = torch.empty(w.nnz, device="cuda")

    def step():
        isp.spmm(A, X, Y)
        isp.spmm(isp.csr_transpose_cached(A)[0], dY, dX)  # cache hit: no device work, capturable
        isp.sddmm(A, dY, X, dA)

    step()
    torch.cuda.synchronize()
    eager = (Y.clone(), dX.clone(), dA.clone())
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        Y.fill_(float("nan")); dX.fill_(float("nan")); dA.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, eager[0]) and torch.equal(dX, eager[1]) and torch.equal(dA, eager[2]), "replay %d" % rep
        # eager work between replays, on new inputs, must not disturb the next replay
        X2 = torch.randn_like(X)
        Y2 = torch.empty_like(X)
        isp.spmm(A, X2, Y2)
        torch.cuda.synchronize()
    ref, mag = oracle.spmm(w.indptr, w.indices, w.values, w.X)
    assert_close(Y, ref, mag, "replayed spmm vs oracle")
    A.destroy()


def test_first_reduction_backward_inside_a_capture():
    """The mean and the min / max backward keep per-handle caches (scaled values, the inverse permutation) that
    the first call fills.  When that first call is being captured the fill must be part of the graph - nothing
    has run yet - and a later eager call must fill the cache itself."""
    w = graphgen.make_config(1, shrink=8)
    A = build(w.indptr, w.indices, w.values)
    isp.csr_transpose_cached(A)
    X, dY = dev(w.X), dev(w.dY)
    _, ref_arg, _ = oracle.spmm_reduce(w.indptr, w.indices, w.values, w.X, "max")
    arg = dev(ref_arg)
    dX_mean, dX_max = torch.full_like(X, float("nan")), torch.full_like(X, float("nan"))
    ref_mean = oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, w.values, w.dY, "mean")
    ref_max = oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, w.values, w.dY, "max", ref_arg)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):  # no warm-up of these two calls: their first use is captured
            isp.spmm_reduce_backward(A, dY, dX_mean, "mean")
            isp.spmm_reduce_backward(A, dY, dX_max, "max", arg)
    torch.cuda.synchronize()
    # eager calls before any replay: the captured fills have not run
    e_mean, e_max = torch.empty_like(X), torch.empty_like(X)
    isp.spmm_reduce_backward(A, dY, e_mean, "mean")
    isp.spmm_reduce_backward(A, dY, e_max, "max", arg)
    torch.cuda.synchronize()
    assert_close(e_mean, *ref_mean, "eager mean backward after a capture")
    assert_close(e_max, *ref_max, "eager max backward after a capture")
    for rep in range(3):
        dX_mean.fill_(float("nan")); dX_max.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(dX_mean, e_mean) and torch.equal(dX_max, e_max), "replay %d" % rep
    A.destroy()
