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


def _capture(fn):
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()  # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            fn()
    torch.cuda.synchronize()
    return g


def test_graph_with_the_packed_layout_the_static_scratch_and_the_one_pass_backward():
    """The packed SpMM layout (forced onto a small graph), the entry point whose scratch is the library's static
    array, and the one-pass FusedMM backward of a symmetric pattern, captured and replayed."""
    import os
    keys = dict(ISP_HUB_THRESHOLD="24", ISP_SEGMENT_LEN="16", ISP_BLOCK_COST="32", ISP_MID_THRESHOLD="10", ISP_MIN_PIECE="4")
    os.environ.update(keys)
    try:
        w = graphgen.make_config(1, shrink=16)
        A = build(w.indptr, w.indices, w.values)
    finally:
        for k in keys:
            os.environ.pop(k, None)
    info = A.info()
    assert info["spmm_pieces"] > 0
    isp.csr_transpose_cached(A)
    assert A.info()["symmetric_pattern"] == 1
    X, dY = dev((0.2 * w.X).astype(np.float32)), dev(w.dY)
    Y, Ys, dX = torch.empty_like(X), torch.empty_like(X), torch.empty_like(X)

    def step():
        isp.spmm(A, X, Y)
        isp.spmm_static_scratch(A, X, Ys)
        isp.fusedmm_backward(A, X, dY, dX)

    step()
    torch.cuda.synchronize()
    eager = (Y.clone(), dX.clone())
    g = _capture(step)
    for rep in range(3):
        Y.fill_(float("nan")); Ys.fill_(float("nan")); dX.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, eager[0]) and torch.equal(Ys, eager[0]) and torch.equal(dX, eager[1]), "replay %d" % rep
        isp.spmm(A, torch.randn_like(X), torch.empty_like(X))  # eager work in between
        torch.cuda.synchronize()
    assert_close(Y, *oracle.spmm(w.indptr, w.indices, w.values, (0.2 * w.X).astype(np.float32)), "replayed packed spmm")
    assert_close(dX, *oracle.fusedmm_backward(w.indptr, w.indices, w.values, (0.2 * w.X).astype(np.float32), w.dY),
                 "replayed one-pass backward")
    A.destroy()


def test_values_changed_reaches_graphs_captured_before_and_a_captured_refresh_replays():
    """isp_csr_values_changed does all its work in stream order: a graph captured earlier (mean backward with the
    per-entry values already filled, so the graph holds no fill pass) reads refreshed values after an eager
    refresh, and a refresh that is itself captured runs again on every replay."""
    w = graphgen.make_config(1, shrink=8)
    vals = dev(w.values.copy())
    A = isp.csr_build(dev(w.indptr), dev(w.indices), vals)
    isp.csr_transpose_cached(A)
    dY = dev(w.dY)
    dX = torch.empty_like(dY)
    isp.spmm_reduce_backward(A, dY, dX, "mean")  # fills value / row length eagerly
    torch.cuda.synchronize()
    g = _capture(lambda: isp.spmm_reduce_backward(A, dY, dX, "mean"))
    new = np.random.default_rng(3).standard_normal(w.nnz).astype(np.float32)
    vals.copy_(dev(new))
    isp.csr_values_changed(A)  # eager: regathers t_values and refills value / row length behind it
    torch.cuda.synchronize()
    ref = oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, new, w.dY, "mean")
    for rep in range(2):
        dX.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert_close(dX, *ref, "graph captured before the values changed, replay %d" % rep)
    # a captured refresh + backward: every replay picks up what the values hold at that moment
    g2 = _capture(lambda: (isp.csr_values_changed(A), isp.spmm_reduce_backward(A, dY, dX, "mean")))
    for seed in (5, 6):
        newer = np.random.default_rng(seed).standard_normal(w.nnz).astype(np.float32)
        vals.copy_(dev(newer))
        torch.cuda.synchronize()
        dX.fill_(float("nan"))
        g2.replay()
        torch.cuda.synchronize()
        assert_close(dX, *oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, newer, w.dY, "mean"),
                     "captured refresh, values of seed %d" % seed)
    A.destroy()
