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
