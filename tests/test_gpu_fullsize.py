"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(default partition parameters).  The oracle's OpenMP row loops finish these in seconds on the
box's host cores, so outputs are compared in full, element by element."""
import numpy as np
import pytest
import torch

import graphgen
import oracle
import paper_2403_14853_amd as isp
from gpu_util import assert_close, build, dev

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def _say(msg):
    print("[fullsize] " + msg, flush=True)


def _transpose_exact(A, w):
    At, _ = isp.csr_transpose_cached(A)
    ti, tj, tv, perm = At.export()
    o_ti, o_tj, o_perm, o_tv = oracle.transpose(w.n, w.n, w.indptr, w.indices, w.values)
    assert np.array_equal(ti.cpu().numpy(), o_ti), "t_indptr differs"
    assert np.array_equal(tj.cpu().numpy(), o_tj), "t_indices differs"
    assert np.array_equal(perm.cpu().numpy(), o_perm), "perm differs"
    if w.values is not None:
        assert np.array_equal(tv.cpu().numpy(), o_tv), "t_values differs"
    del ti, tj, tv, perm
    return At, (o_ti, o_tj, o_tv)


@pytest.mark.parametrize("k", [1, 3])
def test_spmm_forward_backward_full(k):
    _say("config %d: generating" % k)
    w = graphgen.make_config(k)
    A = build(w.indptr, w.indices, w.values)
    info = A.info()
    _say("n=%d nnz=%d max_degree=%d hub_rows=%d items=%d" % (w.n, w.nnz, info["max_degree"], info["n_hub_rows"],
                                                             info["n_row_blocks"] + info["n_segments"]))
    if k == 3:
        assert info["max_degree"] > 10_000 and info["n_hub_rows"] > 0  # the nnz-split hub path is exercised
    X, dY = dev(w.X), dev(w.dY)
    Y = torch.empty_like(X)
    isp.spmm(A, X, Y)
    _say("forward: oracle")
    ref, mag = oracle.spmm(w.indptr, w.indices, w.values, w.X)
    assert_close(Y, ref, mag, "spmm forward")
    del ref, mag
    _say("transpose: oracle")
    At, (o_ti, o_tj, o_tv) = _transpose_exact(A, w)
    isp.spmm(At, dY, Y)
    _say("backward: oracle")
    ref, mag = oracle.spmm(o_ti, o_tj, o_tv, w.dY)
    assert_close(Y, ref, mag, "spmm backward")
    A.destroy()


def test_dense_degree_config2_spmm_and_sddmm_full():
    _say("config 2: generating")
    w = graphgen.make_config(2)
    A = build(w.indptr, w.indices, w.values)
    X, dY = dev(w.X), dev(w.dY)
    Y = torch.empty_like(X)
    isp.spmm(A, X, Y)
    _say("forward: oracle")
    ref, mag = oracle.spmm(w.indptr, w.indices, w.values, w.X)
    assert_close(Y, ref, mag, "spmm forward")
    del ref, mag
    # row-mean values: A 1 = 1 on non-empty rows (closed form, independent of the oracle)
    ones = torch.ones(w.n, 4, device="cuda")
    Y1 = torch.empty_like(ones)
    isp.spmm(A, ones, Y1)
    nonempty = torch.from_numpy(np.diff(w.indptr) > 0).cuda()
    assert torch.allclose(Y1[nonempty], torch.ones_like(Y1[nonempty]), rtol=0, atol=2e-5)
    assert torch.all(Y1[~nonempty] == 0)
    _say("transpose: oracle")
    At, (o_ti, o_tj, o_tv) = _transpose_exact(A, w)
    isp.spmm(At, dY, Y)
    ref, mag = oracle.spmm(o_ti, o_tj, o_tv, w.dY)
    assert_close(Y, ref, mag, "spmm backward")
    del ref, mag, o_ti, o_tj, o_tv
    dA = torch.empty(w.nnz, device="cuda")
    isp.sddmm(A, dY, X, dA)
    _say("sddmm: oracle")
    ref, mag = oracle.sddmm(w.indptr, w.indices, w.values, w.dY, w.X)
    assert_close(dA, ref, mag, "sddmm")
    A.destroy()


def test_fusedmm_config4_full():
    _say("config 4: generating")
    w = graphgen.make_config(4)
    assert w.values is None  # unit edge values: no value array is read
    A = build(w.indptr, w.indices, None)
    X, dY = dev(w.X), dev(w.dY)
    Y = torch.empty_like(X)
    isp.fusedmm(A, X, Y)
    _say("forward: oracle")
    ref, mag = oracle.fusedmm(w.indptr, w.indices, None, w.X)
    assert_close(Y, ref, mag, "fusedmm forward")
    del ref, mag
    At, _ = isp.csr_transpose_cached(A)
    dX = torch.empty_like(X)
    isp.fusedmm_backward(A, X, dY, dX)
    _say("backward: oracle (sequential scatter form)")
    ref, mag = oracle.fusedmm_backward(w.indptr, w.indices, None, w.X, w.dY)
    assert_close(dX, ref, mag, "fusedmm backward")
    A.destroy()


def test_sddmm_config3_full_two_column_passes():
    """Config 3 is large and has many columns, so SDDMM at d = 128 runs as two passes over 64-column halves
    (the second adds its partial dot products): every output against the oracle, and bitwise repeatable."""
    _say("config 3: generating")
    w = graphgen.make_config(3)
    A = build(w.indptr, w.indices, w.values)
    X, dY = dev(w.X), dev(w.dY)
    dA = torch.full((w.nnz,), float("nan"), device="cuda")
    isp.sddmm(A, dY, X, dA)
    _say("sddmm: oracle")
    ref, mag = oracle.sddmm(w.indptr, w.indices, w.values, w.dY, w.X)
    assert_close(dA, ref, mag, "sddmm")
    del ref, mag
    dA2 = torch.empty_like(dA)
    isp.sddmm(A, dY, X, dA2)
    assert torch.equal(dA, dA2)
    isp.sddmm(A, dY, X, dA, scale_by_a=True)
    _say("sddmm scaled: oracle")
    ref, mag = oracle.sddmm(w.indptr, w.indices, w.values, w.dY, w.X, scale_by_a=True)
    assert_close(dA, ref, mag, "sddmm scaled")
    A.destroy()


def test_wide_features_on_the_big_graph():
    """Rows wider than 128 floats on a graph of > 8 Mi entries: SpMM covers 128 columns per launch (the last
    launch 64 here) and SDDMM runs as 64-column passes that add up.  Every output against the oracle."""
    _say("config 3 at d = 192: generating")
    w = graphgen.make_config(3, d=192)
    A = build(w.indptr, w.indices, w.values)
    X, dY = dev(w.X), dev(w.dY)
    Y = torch.full_like(X, float("nan"))
    isp.spmm(A, X, Y)
    _say("spmm: oracle")
    ref, mag = oracle.spmm(w.indptr, w.indices, w.values, w.X)
    assert_close(Y, ref, mag, "spmm d=192")
    del ref, mag
    isp.spmm_reduce(A, X, Y, "mean")
    _say("mean: oracle")
    ref, _, mag = oracle.spmm_reduce(w.indptr, w.indices, w.values, w.X, "mean")
    assert_close(Y, ref, mag, "mean d=192")
    del ref, mag
    dA = torch.full((w.nnz,), float("nan"), device="cuda")
    isp.sddmm(A, dY, X, dA)
    _say("sddmm: oracle")
    ref, mag = oracle.sddmm(w.indptr, w.indices, w.values, w.dY, w.X)
    assert_close(dA, ref, mag, "sddmm d=192")
    A.destroy()


def test_max_and_mean_reductions_config3_full():
    """The benchmark graph at full size: max forward bit for bit (values and positions), max backward (which
    passes over every entry that no column selected - most entries of the long rows) and mean backward (values
    divided by the source rows' lengths, kept in the transpose workspace) against the oracle in full."""
    _say("config 3 reductions: generating")
    w = graphgen.make_config(3)
    A = build(w.indptr, w.indices, w.values)
    isp.csr_transpose_cached(A)
    X, dY = dev(w.X), dev(w.dY)
    Y = torch.full_like(X, float("nan"))
    arg = torch.full((w.n, w.d), -7, dtype=torch.int32, device="cuda")
    isp.spmm_reduce(A, X, Y, "max", arg)
    _say("max forward: oracle")
    ref, ref_arg, _ = oracle.spmm_reduce(w.indptr, w.indices, w.values, w.X, "max", want_mag=False)
    assert np.array_equal(Y.cpu().numpy().astype(np.float64), ref), "max: values differ"
    assert np.array_equal(arg.cpu().numpy(), ref_arg), "max: positions differ"
    del ref
    named = np.zeros(w.nnz, dtype=bool)
    named[ref_arg[ref_arg >= 0]] = True
    _say("entries named by some column: %.1f %%" % (100.0 * named.mean()))
    assert named.mean() < 0.75  # the pass-over path does real work on this graph
    dX = torch.full_like(X, float("nan"))
    isp.spmm_reduce_backward(A, dY, dX, "max", dev(ref_arg))
    _say("max backward: oracle")
    ref, mag = oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, w.values, w.dY, "max", ref_arg)
    assert_close(dX, ref, mag, "max backward")
    del ref, mag, ref_arg
    isp.spmm_reduce_backward(A, dY, dX, "mean")
    _say("mean backward: oracle")
    ref, mag = oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, w.values, w.dY, "mean")
    assert_close(dX, ref, mag, "mean backward")
    A.destroy()
