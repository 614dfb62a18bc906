"""GPU parity of the mean / min / max reductions and their backward (via the cached transpose).
min / max values and positions are compared bit for bit (both sides decide in fp32)."""
import os

import numpy as np
import pytest
import torch

import graphgen
import oracle
import paper_2403_14853_amd as isp
from gpu_util import assert_close, build, dev

pytestmark = pytest.mark.gpu


@pytest.fixture
def small_partition():
    os.environ.update(ISP_HUB_THRESHOLD="24", ISP_SEGMENT_LEN="16", ISP_BLOCK_COST="32")
    yield
    for k in ("ISP_HUB_THRESHOLD", "ISP_SEGMENT_LEN", "ISP_BLOCK_COST"):
        os.environ.pop(k, None)


def _check(indptr, indices, values, n_rows, n_cols, d, seed, integer_inputs=False):
    rng = np.random.default_rng(seed)
    if integer_inputs:  # many equal products: ties must resolve to the first entry on both sides
        values = rng.integers(-1, 2, size=len(indices)).astype(np.float32)
        X = rng.integers(-2, 3, size=(n_cols, d)).astype(np.float32)
    else:
        X = rng.standard_normal((n_cols, d)).astype(np.float32)
    G = rng.standard_normal((n_rows, d)).astype(np.float32)
    A = build(indptr, indices, values, n_cols=n_cols)
    isp.csr_transpose_cached(A)
    Xd, Gd = dev(X), dev(G)
    for reduce in ("mean", "min", "max"):
        print("[reduce] %s d=%d n=%d" % (reduce, d, n_rows), flush=True)
        Y = torch.full((n_rows, d), float("nan"), device="cuda")
        arg = torch.full((n_rows, d), -7, dtype=torch.int32, device="cuda") if reduce != "mean" else None
        isp.spmm_reduce(A, Xd, Y, reduce, arg)
        ref, ref_arg, mag = oracle.spmm_reduce(indptr, indices, values, X, reduce)
        if reduce == "mean":
            assert_close(Y, ref, mag, "mean")
        else:
            assert np.array_equal(Y.cpu().numpy().astype(np.float64), ref), reduce + ": values differ"
            assert np.array_equal(arg.cpu().numpy(), ref_arg), reduce + ": positions differ"
        Y2 = torch.empty_like(Y)
        isp.spmm_reduce(A, Xd, Y2, reduce, arg)
        assert torch.equal(Y, Y2)  # run-to-run bitwise determinism
        dX = torch.full((n_cols, d), float("nan"), device="cuda")
        isp.spmm_reduce_backward(A, Gd, dX, reduce, arg)
        ref, mag = oracle.spmm_reduce_backward(n_cols, indptr, indices, values, G, reduce, ref_arg)
        assert_close(dX, ref, mag, reduce + " backward")
    # 'sum' routes to the plain SpMM
    Y = torch.empty(n_rows, d, device="cuda")
    isp.spmm_reduce(A, Xd, Y, "sum")
    ref, mag = oracle.spmm(indptr, indices, values, X)
    assert_close(Y, ref, mag, "sum")
    A.destroy()


# widths that are multiples of 4 take the grouped min / max kernel, 102 and 130 the generic one with float2
# lanes, 1 and 5 with scalar lanes
@pytest.mark.parametrize("d", [1, 5, 64, 100, 102, 128, 130, 200])
def test_reduce_small_graph_many_items(small_partition, d):
    w = graphgen.make_config(1, shrink=128)
    _check(w.indptr, w.indices, w.values, w.n, w.n, d, seed=d)


def test_reduce_ties_first_entry_wins(small_partition):
    w = graphgen.make_config(1, shrink=128)
    _check(w.indptr, w.indices, w.values, w.n, w.n, 32, seed=1, integer_inputs=True)


def test_reduce_rectangular_unsorted_duplicates_and_empty_rows(small_partition):
    indptr, indices, values = graphgen.random_csr(500, 301, 6000, 9, sorted_cols=False, allow_dup=True)
    _check(indptr, indices, values, 500, 301, 48, seed=2)
    w = graphgen.make_config(4, shrink=256)  # half the rows empty, no value array
    _check(w.indptr, w.indices, None, w.n, w.n, 16, seed=3)


def test_reduce_default_partition_config1():
    w = graphgen.make_config(1, shrink=4)
    _check(w.indptr, w.indices, w.values, w.n, w.n, 128, seed=4)


def test_backward_ignores_positions_outside_the_matrix(small_partition):
    """The min / max backward first marks which stored entries its arg array names.  arg is the caller's
    memory: positions outside [0, nnz) (the -1 of empty rows, or junk) must be passed over, not written
    through, and contribute nothing."""
    w = graphgen.make_config(1, shrink=128)
    d, nnz = 40, len(w.indices)
    rng = np.random.default_rng(11)
    X = rng.standard_normal((w.n, d)).astype(np.float32)
    G = rng.standard_normal((w.n, d)).astype(np.float32)
    _, ref_arg, _ = oracle.spmm_reduce(w.indptr, w.indices, w.values, X, "max")
    junk = rng.random(ref_arg.shape) < 0.2
    bad = rng.choice(np.array([-7, -2**31, nnz, nnz + 1000, 2**31 - 1], dtype=np.int64), size=ref_arg.shape)
    arg_in = np.where(junk, bad, ref_arg).astype(np.int32)
    arg_ref = np.where(junk, -1, ref_arg).astype(np.int32)   # what the definition makes of them: no entry
    A = build(w.indptr, w.indices, w.values)
    isp.csr_transpose_cached(A)
    dX = torch.full((w.n, d), float("nan"), device="cuda")
    isp.spmm_reduce_backward(A, dev(G), dX, "max", dev(arg_in))
    ref, mag = oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, w.values, G, "max", arg_ref)
    assert_close(dX, ref, mag, "max backward with junk positions")
    A.destroy()


def test_reduce_argument_errors():
    w = graphgen.make_config(0)
    A = build(w.indptr, w.indices, w.values)
    X = torch.ones(w.n, 8, device="cuda")
    Y = torch.empty_like(X)
    with pytest.raises(isp.IspError) as e:  # min without an arg array
        isp.spmm_reduce(A, X, Y, "min", None)
    assert e.value.status_name == "ISP_EINVAL"
    with pytest.raises(isp.IspError) as e:  # backward before the transpose exists
        isp.spmm_reduce_backward(A, X, Y, "mean")
    assert e.value.status_name == "ISP_EINVAL"
    A.destroy()
