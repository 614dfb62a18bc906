"""The packed SpMM layout (rows above a threshold cut into column-band pieces that share work items, in a
derived copy of the matrix): forced onto small graphs with tiny thresholds so that a few thousand entries
span short-row blocks, piece blocks with many pieces each, pieces of one entry, cut rows with one piece and
with dozens.  SpMM forward / backward / mean against the oracle element by element, bit-identical repeats,
values rewritten in place, the static-scratch entry point, and the handle's report of the layout."""
import os

import numpy as np
import pytest
import torch

import graphgen
import oracle
import paper_2403_14853_amd as isp
from gpu_util import assert_close, build, dev

pytestmark = pytest.mark.gpu

KEYS = ("ISP_HUB_THRESHOLD", "ISP_SEGMENT_LEN", "ISP_BLOCK_COST", "ISP_MID_THRESHOLD", "ISP_MIN_PIECE", "ISP_BANDS")


def _env(**kw):
    for k in KEYS:
        os.environ.pop(k, None)
    for k, v in kw.items():
        os.environ[k] = str(v)


@pytest.fixture(autouse=True)
def _clean_env(request):
    print("\n[case] %s" % request.node.nodeid, flush=True)
    yield
    torch.cuda.synchronize()
    _env()


def _spmm_both_ways(w, d, seed, expect_packed=True):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((w.n, d)).astype(np.float32)
    G = rng.standard_normal((w.n, d)).astype(np.float32)
    A = build(w.indptr, w.indices, w.values)
    info = A.info()
    if expect_packed:
        deg = np.diff(w.indptr)
        assert info["spmm_mid_threshold"] > 0 and info["spmm_cut_rows"] == int((deg > info["spmm_mid_threshold"]).sum())
        assert info["spmm_pieces"] >= info["spmm_cut_rows"] > 0 and info["spmm_row_blocks"] > 0
    else:
        assert info["spmm_pieces"] == 0
    Y = torch.full((w.n, d), float("nan"), device="cuda")
    isp.spmm(A, dev(X), Y)
    ref, mag = oracle.spmm(w.indptr, w.indices, w.values, X)
    assert_close(Y, ref, mag, "packed spmm d=%d" % d)
    Y2 = torch.empty_like(Y)
    isp.spmm(A, dev(X), Y2)
    assert torch.equal(Y, Y2)
    At, _ = isp.csr_transpose_cached(A)
    ti, tj, _, tv = oracle.transpose(w.n, w.n, w.indptr, w.indices, w.values)
    dX = torch.full((w.n, d), float("nan"), device="cuda")
    isp.spmm(At, dev(G), dX)
    ref, mag = oracle.spmm(ti, tj, tv, G)
    assert_close(dX, ref, mag, "packed spmm backward d=%d" % d)
    return A, X, G, Y


@pytest.mark.parametrize("d", [1, 3, 32, 64, 100, 128, 130, 256, 300])
@pytest.mark.parametrize("mid,seg,min_piece,bands", [(10, 16, 4, 8), (6, 8, 4, 32), (40, 64, 8, 4)])
def test_forced_packed_layout_small_graph(d, mid, seg, min_piece, bands):
    _env(ISP_HUB_THRESHOLD=max(24, mid), ISP_SEGMENT_LEN=seg, ISP_BLOCK_COST=32, ISP_MID_THRESHOLD=mid,
         ISP_MIN_PIECE=min_piece, ISP_BANDS=bands)
    w = graphgen.make_config(1, shrink=128)
    A, X, G, Y = _spmm_both_ways(w, d, seed=d)
    # mean forward (rows divided by their length: short rows in the block, cut rows in the fix-up) and backward
    Ym = torch.full((w.n, d), float("nan"), device="cuda")
    isp.spmm_reduce(A, dev(X), Ym, "mean")
    ref, _, mag = oracle.spmm_reduce(w.indptr, w.indices, w.values, X, "mean")
    assert_close(Ym, ref, mag, "packed mean d=%d" % d)
    dXm = torch.full((w.n, d), float("nan"), device="cuda")
    isp.spmm_reduce_backward(A, dev(G), dXm, "mean")
    ref, mag = oracle.spmm_reduce_backward(w.n, w.indptr, w.indices, w.values, G, "mean")
    assert_close(dXm, ref, mag, "packed mean backward d=%d" % d)
    # the entry point with the static scratch shares the layout
    Ys = torch.full((w.n, d), float("nan"), device="cuda")
    isp.spmm_static_scratch(A, dev(X), Ys)
    assert torch.equal(Ys, Y)
    A.destroy()


def test_values_rewritten_in_place_reach_the_packed_copy():
    _env(ISP_HUB_THRESHOLD=24, ISP_SEGMENT_LEN=16, ISP_BLOCK_COST=32, ISP_MID_THRESHOLD=10, ISP_MIN_PIECE=4)
    w = graphgen.make_config(1, shrink=64)
    d = 64
    X = np.random.default_rng(0).standard_normal((w.n, d)).astype(np.float32)
    vals = dev(w.values.copy())
    A = isp.csr_build(dev(w.indptr), dev(w.indices), vals)
    assert A.info()["spmm_pieces"] > 0
    At, _ = isp.csr_transpose_cached(A)
    Y = torch.empty(w.n, d, device="cuda")
    isp.spmm(A, dev(X), Y)
    new = (np.random.default_rng(1).standard_normal(w.nnz)).astype(np.float32)
    vals.copy_(dev(new))
    isp.csr_values_changed(A)
    isp.spmm(A, dev(X), Y)
    assert_close(Y, *oracle.spmm(w.indptr, w.indices, new, X), "spmm after the values changed")
    ti, tj, _, tv = oracle.transpose(w.n, w.n, w.indptr, w.indices, new)
    isp.spmm(At, dev(X), Y)
    assert_close(Y, *oracle.spmm(ti, tj, tv, X), "backward after the values changed")
    A.destroy()


def test_unsorted_duplicated_rectangular_and_no_values():
    _env(ISP_HUB_THRESHOLD=24, ISP_SEGMENT_LEN=16, ISP_BLOCK_COST=32, ISP_MID_THRESHOLD=8, ISP_MIN_PIECE=4)
    for seed, (nr, nc, nz) in enumerate([(300, 200, 6000), (50, 4000, 3000), (2000, 37, 9000), (1, 500, 400)]):
        indptr, indices, values = graphgen.random_csr(nr, nc, nz, seed, sorted_cols=bool(seed % 2), allow_dup=True)
        for vals in (values, None):
            for d in (8, 36):
                X = np.random.default_rng(seed).standard_normal((nc, d)).astype(np.float32)
                A = build(indptr, indices, vals, n_cols=nc)
                Y = torch.full((nr, d), float("nan"), device="cuda")
                isp.spmm(A, dev(X), Y)
                assert_close(Y, *oracle.spmm(indptr, indices, vals, X), "packed spmm on a general CSR")
                A.destroy()


def test_layout_is_off_by_default_on_small_graphs_and_can_be_switched_off():
    w = graphgen.make_config(1, shrink=16)
    A, *_ = _spmm_both_ways(w, 32, seed=0, expect_packed=False)
    A.destroy()
    _env(ISP_MID_THRESHOLD=0)
    A, *_ = _spmm_both_ways(w, 32, seed=0, expect_packed=False)
    A.destroy()
