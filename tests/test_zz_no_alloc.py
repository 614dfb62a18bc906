"""isp_spmm_static_scratch (SpMM whose hub-row partial sums live in the library's static device array, for
callers that cannot allocate): same results as isp_spmm, bit for bit, and within the SpMM tolerance of the
oracle; two calls in a row, the second on a smaller input, share the array.  Collected last."""
import os

import numpy as np
import pytest
import torch

import graphgen
import oracle
import paper_2403_14853_amd as isp
from gpu_util import assert_close, build, dev

pytestmark = pytest.mark.gpu


def _both(w, d=None, transpose=False):
    """(static-scratch result, isp_spmm result, oracle result, oracle scale, handle info) for workload w."""
    A = build(w.indptr, w.indices, w.values)
    H = A
    indptr, indices, values = w.indptr, w.indices, w.values
    if transpose:
        H, _ = isp.csr_transpose_cached(A)
        indptr, indices, _, values = oracle.transpose(w.n, w.n, w.indptr, w.indices, w.values)
    Xh = w.X if d is None else w.X[:, :d].copy()
    X = dev(Xh)
    Y0 = torch.full_like(X, float("nan"))
    Y1 = torch.full_like(X, float("nan"))
    isp.spmm(H, X, Y0)
    isp.spmm_static_scratch(H, X, Y1)
    torch.cuda.synchronize()
    ref, mag = oracle.spmm(indptr, indices, values, Xh)
    info = H.info()
    return Y1, Y0, ref, mag, info, A


def test_two_calls_in_a_row_second_smaller():
    big = graphgen.make_config(1)               # 2.4 M entries, hub rows of up to 10,294 entries
    small = graphgen.make_config(1, shrink=8)   # the same recipe an eighth the size
    seen = []
    for w, d, tr in ((big, None, False), (small, 64, False), (big, None, True), (small, 100, True)):
        print("static scratch: %s d=%s transpose=%s" % (w.name, d or w.d, tr), flush=True)
        Y1, Y0, ref, mag, info, A = _both(w, d, tr)
        assert 0 < info["n_segments"] <= 32768, info  # the scratch is really used, and within its limit
        seen.append(info["n_segments"])
        assert torch.equal(Y1, Y0), "static-scratch SpMM differs from isp_spmm"
        assert_close(Y1, ref, mag, "static-scratch spmm on " + w.name)
        A.destroy()
    assert seen[1] < seen[0]  # the second call used fewer partial rows than the first left behind


def test_repeat_is_bitwise_identical_and_interleaves_with_isp_spmm():
    w = graphgen.make_config(1, shrink=4)
    A = build(w.indptr, w.indices, w.values)
    X = dev(w.X)
    outs = []
    for k in range(3):
        Y = torch.empty_like(X)
        isp.spmm_static_scratch(A, X, Y)
        Z = torch.empty_like(X)
        isp.spmm(A, X, Z)  # the handle's own scratch in between
        outs.append((Y, Z))
    torch.cuda.synchronize()
    for Y, Z in outs:
        assert torch.equal(Y, outs[0][0]) and torch.equal(Z, Y)
    A.destroy()


def test_too_many_segments_is_rejected_cleanly():
    w = graphgen.make_config(1)
    old = {k: os.environ.get(k) for k in ("ISP_HUB_THRESHOLD", "ISP_SEGMENT_LEN", "ISP_BLOCK_COST")}
    os.environ.update(ISP_HUB_THRESHOLD="8", ISP_SEGMENT_LEN="8", ISP_BLOCK_COST="16")
    try:
        A = build(w.indptr, w.indices, w.values)
    finally:
        for k, v in old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
    assert A.info()["n_segments"] > 32768
    X = dev(w.X)
    Y = torch.zeros_like(X)
    with pytest.raises(isp.IspError) as e:
        isp.spmm_static_scratch(A, X, Y)
    assert e.value.status_name == "ISP_EUNSUPPORTED"
    torch.cuda.synchronize()
    assert float(Y.abs().max()) == 0.0  # nothing was launched
    ref, mag = oracle.spmm(w.indptr, w.indices, w.values, w.X)
    isp.spmm(A, X, Y)  # the ordinary entry point still serves the same handle
    assert_close(Y, ref, mag, "isp_spmm after the rejection")
    A.destroy()


def test_no_segments_and_empty_matrix():
    w = graphgen.make_config(0)  # no hub rows at all
    A = build(w.indptr, w.indices, w.values)
    X = dev(w.X)
    Y, Z = torch.empty_like(X), torch.empty_like(X)
    isp.spmm_static_scratch(A, X, Y)
    isp.spmm(A, X, Z)
    assert torch.equal(Y, Z)
    A.destroy()
    E = build(np.zeros(6, dtype=np.int64), np.zeros(0, dtype=np.int32), None, n_cols=4)
    Ye = torch.full((5, 8), 7.0, device="cuda")
    isp.spmm_static_scratch(E, torch.zeros(4, 8, device="cuda"), Ye)
    assert float(Ye.abs().max()) == 0.0
    E.destroy()
