"""isp_csr_alias: a second handle on the same matrix with scratch of its own.  Every operation gives the
source handle's results bit for bit (and the oracle's within tolerance); calls on the source and on aliases
that overlap on several streams give the results of the same calls run one after the other; the error paths."""
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


def _all_ops(H, X, G, d, ops):
    """Every operation on handle H; returns the outputs in a fixed order."""
    n = X.shape[0]
    out = []
    new = lambda *shape, dtype=torch.float32: torch.full(shape, float("nan") if dtype == torch.float32 else -7,
                                                         device="cuda", dtype=dtype)
    Ht, _ = isp.csr_transpose_cached(H)
    if "spmm" in ops:
        Y = new(n, d); isp.spmm(H, X, Y); out.append(Y)
        dX = new(n, d); isp.spmm(Ht, G, dX); out.append(dX)
    if "sddmm" in ops:
        o = new(H.nnz); isp.sddmm(H, G, X, o); out.append(o)
        o2 = new(H.nnz); isp.sddmm(H, G, X, o2, scale_by_a=True); out.append(o2)
    if "fusedmm" in ops:
        Xs = X * 0.1
        for op in ("sigmoid", "dot"):
            Y = new(n, d); isp.fusedmm(H, Xs, Y, op=isp.binding.EDGE_OPS[op]); out.append(Y)
            dX = new(n, d); isp.fusedmm_backward(H, Xs, G, dX, op=isp.binding.EDGE_OPS[op]); out.append(dX)
    if "reduce" in ops:
        for red in ("mean", "min", "max"):
            Y = new(n, d)
            arg = None if red == "mean" else new(n, d, dtype=torch.int32)
            isp.spmm_reduce(H, X, Y, red, arg); out.append(Y)
            if arg is not None:
                out.append(arg)
            dX = new(n, d); isp.spmm_reduce_backward(H, G, dX, red, arg); out.append(dX)
    return out


def _same(a, b, what):
    assert len(a) == len(b)
    for k, (x, y) in enumerate(zip(a, b)):
        assert torch.equal(x, y), "%s: output %d of the alias differs from the source handle's" % (what, k)


@pytest.mark.parametrize("d", [32, 100, 128])
def test_alias_gives_the_source_handles_results(d):
    w = graphgen.make_config(1, shrink=4)  # R-MAT with hub rows: the partial rows are really used
    rng = np.random.default_rng(d)
    X = dev(rng.standard_normal((w.n, d)).astype(np.float32))
    G = dev(rng.standard_normal((w.n, d)).astype(np.float32))
    A = build(w.indptr, w.indices, w.values)
    assert A.info()["n_segments"] > 0
    isp.csr_transpose_cached(A)
    B = isp.csr_alias(A, max_d=d)
    assert B.info()["has_cached_transpose"] == 1
    ops = ("spmm", "sddmm", "fusedmm", "reduce")
    ra = _all_ops(A, X, G, d, ops)
    # poison the alias's workspace: nothing in it may need a particular starting value
    B._keep[1].fill_(0xFF)
    rb = _all_ops(B, X, G, d, ops)
    _same(ra, rb, "config 1 / 4, d=%d" % d)
    rb2 = _all_ops(B, X, G, d, ops)  # a second round on the used workspace
    _same(ra, rb2, "second round")
    # and the first of them against the oracle, so that "identical" is not "identically wrong"
    ref, mag = oracle.spmm(w.indptr, w.indices, w.values, X.cpu().numpy())
    assert_close(rb[0], ref, mag, "alias spmm")
    B.destroy()
    Y = torch.empty_like(X)
    isp.spmm(A, X, Y)  # the source handle outlives its alias
    assert torch.equal(Y, ra[0])


def test_alias_of_a_packed_layout_and_of_wide_fusedmm():
    _env(ISP_HUB_THRESHOLD=24, ISP_SEGMENT_LEN=16, ISP_BLOCK_COST=32, ISP_MID_THRESHOLD=10, ISP_MIN_PIECE=4, ISP_BANDS=8)
    w = graphgen.make_config(1, shrink=128)
    A = build(w.indptr, w.indices, w.values)
    info = A.info()
    assert info["spmm_pieces"] > info["n_segments"] > 0  # the pieces, not the segments, size the workspace
    isp.csr_transpose_cached(A)
    for d, max_d in ((128, 128), (600, 600), (600, 64)):  # (wider than max_d still works: one group per launch)
        rng = np.random.default_rng(d)
        X = dev(rng.standard_normal((w.n, d)).astype(np.float32))
        G = dev(rng.standard_normal((w.n, d)).astype(np.float32))
        B = isp.csr_alias(A, max_d=max_d)
        need = isp.csr_alias_workspace(A, max_d)
        groups = (max_d + 255) // 256
        assert need >= 1024 * max(info["spmm_pieces"], info["n_segments"] * groups)
        _same(_all_ops(A, X, G, d, ("spmm", "fusedmm")), _all_ops(B, X, G, d, ("spmm", "fusedmm")), "d=%d" % d)
        B.destroy()


def test_overlapping_calls_on_source_and_aliases():
    """Three handles on one matrix, three streams, no synchronisation between the streams: every result equals
    the one the same call gives when run alone."""
    w = graphgen.make_config(1, shrink=2)
    d = 64
    A = build(w.indptr, w.indices, w.values)
    isp.csr_transpose_cached(A)
    handles = [A, isp.csr_alias(A, max_d=d), isp.csr_alias(A, max_d=d)]
    rng = np.random.default_rng(5)
    Xs = [dev(rng.standard_normal((w.n, d)).astype(np.float32)) for _ in handles]
    Gs = [dev(rng.standard_normal((w.n, d)).astype(np.float32)) for _ in handles]

    def work(H, X, G, stream):
        Ht, _ = isp.csr_transpose_cached(H)
        outs = [torch.empty_like(X) for _ in range(4)]
        isp.spmm(H, X, outs[0], stream=stream)
        isp.spmm(Ht, G, outs[1], stream=stream)
        isp.fusedmm(H, X, outs[2], stream=stream)
        isp.fusedmm_backward(H, X, G, outs[3], stream=stream)
        return outs

    alone = []
    for H, X, G in zip(handles, Xs, Gs):
        alone.append(work(H, X, G, None))
        torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in handles]
    for rep in range(10):
        torch.cuda.synchronize()
        together = [work(H, X, G, s) for H, X, G, s in zip(handles, Xs, Gs, streams)]
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(zip(alone, together)):
            _same(a, b, "repeat %d, handle %d, overlapping" % (rep, k))


def test_alias_errors_and_staleness():
    w = graphgen.make_config(0)
    A = build(w.indptr, w.indices, w.values)
    X = dev(w.X)
    Y = torch.empty_like(X)
    B0 = isp.csr_alias(A)  # made before the transpose exists: it has none and cannot build one
    with pytest.raises(isp.IspError, match="source handle"):
        isp.csr_transpose_cached(B0)
    isp.spmm(B0, X, Y)
    At, _ = isp.csr_transpose_cached(A)
    B = isp.csr_alias(A)
    need = isp.csr_alias_workspace(A)
    with pytest.raises(AssertionError):
        isp.csr_alias(A, workspace=torch.empty(need - 256, dtype=torch.uint8, device="cuda"))
    lib = isp.load_library()
    import ctypes
    h = ctypes.c_void_p()
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    assert lib.isp_csr_alias(A.handle, 256, small.data_ptr(), need - 1, ctypes.byref(h)) == 1  # ISP_EINVAL
    assert b"too small" in lib.isp_last_error()
    big = torch.empty(need + 512, dtype=torch.uint8, device="cuda")
    assert lib.isp_csr_alias(A.handle, 256, big.data_ptr() + 4, need, ctypes.byref(h)) == 1
    assert b"aligned" in lib.isp_last_error()
    assert lib.isp_csr_alias(A.handle, 0, big.data_ptr(), need, ctypes.byref(h)) == 1
    assert lib.isp_csr_alias(None, 256, big.data_ptr(), need, ctypes.byref(h)) == 1
    with pytest.raises(isp.IspError, match="not an alias"):
        isp.csr_alias(B)
    with pytest.raises(isp.IspError, match="transpose"):
        isp.csr_alias(At)
    with pytest.raises(isp.IspError, match="not an alias"):
        isp.csr_values_changed(B)
    # values rewritten in place: aliases made before are refused, new ones see the new values
    vals = A._keep[2]
    vals.mul_(2.0)
    isp.csr_values_changed(A)
    with pytest.raises(isp.IspError, match="make a new one"):
        isp.spmm(B, X, Y)
    Bt, _ = isp.csr_transpose_cached(B)
    with pytest.raises(isp.IspError, match="make a new one"):
        isp.spmm(Bt, X, Y)
    C = isp.csr_alias(A)
    Ya = torch.empty_like(X)
    isp.spmm(A, X, Ya)
    isp.spmm(C, X, Y)
    assert torch.equal(Y, Ya)
    ref, mag = oracle.spmm(w.indptr, w.indices, w.values * np.float32(2.0), w.X)
    assert_close(Y, ref, mag, "alias after values_changed")
    Ct, _ = isp.csr_transpose_cached(C)
    dXa, dX = torch.empty_like(X), torch.empty_like(X)
    isp.spmm(At, X, dXa)
    isp.spmm(Ct, X, dX)
    assert torch.equal(dX, dXa)
