"""Close to the largest matrix the index types allow (nnz = 2.12e9, 99 % of 2^31 - 2): int64
offsets, grid sizes and the radix sort's tables at full scale.  About half a minute and ~50 GB of
host memory on the GPU machine; collected last, and skipped when ISP_SKIP_HUGE=1.  Outputs are checked
on sampled rows / columns against the oracle."""
import os
import time

import numpy as np
import pytest
import torch

import graphgen
import oracle
import paper_2403_14853_amd as isp
from gpu_util import assert_close, dev, sub_csr

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500),
              pytest.mark.skipif(os.environ.get("ISP_SKIP_HUGE") == "1", reason="ISP_SKIP_HUGE=1")]


def _say(msg, t0=[time.time()]):
    print("[huge %6.1fs] %s" % (time.time() - t0[0], msg), flush=True)


def test_two_billion_entries():
    n, d = 4_000_000, 16
    _say("generating ER graph n=%d, ~2.1e9 draws" % n)
    indptr, indices = graphgen.er_graph(n, 531.0, 7, self_loops=False)
    nnz = len(indices)
    _say("nnz = %d (limit %d)" % (nnz, 2**31 - 2))
    assert 1.9e9 < nnz < 2**31 - 1
    rng = np.random.default_rng(0)
    values = rng.random(nnz, dtype=np.float32) + 0.5
    X = rng.standard_normal((n, d)).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    _say("to device")
    d_indptr, d_indices, d_values = dev(indptr), dev(indices), dev(values)
    A = isp.csr_build(d_indptr, d_indices, d_values)
    info = A.info()
    _say("built: items=%d" % (info["n_row_blocks"] + info["n_segments"]))
    Xd, Gd = dev(X), dev(G)
    Y = torch.empty(n, d, device="cuda")
    isp.spmm(A, Xd, Y)
    torch.cuda.synchronize()
    _say("spmm done; sampled rows vs oracle")
    rows = np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, size=3000)]))
    sp, si, sv, pos = sub_csr(indptr, indices, values, rows)
    ref, mag = oracle.spmm(sp, si, sv, X)
    assert_close(Y[torch.from_numpy(rows).cuda()], ref, mag, "spmm (sampled rows)")
    out = torch.empty(nnz, device="cuda")
    isp.sddmm(A, Gd, Xd, out)
    torch.cuda.synchronize()
    ref, mag = oracle.sddmm(sp, si, sv, G[rows], X)
    assert_close(out[torch.from_numpy(pos).cuda()], ref, mag, "sddmm (sampled rows)")
    _say("transpose")
    At, _ = isp.csr_transpose_cached(A)
    torch.cuda.synchronize()
    ti, tj, tv, perm = At.export()
    _say("transpose done; checking structure")
    hist = np.bincount(indices, minlength=n)
    assert np.array_equal(ti.cpu().numpy(), np.concatenate([[0], np.cumsum(hist)]))
    del hist
    # stable order and consistency on sampled columns
    h_ti = ti.cpu().numpy()
    rows_of = None
    for c in np.concatenate([[0, n - 1], rng.integers(0, n, size=200)]):
        s, e = int(h_ti[c]), int(h_ti[c + 1])
        p = perm[s:e].cpu().numpy().astype(np.int64)
        assert np.all(np.diff(p) > 0), "entries of a column are not in source order"
        assert np.all(indices[p] == c)
        assert np.array_equal(tv[s:e].cpu().numpy(), values[p])
        src_rows = np.searchsorted(indptr, p, side="right") - 1
        assert np.array_equal(tj[s:e].cpu().numpy(), src_rows)
    dX = torch.empty(n, d, device="cuda")
    isp.spmm(At, Gd, dX)
    torch.cuda.synchronize()
    _say("backward spmm done; sampled rows vs the oracle's scatter-free definition")
    cols = np.unique(rng.integers(0, n, size=300))
    refs = np.zeros((len(cols), d))
    mags = np.zeros((len(cols), d))
    for k, c in enumerate(cols):
        s, e = int(h_ti[c]), int(h_ti[c + 1])
        p = perm[s:e].cpu().numpy().astype(np.int64)
        src_rows = np.searchsorted(indptr, p, side="right") - 1
        t = values[p].astype(np.float64)[:, None] * G[src_rows].astype(np.float64)
        refs[k], mags[k] = t.sum(0), np.abs(t).sum(0)
    assert_close(dX[torch.from_numpy(cols).cuda()], refs, mags, "spmm backward (sampled rows)")
    A.destroy()
    _say("ok")
