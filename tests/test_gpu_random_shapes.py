"""Seeded sweep over random matrix shapes, feature widths, partition parameters and CSR
irregularities (unsorted rows, repeated columns, missing value array, ld > d): every operation
against the oracle."""
import os

import numpy as np
import pytest
import torch

import graphgen
import oracle
import paper_2403_14853_amd as isp
from gpu_util import assert_close, build, dev

pytestmark = pytest.mark.gpu

WIDTHS = [1, 2, 4, 7, 8, 12, 16, 24, 32, 36, 48, 64, 72, 96, 100, 128, 132, 160, 192, 256, 260, 320, 512]


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    square = bool(rng.integers(0, 2))
    n_rows = int(rng.integers(1, 2500))
    n_cols = n_rows if square else int(rng.integers(1, 2500))
    nnz = int(rng.integers(0, 30000))
    d = int(rng.choice(WIDTHS))
    env = dict(ISP_HUB_THRESHOLD=str(int(rng.choice([8, 24, 100, 512]))),
               ISP_SEGMENT_LEN=str(int(rng.choice([8, 16, 64, 512]))),
               ISP_BLOCK_COST=str(int(rng.choice([16, 32, 100, 256]))))
    c = dict(square=square, n_rows=n_rows, n_cols=n_cols, nnz=nnz, d=d, env=env,
             sorted_cols=bool(rng.integers(0, 2)), allow_dup=bool(rng.integers(0, 2)),
             has_values=bool(rng.integers(0, 4)), pad=int(rng.choice([0, 0, 4, 12])), skew=bool(rng.integers(0, 2)))
    # column bands of the hub rows (drawn last, so the fields above keep their values per seed)
    env["ISP_BANDS"] = str(int(rng.choice([1, 2, 8, 32])))
    env["ISP_MIN_PIECE"] = str(int(rng.choice([4, 16, 64, 256])))
    # the packed SpMM layout: off, or rows above a small threshold cut into pieces that share work items
    env["ISP_MID_THRESHOLD"] = str(int(rng.choice([0, 8, 20, 64])))
    return c


# ISP_RANDOM_SHAPES=N widens the sweep for a one-off soak of the host and partition logic
@pytest.mark.parametrize("seed", range(int(os.environ.get("ISP_RANDOM_SHAPES", "48"))))
def test_random_shape(seed):
    c = _case(seed)
    print("[random-shape] seed=%d %s" % (seed, {k: v for k, v in c.items()}), flush=True)
    os.environ.update(c["env"])
    try:
        indptr, indices, values = graphgen.random_csr(c["n_rows"], c["n_cols"], c["nnz"], seed, sorted_cols=c["sorted_cols"],
                                                      allow_dup=c["allow_dup"])
        if c["skew"] and len(indices):  # pile a third of the entries onto a few hub columns / rows
            rng = np.random.default_rng(seed)
            hubs = rng.integers(0, c["n_cols"], size=3)
            pick = rng.random(len(indices)) < 0.33
            indices = np.where(pick, hubs[rng.integers(0, 3, size=len(indices))], indices).astype(np.int32)
        if not c["has_values"]:
            values = None
        n_rows, n_cols, d, ld = c["n_rows"], c["n_cols"], c["d"], c["d"] + c["pad"]
        rng = np.random.default_rng(seed + 5)
        Xf = rng.standard_normal((n_cols, ld)).astype(np.float32)
        Gf = rng.standard_normal((n_rows, ld)).astype(np.float32)
        X, G = Xf[:, :d], Gf[:, :d]
        Xd, Gd = dev(Xf)[:, :d], dev(Gf)[:, :d]
        A = build(indptr, indices, values, n_cols=n_cols)
        Ybuf = torch.full((n_rows, ld), 3.0, device="cuda")
        isp.spmm(A, Xd, Ybuf[:, :d])
        assert_close(Ybuf[:, :d].contiguous(), *oracle.spmm(indptr, indices, values, X), "spmm")
        assert torch.all(Ybuf[:, d:] == 3.0)
        At, _ = isp.csr_transpose_cached(A)
        ti, tj, tv, perm = At.export()
        o_ti, o_tj, o_perm, o_tv = oracle.transpose(n_rows, n_cols, indptr, indices, values)
        assert np.array_equal(ti.cpu().numpy(), o_ti) and np.array_equal(tj.cpu().numpy(), o_tj)
        assert np.array_equal(perm.cpu().numpy(), o_perm)
        if values is not None:
            assert np.array_equal(tv.cpu().numpy(), o_tv)
        dXbuf = torch.full((n_cols, ld), 3.0, device="cuda")
        isp.spmm(At, Gd, dXbuf[:, :d])
        assert_close(dXbuf[:, :d].contiguous(), *oracle.spmm(o_ti, o_tj, o_tv, G), "spmm backward")
        out = torch.full((len(indices),), float("nan"), device="cuda")
        isp.sddmm(A, Gd, Xd, out, scale_by_a=bool(seed % 2))
        assert_close(out, *oracle.sddmm(indptr, indices, values, G, X, scale_by_a=bool(seed % 2)), "sddmm")
        if c["square"] and (d <= 256 or d % 4 == 0):  # (FusedMM beyond 256 columns: multiples of 4, up to 1024)
            op = ("sigmoid", "dot", "one")[seed % 3]
            Xs = (0.3 * Xf).astype(np.float32)
            Xsd = dev(Xs)[:, :d]
            Yf = torch.full((n_rows, ld), 3.0, device="cuda")
            isp.fusedmm(A, Xsd, Yf[:, :d], op=op)
            assert_close(Yf[:, :d].contiguous(), *oracle.fusedmm(indptr, indices, values, Xs[:, :d], op=op), "fusedmm " + op)
            dXf = torch.full((n_rows, ld), 3.0, device="cuda")
            isp.fusedmm_backward(A, Xsd, Gd, dXf[:, :d], op=op)
            assert_close(dXf[:, :d].contiguous(), *oracle.fusedmm_backward(indptr, indices, values, Xs[:, :d], G, op=op),
                         "fusedmm backward " + op)
            assert torch.all(Yf[:, d:] == 3.0) and torch.all(dXf[:, d:] == 3.0)
        # one of the other reductions, forward (min / max bit for bit) and backward, on padded rows too
        reduce = ("mean", "min", "max")[(seed // 3) % 3]
        Yr = torch.full((n_rows, ld), 3.0, device="cuda")
        arg = torch.full((n_rows, d), -7, dtype=torch.int32, device="cuda") if reduce != "mean" else None
        isp.spmm_reduce(A, Xd, Yr[:, :d], reduce, arg)
        ref, ref_arg, mag = oracle.spmm_reduce(indptr, indices, values, X, reduce)
        if reduce == "mean":
            assert_close(Yr[:, :d].contiguous(), ref, mag, "mean")
        else:
            assert np.array_equal(Yr[:, :d].cpu().numpy().astype(np.float64), ref), reduce + ": values differ"
            assert np.array_equal(arg.cpu().numpy(), ref_arg), reduce + ": positions differ"
        dXr = torch.full((n_cols, ld), 3.0, device="cuda")
        isp.spmm_reduce_backward(A, Gd, dXr[:, :d], reduce, None if reduce == "mean" else dev(ref_arg))
        assert_close(dXr[:, :d].contiguous(), *oracle.spmm_reduce_backward(n_cols, indptr, indices, values, G, reduce, ref_arg),
                     reduce + " backward")
        assert torch.all(Yr[:, d:] == 3.0) and torch.all(dXr[:, d:] == 3.0)
        A.destroy()
    finally:
        for k in c["env"]:
            os.environ.pop(k, None)
