"""Pins for the oracle's mean / min / max reductions and their backward (CPU only): dense brute
force written here, tie handling on small-integer inputs, closed forms, finite differences."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import graphgen
import oracle
from test_oracle_pins import _dense, _rows, small_csr


def _brute(indptr, indices, values, X, reduce):
    """Loop definition, products in fp32 for min / max (first winner on ties), fp64 for mean."""
    n, d = len(indptr) - 1, X.shape[1]
    Y = np.zeros((n, d))
    arg = -np.ones((n, d), dtype=np.int64)
    for i in range(n):
        ps = range(indptr[i], indptr[i + 1])
        for k in range(d):
            if reduce == "mean":
                if len(ps):
                    Y[i, k] = sum(float(values[p]) * float(X[indices[p], k]) for p in ps) / len(ps)
                continue
            best = None
            for p in ps:
                t = np.float32(values[p]) * np.float32(X[indices[p], k])
                if best is None or (t < best if reduce == "min" else t > best):
                    best, arg[i, k] = t, p
            Y[i, k] = 0.0 if best is None else float(best)
    return Y, arg


@settings(max_examples=50, deadline=None)
@given(small_csr(), st.sampled_from(["mean", "min", "max"]), st.booleans())
def test_reduce_matches_bruteforce(case, reduce, integer_inputs):
    n_rows, n_cols, d, seed, indptr, indices, values = case
    rng = np.random.default_rng(seed)
    if integer_inputs:  # few distinct products => ties, which must resolve to the first entry
        values = rng.integers(-1, 2, size=len(indices)).astype(np.float32)
        X = rng.integers(-2, 3, size=(n_cols, d)).astype(np.float32)
    else:
        X = rng.standard_normal((n_cols, d)).astype(np.float32)
    Y, arg, mag = oracle.spmm_reduce(indptr, indices, values, X, reduce)
    refY, refarg = _brute(indptr, indices, values, X, reduce)
    if reduce == "mean":
        np.testing.assert_allclose(Y, refY, rtol=1e-12, atol=1e-12)
        assert arg is None and np.all(mag + 1e-12 >= np.abs(Y))
    else:
        assert np.array_equal(Y, refY)
        assert np.array_equal(arg, refarg)
        # the winner really attains the value; nobody earlier does
        rows = _rows(indptr)
        for i in range(n_rows):
            for k in range(d):
                p = arg[i, k]
                if p < 0:
                    assert indptr[i] == indptr[i + 1] and Y[i, k] == 0
                else:
                    assert rows[p] == i
                    assert float(np.float32(values[p]) * np.float32(X[indices[p], k])) == Y[i, k]


def test_mean_closed_forms():
    w = graphgen.make_config(1, shrink=64)
    deg = np.diff(w.indptr)
    # unit values, constant X  => mean = that constant on non-empty rows
    X = np.full((w.n, 3), 2.5, dtype=np.float32)
    Y, _, _ = oracle.spmm_reduce(w.indptr, w.indices, None, X, "mean")
    np.testing.assert_allclose(Y[deg > 0], 2.5, rtol=1e-13)
    # mean = sum / degree
    S, _ = oracle.spmm(w.indptr, w.indices, w.values, w.X)
    M, _, _ = oracle.spmm_reduce(w.indptr, w.indices, w.values, w.X, "mean")
    np.testing.assert_allclose(M, S / np.maximum(deg, 1)[:, None], rtol=1e-13, atol=0)
    # max of unit-valued A over one-hot node indicators = 1 where the row has any entry
    Y, arg, _ = oracle.spmm_reduce(w.indptr, w.indices, None, np.ones((w.n, 1), dtype=np.float32), "max")
    assert np.array_equal(Y[:, 0], (deg > 0).astype(np.float64))
    assert np.array_equal(arg[:, 0], np.where(deg > 0, w.indptr[:-1], -1))  # first entry wins every tie


@settings(max_examples=30, deadline=None)
@given(small_csr(), st.sampled_from(["mean", "min", "max"]))
def test_reduce_backward_is_the_adjoint_of_the_selected_linear_map(case, reduce):
    """With the selection frozen, Y is linear in X; its adjoint applied to dY must be dX:
    <dY, Y(X)> = <dX, X> (exact up to fp64 rounding; min/max products are fp32-rounded, hence rtol)."""
    n_rows, n_cols, d, seed, indptr, indices, values = case
    rng = np.random.default_rng(seed + 7)
    X = rng.standard_normal((n_cols, d)).astype(np.float32)
    G = rng.standard_normal((n_rows, d)).astype(np.float32)
    Y, arg, _ = oracle.spmm_reduce(indptr, indices, values, X, reduce)
    dX, mag = oracle.spmm_reduce_backward(n_cols, indptr, indices, values, G, reduce, arg)
    lhs = np.sum(G.astype(np.float64) * Y)
    rhs = np.sum(dX * X.astype(np.float64))
    assert abs(lhs - rhs) <= 1e-6 * (1 + np.sum(np.abs(G.astype(np.float64) * Y)))
    assert np.all(mag + 1e-12 >= np.abs(dX))
    # dense check of the mean backward: dX = (D^-1 A)^T dY
    if reduce == "mean":
        A = _dense(n_rows, n_cols, indptr, indices, values)
        deg = np.maximum(np.diff(indptr), 1)[:, None]
        np.testing.assert_allclose(dX, (A / deg).T @ G.astype(np.float64), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("reduce", ["min", "max"])
def test_minmax_backward_finite_differences(reduce):
    """Away from ties the reduction is locally linear, so a central difference of <dY, Y(X)> with Y
    from the brute-force definition reproduces dX."""
    rng = np.random.default_rng(3)
    n, m, d = 7, 6, 3
    indptr, indices, values = graphgen.random_csr(n, m, 20, 4)
    X = (np.round(rng.standard_normal((m, d)) * 32) / 32 + 0.003 * np.arange(m * d).reshape(m, d)).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    _, arg, _ = oracle.spmm_reduce(indptr, indices, values, X, reduce)
    dX, _ = oracle.spmm_reduce_backward(m, indptr, indices, values, G, reduce, arg)
    h = 2.0 ** -8
    fd = np.zeros((m, d))
    for r in range(m):
        for k in range(d):
            Xp, Xm = X.copy(), X.copy()
            Xp[r, k] += np.float32(h)
            Xm[r, k] -= np.float32(h)
            fp = np.sum(G.astype(np.float64) * _brute(indptr, indices, values, Xp, reduce)[0])
            fm = np.sum(G.astype(np.float64) * _brute(indptr, indices, values, Xm, reduce)[0])
            fd[r, k] = (fp - fm) / (2 * h)
    np.testing.assert_allclose(dX, fd, rtol=1e-4, atol=1e-4)
