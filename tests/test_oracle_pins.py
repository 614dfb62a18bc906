"""Pins for the CPU oracle: each oracle function is checked against something that is not
itself -- a hand-worked fixture, dense brute force written here in numpy, scipy's own
routines, closed forms, adjoint identities and finite differences.  CPU only."""
import os

import numpy as np
import pytest
import scipy.sparse as sp
from hypothesis import given, settings, strategies as st

import graphgen
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            out[key] = np.array([float(v) for v in vals])
    return out


def _dense(n_rows, n_cols, indptr, indices, values):
    """Densify a CSR (duplicates add up) in fp64."""
    A = np.zeros((n_rows, n_cols), dtype=np.float64)
    rows = np.repeat(np.arange(n_rows), np.diff(indptr))
    vals = np.ones(len(indices)) if values is None else values.astype(np.float64)
    np.add.at(A, (rows, indices), vals)
    return A


def _rows(indptr):
    return np.repeat(np.arange(len(indptr) - 1), np.diff(indptr))


# ---------------------------------------------------------------- hand-worked fixture
def test_hand_worked_example():
    g = _read_golden("spmm_hand_3x4.txt")
    indptr = g["indptr"].astype(np.int64)
    indices = g["indices"].astype(np.int32)
    values = g["values"].astype(np.float32)
    X = g["X"].reshape(4, 2).astype(np.float32)
    W = g["W"].reshape(3, 2).astype(np.float32)
    Y, mag = oracle.spmm(indptr, indices, values, X)
    assert np.array_equal(Y, g["Y"].reshape(3, 2))
    assert np.array_equal(mag[0], [2.0, 9.0]) and np.array_equal(mag[2], [17.5, 6.0])
    t_indptr, t_indices, perm, t_values = oracle.transpose(3, 4, indptr, indices, values)
    assert np.array_equal(t_indptr, g["t_indptr"])
    assert np.array_equal(t_indices, g["t_indices"])
    assert np.array_equal(perm, g["perm"])
    assert np.array_equal(t_values, g["t_values"])
    AtW, _ = oracle.spmm(t_indptr, t_indices, t_values, W)
    assert np.array_equal(AtW, g["AtW"].reshape(4, 2))
    assert np.array_equal(oracle.spmm_scatter(4, indptr, indices, values, W), g["AtW"].reshape(4, 2))
    out, _ = oracle.sddmm(indptr, indices, values, W, X)
    assert np.array_equal(out, g["sddmm"])
    out_s, _ = oracle.sddmm(indptr, indices, values, W, X, scale_by_a=True)
    assert np.array_equal(out_s, g["sddmm"] * g["values"])


# ---------------------------------------------------------------- random small CSR strategy
@st.composite
def small_csr(draw, square=False):
    n_rows = draw(st.integers(1, 12))
    n_cols = n_rows if square else draw(st.integers(1, 12))
    nnz = draw(st.integers(0, 40))
    seed = draw(st.integers(0, 2**31 - 1))
    sorted_cols = draw(st.booleans())
    allow_dup = draw(st.booleans())
    d = draw(st.sampled_from([1, 2, 3, 5, 8]))
    return (n_rows, n_cols, d, seed) + graphgen.random_csr(n_rows, n_cols, nnz, seed, sorted_cols=sorted_cols,
                                                           allow_dup=allow_dup)


@settings(max_examples=60, deadline=None)
@given(small_csr())
def test_spmm_matches_dense_bruteforce(case):
    n_rows, n_cols, d, seed, indptr, indices, values = case
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n_cols, d)).astype(np.float32)
    Y, mag = oracle.spmm(indptr, indices, values, X)
    A = _dense(n_rows, n_cols, indptr, indices, values)
    ref = np.zeros((n_rows, d))
    for i in range(n_rows):  # triple loop, definition of the product
        for j in range(n_cols):
            for k in range(d):
                ref[i, k] += A[i, j] * float(X[j, k])
    np.testing.assert_allclose(Y, ref, rtol=1e-12, atol=1e-12)
    # magnitude: |A| |X| when no duplicates cancel; always >= |Y|
    assert np.all(mag + 1e-12 >= np.abs(Y))
    absA = _dense(n_rows, n_cols, indptr, indices, np.abs(values))
    np.testing.assert_allclose(mag, absA @ np.abs(X.astype(np.float64)), rtol=1e-12, atol=1e-12)
    # values=None means all ones
    Y1, _ = oracle.spmm(indptr, indices, None, X)
    np.testing.assert_allclose(Y1, _dense(n_rows, n_cols, indptr, indices, None) @ X.astype(np.float64),
                               rtol=1e-12, atol=1e-12)


@settings(max_examples=60, deadline=None)
@given(small_csr())
def test_transpose_properties(case):
    n_rows, n_cols, d, seed, indptr, indices, values = case
    t_indptr, t_indices, perm, t_values = oracle.transpose(n_rows, n_cols, indptr, indices, values)
    nnz = len(indices)
    # perm is a permutation, equal to the stable argsort of the column indices
    assert np.array_equal(np.sort(perm), np.arange(nnz))
    assert np.array_equal(perm, np.argsort(indices, kind="stable"))
    assert np.array_equal(t_values, values[perm])
    assert np.array_equal(t_indices, _rows(indptr)[perm])
    # t_indptr = exclusive scan of the column histogram
    hist = np.bincount(indices, minlength=n_cols)
    assert np.array_equal(t_indptr, np.concatenate([[0], np.cumsum(hist)]))
    # dense transposes agree
    assert np.array_equal(_dense(n_cols, n_rows, t_indptr, t_indices, t_values),
                          _dense(n_rows, n_cols, indptr, indices, values).T)
    # transposing twice restores A bit for bit when A's rows are column-sorted
    cols_sorted = all(np.all(np.diff(indices[indptr[i]:indptr[i + 1]]) >= 0) for i in range(n_rows))
    tt = oracle.transpose(n_cols, n_rows, t_indptr, t_indices, t_values)
    if cols_sorted:
        assert np.array_equal(tt[0], indptr) and np.array_equal(tt[1], indices) and np.array_equal(tt[3], values)
    else:  # otherwise it is A with every row stably column-sorted
        assert np.array_equal(tt[0], indptr)
        for i in range(n_rows):
            s, e = indptr[i], indptr[i + 1]
            o = np.argsort(indices[s:e], kind="stable")
            assert np.array_equal(tt[1][s:e], indices[s:e][o]) and np.array_equal(tt[3][s:e], values[s:e][o])


def test_transpose_matches_scipy_and_rejects_bad_column():
    indptr, indices, values = graphgen.random_csr(300, 211, 5000, 7)
    t_indptr, t_indices, perm, t_values = oracle.transpose(300, 211, indptr, indices, values)
    T = sp.csr_matrix((values, indices, indptr), shape=(300, 211)).T.tocsr()
    assert np.array_equal(T.indptr, t_indptr) and np.array_equal(T.indices, t_indices)
    assert np.array_equal(T.data, t_values)
    bad = indices.copy()
    bad[17] = 211
    with pytest.raises(ValueError):
        oracle.transpose(300, 211, indptr, bad, values)


def test_transpose_symmetric_pattern_is_fixed_point():
    w = graphgen.make_config(1, shrink=64)
    t_indptr, t_indices, perm, t_values = oracle.transpose(w.n, w.n, w.indptr, w.indices, w.values)
    assert np.array_equal(t_indptr, w.indptr) and np.array_equal(t_indices, w.indices)
    # GCN normalisation of a symmetric pattern is symmetric
    assert np.array_equal(t_values, w.values)


def test_spmm_matches_scipy_medium():
    w = graphgen.make_config(1, shrink=16)
    Y, _ = oracle.spmm(w.indptr, w.indices, w.values, w.X)
    A = sp.csr_matrix((w.values.astype(np.float64), w.indices, w.indptr), shape=(w.n, w.n))
    np.testing.assert_allclose(Y, A @ w.X.astype(np.float64), rtol=1e-11, atol=1e-11)


def test_spmm_closed_forms():
    for k, shrink in ((1, 32), (4, 256), (0, 1)):
        w = graphgen.make_config(k, shrink=shrink)
        deg = np.diff(w.indptr).astype(np.float64)
        ones = np.ones((w.n, 3), dtype=np.float32)
        # unit values: A 1 = degree vector, exactly
        Y, _ = oracle.spmm(w.indptr, w.indices, None, ones)
        assert np.array_equal(Y, np.repeat(deg[:, None], 3, axis=1))
        # row-mean values: A 1 = 1 on non-empty rows, 0 on empty ones
        vm = graphgen.edge_values(w.indptr, w.indices, "rowmean")
        Y, _ = oracle.spmm(w.indptr, w.indices, vm, ones)
        np.testing.assert_allclose(Y[:, 0], (deg > 0).astype(np.float64), rtol=0, atol=1e-6)
    # symmetric GCN normalisation: A_hat D^{1/2} 1 = D^{1/2} 1
    w = graphgen.make_config(1, shrink=32)
    deg = np.diff(w.indptr).astype(np.float64)
    v = np.sqrt(deg).astype(np.float32)[:, None]
    Y, _ = oracle.spmm(w.indptr, w.indices, w.values, v)
    np.testing.assert_allclose(Y[:, 0], v[:, 0].astype(np.float64), rtol=1e-6)


@settings(max_examples=40, deadline=None)
@given(small_csr())
def test_backward_adjoint_and_scatter(case):
    n_rows, n_cols, d, seed, indptr, indices, values = case
    rng = np.random.default_rng(seed + 1)
    X = rng.standard_normal((n_cols, d)).astype(np.float32)
    W = rng.standard_normal((n_rows, d)).astype(np.float32)
    AX, _ = oracle.spmm(indptr, indices, values, X)
    t_indptr, t_indices, perm, t_values = oracle.transpose(n_rows, n_cols, indptr, indices, values)
    AtW, _ = oracle.spmm(t_indptr, t_indices, t_values, W)
    # <A X, W> = <X, A^T W>
    lhs, rhs = np.sum(AX * W), np.sum(X.astype(np.float64) * AtW)
    assert abs(lhs - rhs) <= 1e-10 * (1 + abs(lhs))
    # scatter form agrees (different summation order only)
    np.testing.assert_allclose(oracle.spmm_scatter(n_cols, indptr, indices, values, W), AtW, rtol=1e-12, atol=1e-12)
    # and equals the dense A^T W
    np.testing.assert_allclose(AtW, _dense(n_rows, n_cols, indptr, indices, values).T @ W.astype(np.float64),
                               rtol=1e-12, atol=1e-12)


@settings(max_examples=40, deadline=None)
@given(small_csr())
def test_sddmm_bruteforce_and_identity(case):
    n_rows, n_cols, d, seed, indptr, indices, values = case
    rng = np.random.default_rng(seed + 2)
    U = rng.standard_normal((n_rows, d)).astype(np.float32)
    V = rng.standard_normal((n_cols, d)).astype(np.float32)
    out, mag = oracle.sddmm(indptr, indices, values, U, V)
    full = U.astype(np.float64) @ V.astype(np.float64).T  # dense U V^T, then sample the pattern
    rows = _rows(indptr)
    np.testing.assert_allclose(out, full[rows, indices], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(mag, (np.abs(U.astype(np.float64)) @ np.abs(V.astype(np.float64)).T)[rows, indices],
                               rtol=1e-12, atol=1e-12)
    out_s, mag_s = oracle.sddmm(indptr, indices, values, U, V, scale_by_a=True)
    np.testing.assert_allclose(out_s, out * values, rtol=1e-14, atol=0)
    np.testing.assert_allclose(mag_s, mag * np.abs(values), rtol=1e-14, atol=0)
    # dA identity: <U, A V> = sum_p a_p out_p   (ties SpMM to SDDMM; the map is linear in a)
    AV, _ = oracle.spmm(indptr, indices, values, V)
    lhs = np.sum(U.astype(np.float64) * AV)
    rhs = np.sum(values.astype(np.float64) * out)
    assert abs(lhs - rhs) <= 1e-10 * (1 + abs(lhs))


# ---------------------------------------------------------------- FusedMM
def _fused_dense(A, X, op="sigmoid"):
    """Unfused composition in dense fp64: S = f(X X^T), Y = (A * S) X."""
    Z = X @ X.T
    S = {"sigmoid": lambda z: 1.0 / (1.0 + np.exp(-z)), "dot": lambda z: z, "one": lambda z: np.ones_like(z)}[op](Z)
    return (A * S) @ X


@settings(max_examples=40, deadline=None)
@given(small_csr(square=True))
def test_fusedmm_forward_is_unfused_composition(case):
    n, _, d, seed, indptr, indices, values = case
    rng = np.random.default_rng(seed + 3)
    X = (0.5 * rng.standard_normal((n, d))).astype(np.float32)
    for op in ("dot", "one"):
        Yo, mo = oracle.fusedmm(indptr, indices, values, X, op=op)
        np.testing.assert_allclose(Yo, _fused_dense(_dense(n, n, indptr, indices, values), X.astype(np.float64), op),
                                   rtol=1e-11, atol=1e-12)
        assert np.all(mo + 1e-12 >= np.abs(Yo))
    # the constant-one edge function is the plain SpMM
    np.testing.assert_allclose(oracle.fusedmm(indptr, indices, values, X, op="one")[0],
                               oracle.spmm(indptr, indices, values, X)[0], rtol=1e-13, atol=1e-13)
    Y, mag = oracle.fusedmm(indptr, indices, values, X)
    # route 1: dense
    np.testing.assert_allclose(Y, _fused_dense(_dense(n, n, indptr, indices, values), X.astype(np.float64)),
                               rtol=1e-11, atol=1e-12)
    # route 2: oracle sddmm -> sigmoid -> oracle spmm with the edge values scaled
    z, _ = oracle.sddmm(indptr, indices, None, X, X)
    s = 1.0 / (1.0 + np.exp(-z))
    rows = _rows(indptr)
    ref = np.zeros((n, d))
    np.add.at(ref, rows, (values.astype(np.float64) * s)[:, None] * X.astype(np.float64)[indices])
    np.testing.assert_allclose(Y, ref, rtol=1e-11, atol=1e-12)
    assert np.all(mag + 1e-12 >= np.abs(Y))


def test_fusedmm_special_cases():
    w = graphgen.make_config(4, shrink=512)
    n, d = w.n, 8
    deg = np.diff(w.indptr).astype(np.float64)
    # X = 0  =>  Y = 0
    Y, _ = oracle.fusedmm(w.indptr, w.indices, None, np.zeros((n, d), dtype=np.float32))
    assert np.all(Y == 0)
    # every node carries the same vector c*e: z = c^2 |e|^2 everywhere, y_i = deg_i sigmoid(z) x
    e = np.zeros(d, dtype=np.float32)
    e[2] = 1.0
    c = 0.75
    X = np.tile(c * e, (n, 1)).astype(np.float32)
    Y, _ = oracle.fusedmm(w.indptr, w.indices, None, X)
    sig = 1.0 / (1.0 + np.exp(-c * c))
    np.testing.assert_allclose(Y, deg[:, None] * sig * X.astype(np.float64), rtol=1e-13, atol=0)


@pytest.mark.parametrize("op", ["sigmoid", "dot", "one"])
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_fusedmm_backward_finite_differences(seed, op):
    """dX from the oracle equals the central finite difference of L = <dY, Y(X)>, where Y(X) is
    evaluated by the independent dense composition above (not by the oracle)."""
    rng = np.random.default_rng(seed)
    n, d = 9, 4
    indptr, indices, values = graphgen.random_csr(n, n, 30, seed + 10, sorted_cols=bool(seed % 2),
                                                  allow_dup=bool(seed // 2))
    # force at least one self-loop so the i == j case is exercised
    indices[0] = 0 if indptr[1] > 0 else indices[0]
    # inputs on a coarse binary grid so X +/- h is exact in fp32
    X = (np.round(rng.standard_normal((n, d)) * 64) / 128).astype(np.float32)
    G = (np.round(rng.standard_normal((n, d)) * 64) / 64).astype(np.float32)
    A = _dense(n, n, indptr, indices, values)
    dX, mag = oracle.fusedmm_backward(indptr, indices, values, X, G, op=op)
    h = 2.0 ** -12
    X64, G64 = X.astype(np.float64), G.astype(np.float64)
    fd = np.zeros((n, d))
    for r in range(n):
        for k in range(d):
            Xp, Xm = X64.copy(), X64.copy()
            Xp[r, k] += h
            Xm[r, k] -= h
            fd[r, k] = (np.sum(G64 * _fused_dense(A, Xp, op)) - np.sum(G64 * _fused_dense(A, Xm, op))) / (2 * h)
    np.testing.assert_allclose(dX, fd, rtol=1e-6, atol=1e-6)
    assert np.all(mag >= 0)


def test_fusedmm_backward_linear_part_adjoint():
    """With the sigmoid frozen (X tiny => s = 1/2, dz ~ 0) the map is Y = (A/2) X, so dX -> (A/2)^T dY."""
    n, d = 40, 6
    indptr, indices, values = graphgen.random_csr(n, n, 200, 3)
    rng = np.random.default_rng(5)
    X = (1e-20 * rng.standard_normal((n, d))).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    dX, _ = oracle.fusedmm_backward(indptr, indices, values, X, G)
    ref = 0.5 * oracle.spmm_scatter(n, indptr, indices, values, G)
    np.testing.assert_allclose(dX, ref, rtol=1e-12, atol=1e-15)


# ---------------------------------------------------------------- planted mistakes must be caught
def test_pins_catch_a_transposed_operand():
    """A rectangular case separates A X from A^T X and U V^T from V U^T: a sanity check that the
    pins above would fail for a transposed-operand mistake."""
    indptr, indices, values = graphgen.random_csr(5, 9, 20, 11)
    X = np.random.default_rng(0).standard_normal((9, 3)).astype(np.float32)
    Y, _ = oracle.spmm(indptr, indices, values, X)
    assert Y.shape == (5, 3)
    t = oracle.transpose(5, 9, indptr, indices, values)
    assert t[0].shape[0] == 10 and t[1].max() < 5
