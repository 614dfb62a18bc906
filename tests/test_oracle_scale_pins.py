"""Pins for the error-scale outputs (``mag``) of the oracle.  Every FusedMM and reduction parity test
divides its error by these scales, so each is recomputed here in dense fp64 numpy from the formula
it is defined by and compared to 1e-12: a scale that is too large would loosen the GPU tests without
any other pin noticing.  SpMM's and SDDMM's scales are pinned in test_oracle_pins.py.  CPU only."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from test_oracle_pins import _dense, small_csr

# bounds on |f'| and |f''| of the three edge functions (sigmoid, identity, constant one)
L1 = {"sigmoid": 0.25, "dot": 1.0, "one": 0.0}
L2 = {"sigmoid": 0.1, "dot": 0.0, "one": 0.0}


def _score(Z, op):
    """(|f(z)|, |f'(z)|) of the edge function, dense."""
    if op == "sigmoid":
        S = 1.0 / (1.0 + np.exp(-Z))
        return S, S * (1.0 - S)
    if op == "dot":
        return np.abs(Z), np.ones_like(Z)
    return np.ones_like(Z), np.zeros_like(Z)


def _sum_over_entries(n, indptr, indices, values, per_pair):
    """Dense n x n matrix W with W[i, j] = sum over the stored entries p = (i, j) of |a_p| * per_pair[i, j]
    (duplicates are separate entries and add up)."""
    absA = _dense(n, n, indptr, indices, np.abs(values))
    return absA * per_pair


@settings(max_examples=40, deadline=None)
@given(small_csr(square=True), st.sampled_from(["sigmoid", "dot", "one"]))
def test_fusedmm_forward_scale(case, op):
    """mag[i,k] = sum_p |a_p| (|s_p| + L1 za_p) |x_jk|,  za_p = sum_k |x_ik x_jk|."""
    n, _, d, seed, indptr, indices, values = case
    X = (0.7 * np.random.default_rng(seed + 21).standard_normal((n, d))).astype(np.float32)
    _, mag = oracle.fusedmm(indptr, indices, values, X, op=op)
    X64 = X.astype(np.float64)
    absS, _ = _score(X64 @ X64.T, op)
    ZA = np.abs(X64) @ np.abs(X64).T
    ref = _sum_over_entries(n, indptr, indices, values, absS + L1[op] * ZA) @ np.abs(X64)
    np.testing.assert_allclose(mag, ref, rtol=1e-12, atol=1e-14)


@settings(max_examples=25, deadline=None)
@given(small_csr(square=True))
def test_fusedmm_scale_reduces_to_the_spmm_bound(case):
    """With the constant edge function the scale is exactly the SpMM bound sum |a_p x_jk| the
    benchmark's tolerance is written in; for the other two it contains that bound times |s|."""
    n, _, d, seed, indptr, indices, values = case
    X = np.random.default_rng(seed + 22).standard_normal((n, d)).astype(np.float32)
    _, m_spmm = oracle.spmm(indptr, indices, values, X)
    _, m_one = oracle.fusedmm(indptr, indices, values, X, op="one")
    np.testing.assert_allclose(m_one, m_spmm, rtol=1e-13, atol=0)
    # sigmoid: |s| < 1 and za >= 0, so the scale lies between 0 and (1 + za_max / 4) x the SpMM bound
    _, m_sig = oracle.fusedmm(indptr, indices, values, X)
    za_max = (np.abs(X.astype(np.float64)) @ np.abs(X.astype(np.float64)).T).max() if n else 0.0
    assert np.all(m_sig <= (1.0 + 0.25 * za_max) * m_spmm + 1e-12)


@settings(max_examples=40, deadline=None)
@given(small_csr(square=True), st.sampled_from(["sigmoid", "dot", "one"]))
def test_fusedmm_backward_scale(case, op):
    """With ga = sum_k |g_ik x_jk| and dzm_p = |a_p| ga_p (|f'(z_p)| + L2 za_p):
    mag[i,:] += dzm_p |x_j|;   mag[j,:] += |a_p| (|s_p| + L1 za_p) |g_i| + dzm_p |x_i|."""
    n, _, d, seed, indptr, indices, values = case
    rng = np.random.default_rng(seed + 23)
    X = (0.7 * rng.standard_normal((n, d))).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    _, mag = oracle.fusedmm_backward(indptr, indices, values, X, G, op=op)
    X64, G64 = X.astype(np.float64), G.astype(np.float64)
    absS, absdF = _score(X64 @ X64.T, op)
    ZA = np.abs(X64) @ np.abs(X64).T
    GA = np.abs(G64) @ np.abs(X64).T  # [i, j] = sum_k |g_ik x_jk|
    DZM = _sum_over_entries(n, indptr, indices, values, GA * (absdF + L2[op] * ZA))
    SM = _sum_over_entries(n, indptr, indices, values, absS + L1[op] * ZA)
    ref = DZM @ np.abs(X64) + SM.T @ np.abs(G64) + DZM.T @ np.abs(X64)
    np.testing.assert_allclose(mag, ref, rtol=1e-12, atol=1e-14)


@settings(max_examples=40, deadline=None)
@given(small_csr())
def test_mean_scale(case):
    """mean: mag[i,k] = sum_p |a_p x_jk| / len_i, 0 on an empty row."""
    n_rows, n_cols, d, seed, indptr, indices, values = case
    X = np.random.default_rng(seed + 24).standard_normal((n_cols, d)).astype(np.float32)
    _, _, mag = oracle.spmm_reduce(indptr, indices, values, X, "mean")
    absA = _dense(n_rows, n_cols, indptr, indices, np.abs(values))
    ref = (absA @ np.abs(X.astype(np.float64))) / np.maximum(np.diff(indptr), 1)[:, None]
    np.testing.assert_allclose(mag, ref, rtol=1e-12, atol=1e-14)
    assert np.all(mag[np.diff(indptr) == 0] == 0)


@settings(max_examples=40, deadline=None)
@given(small_csr(), st.sampled_from(["mean", "min", "max"]))
def test_reduce_backward_scale(case, reduce):
    """mean: mag[j,k] = sum_{p=(i,j)} |a_p g_ik| / len_i;  min / max: mag[col(p),k] = sum over the (i,k)
    whose arg is p of |a_p g_ik|."""
    n_rows, n_cols, d, seed, indptr, indices, values = case
    rng = np.random.default_rng(seed + 25)
    X = rng.standard_normal((n_cols, d)).astype(np.float32)
    G = rng.standard_normal((n_rows, d)).astype(np.float32)
    _, arg, _ = oracle.spmm_reduce(indptr, indices, values, X, reduce)
    _, mag = oracle.spmm_reduce_backward(n_cols, indptr, indices, values, G, reduce, arg)
    G64 = np.abs(G.astype(np.float64))
    if reduce == "mean":
        absA = _dense(n_rows, n_cols, indptr, indices, np.abs(values))
        ref = (absA / np.maximum(np.diff(indptr), 1)[:, None]).T @ G64
    else:
        ref = np.zeros((n_cols, d))
        for i in range(n_rows):
            for k in range(d):
                p = arg[i, k]
                if p >= 0:
                    ref[indices[p], k] += abs(float(values[p])) * G64[i, k]
    np.testing.assert_allclose(mag, ref, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- min / max against the plain fp64 definition
@settings(max_examples=60, deadline=None)
@given(small_csr(), st.sampled_from(["min", "max"]), st.booleans())
def test_minmax_against_the_fp64_definition(case, reduce, integer_inputs):
    """The oracle forms and compares the products of min / max in fp32 (the precision of the method's
    arithmetic) so that positions can be compared bit for bit.  This ties that choice to the plain
    definition in fp64.  The product of two fp32 numbers is exact in fp64 and rounding to fp32 is
    monotone, so (1) the value is the fp64 extremum rounded once to fp32; (2) the position named attains
    that value after rounding, and no earlier entry of the row does (first winner); (3) near-tie rule:
    the position may differ from the fp64 definition's winner only when both products round to the
    same fp32 number."""
    n_rows, n_cols, d, seed, indptr, indices, values = case
    rng = np.random.default_rng(seed + 26)
    if integer_inputs:
        values = rng.integers(-1, 2, size=len(indices)).astype(np.float32)
        X = rng.integers(-2, 3, size=(n_cols, d)).astype(np.float32)
    else:  # (1 + a ulp)(1 + b ulp) = 1 + (a + b) ulp + a b ulp^2: products with equal a + b differ only beyond fp32
        X = (rng.choice([-1.0, 1.0], size=(n_cols, d)) * (1.0 + rng.integers(0, 4, size=(n_cols, d)) * 2.0 ** -23))
        X = X.astype(np.float32)
        values = (1.0 + rng.integers(0, 4, size=len(indices)) * 2.0 ** -23).astype(np.float32)
    Y, arg, _ = oracle.spmm_reduce(indptr, indices, values, X, reduce)
    pick = np.min if reduce == "min" else np.max
    where = np.argmin if reduce == "min" else np.argmax
    for i in range(n_rows):
        s, e = indptr[i], indptr[i + 1]
        for k in range(d):
            if s == e:
                assert Y[i, k] == 0 and arg[i, k] == -1
                continue
            prod = values[s:e].astype(np.float64) * X[indices[s:e], k].astype(np.float64)  # exact
            assert Y[i, k] == float(np.float32(pick(prod)))
            p = arg[i, k]
            assert s <= p < e
            rounded = prod.astype(np.float32)
            assert float(rounded[p - s]) == Y[i, k]
            assert not np.any(rounded[:p - s] == rounded[p - s])
            p64 = s + int(where(prod))  # first fp64 winner
            assert p == p64 or rounded[p - s] == rounded[p64 - s]
