"""ctypes front end of the CPU oracle (``isp_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the benchmark's
cpu_baseline leg, never by the GPU library or its binding.  Everything returned is fp64
(structural outputs keep their integer types).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "isp_oracle.c")
_LIB = os.path.join(_HERE, "libisp_oracle.so")
_lib = None


def compile_source(src: str, out: str) -> str:
    """gcc line shared by the real build and by the tests that compile deliberately broken copies."""
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", src, "-o", out, "-lm"])
    return out


def build(force: bool = False) -> str:
    """Compile isp_oracle.c into libisp_oracle.so with gcc."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        compile_source(_SRC, tmp)
        os.replace(tmp, _LIB)
    return _LIB


def use_library(path):
    """Point this module at another build of the oracle (tests of the pins use broken copies);
    ``None`` goes back to the real one."""
    global _lib
    _lib = None
    if path is not None:
        _lib = _bind(ctypes.CDLL(path))


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    _lib = _bind(ctypes.CDLL(_LIB))
    return _lib


def _bind(lib):
    vp = ctypes.c_void_p
    i64, i32 = ctypes.c_int64, ctypes.c_int32
    lib.isp_oracle_max_threads.restype = ctypes.c_int
    lib.isp_oracle_set_threads.argtypes = [ctypes.c_int]
    lib.isp_oracle_transpose.argtypes = [i64, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.isp_oracle_transpose.restype = ctypes.c_int
    lib.isp_oracle_spmm.argtypes = [i64, vp, vp, vp, vp, i64, i32, vp, vp]
    lib.isp_oracle_spmm.restype = None
    lib.isp_oracle_spmm_scatter.argtypes = [i64, i64, vp, vp, vp, vp, i64, i32, vp]
    lib.isp_oracle_spmm_scatter.restype = None
    lib.isp_oracle_sddmm.argtypes = [i64, vp, vp, vp, vp, i64, vp, i64, i32, ctypes.c_int, vp, vp]
    lib.isp_oracle_sddmm.restype = None
    lib.isp_oracle_fusedmm.argtypes = [i64, vp, vp, vp, vp, i64, i32, ctypes.c_int, vp, vp]
    lib.isp_oracle_fusedmm.restype = None
    lib.isp_oracle_fusedmm_backward.argtypes = [i64, vp, vp, vp, vp, i64, vp, i64, i32, ctypes.c_int, vp, vp]
    lib.isp_oracle_fusedmm_backward.restype = None
    lib.isp_oracle_spmm_reduce.argtypes = [i64, vp, vp, vp, vp, i64, i32, ctypes.c_int, vp, vp, vp]
    lib.isp_oracle_spmm_reduce.restype = None
    lib.isp_oracle_spmm_reduce_backward.argtypes = [i64, i64, vp, vp, vp, vp, i64, i32, ctypes.c_int, vp, vp, vp]
    lib.isp_oracle_spmm_reduce_backward.restype = None
    return lib


def max_threads() -> int:
    return int(_load().isp_oracle_max_threads())


def set_threads(t: int) -> None:
    _load().isp_oracle_set_threads(int(t))


def _ptr(a):
    return None if a is None else a.ctypes.data


def _csr(indptr, indices, values):
    indptr = np.ascontiguousarray(indptr, dtype=np.int64)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    if values is not None:
        values = np.ascontiguousarray(values, dtype=np.float32)
        assert values.shape[0] == indices.shape[0]
    assert indptr[-1] == indices.shape[0]
    return indptr, indices, values


def _dense(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.ndim == 2
    return a


def transpose(n_rows, n_cols, indptr, indices, values=None):
    """Stable transpose.  Returns (t_indptr int64, t_indices int32, perm int32, t_values fp32|None)."""
    indptr, indices, values = _csr(indptr, indices, values)
    nnz = indices.shape[0]
    t_indptr = np.empty(n_cols + 1, dtype=np.int64)
    t_indices = np.empty(nnz, dtype=np.int32)
    perm = np.empty(nnz, dtype=np.int32)
    t_values = np.empty(nnz, dtype=np.float32) if values is not None else None
    rc = _load().isp_oracle_transpose(n_rows, n_cols, _ptr(indptr), _ptr(indices), _ptr(values), _ptr(t_indptr),
                                      _ptr(t_indices), _ptr(perm), _ptr(t_values))
    if rc != 0:
        raise ValueError("column index out of range" if rc == -1 else "out of memory")
    return t_indptr, t_indices, perm, t_values


def spmm(indptr, indices, values, X, want_mag=True):
    """Y = A X in fp64 and the per-element magnitude sum |a x| (or None)."""
    indptr, indices, values = _csr(indptr, indices, values)
    X = _dense(X)
    n, d = indptr.shape[0] - 1, X.shape[1]
    if indices.size:
        assert indices.max() < X.shape[0] and indices.min() >= 0
    Y = np.empty((n, d), dtype=np.float64)
    mag = np.empty((n, d), dtype=np.float64) if want_mag else None
    _load().isp_oracle_spmm(n, _ptr(indptr), _ptr(indices), _ptr(values), _ptr(X), X.shape[1], d, _ptr(Y), _ptr(mag))
    return Y, mag


def spmm_scatter(n_cols, indptr, indices, values, dY):
    """A^T dY by scattering, no transpose involved (second route for the backward)."""
    indptr, indices, values = _csr(indptr, indices, values)
    dY = _dense(dY)
    n, d = indptr.shape[0] - 1, dY.shape[1]
    assert dY.shape[0] == n
    if indices.size:
        assert indices.max() < n_cols and indices.min() >= 0
    dX = np.empty((n_cols, d), dtype=np.float64)
    _load().isp_oracle_spmm_scatter(n, n_cols, _ptr(indptr), _ptr(indices), _ptr(values), _ptr(dY), d, d, _ptr(dX))
    return dX


def sddmm(indptr, indices, values, U, V, scale_by_a=False, want_mag=True):
    """out[p] = <U[i], V[col_p]> (times a_p when scale_by_a) in fp64, plus magnitudes."""
    indptr, indices, values = _csr(indptr, indices, values)
    U, V = _dense(U), _dense(V)
    n, d = indptr.shape[0] - 1, U.shape[1]
    assert U.shape[0] == n and V.shape[1] == d
    if indices.size:
        assert indices.max() < V.shape[0] and indices.min() >= 0
    out = np.empty(indices.shape[0], dtype=np.float64)
    mag = np.empty(indices.shape[0], dtype=np.float64) if want_mag else None
    _load().isp_oracle_sddmm(n, _ptr(indptr), _ptr(indices), _ptr(values), _ptr(U), d, _ptr(V), d, d,
                             int(bool(scale_by_a)), _ptr(out), _ptr(mag))
    return out, mag


EDGE_OPS = {"sigmoid": 0, "dot": 1, "one": 2}


def fusedmm(indptr, indices, values, X, want_mag=True, op="sigmoid"):
    """FusedMM forward: y_i = sum_j a_ij f(<x_i,x_j>) x_j, f = sigmoid | dot (identity) | one."""
    indptr, indices, values = _csr(indptr, indices, values)
    X = _dense(X)
    n, d = indptr.shape[0] - 1, X.shape[1]
    assert X.shape[0] >= n  # a row-prefix of a square matrix is accepted (rows i < n, columns < X rows)
    if indices.size:
        assert indices.max() < X.shape[0] and indices.min() >= 0
    Y = np.empty((n, d), dtype=np.float64)
    mag = np.empty((n, d), dtype=np.float64) if want_mag else None
    _load().isp_oracle_fusedmm(n, _ptr(indptr), _ptr(indices), _ptr(values), _ptr(X), d, d, EDGE_OPS[op], _ptr(Y),
                               _ptr(mag))
    return Y, mag


def fusedmm_backward(indptr, indices, values, X, dY, want_mag=True, op="sigmoid"):
    """dX of FusedMM (edge function op) for upstream gradient dY."""
    indptr, indices, values = _csr(indptr, indices, values)
    X, dY = _dense(X), _dense(dY)
    n, d = indptr.shape[0] - 1, X.shape[1]
    assert X.shape[0] == n and dY.shape == X.shape
    if indices.size:
        assert indices.max() < n and indices.min() >= 0
    dX = np.empty((n, d), dtype=np.float64)
    mag = np.empty((n, d), dtype=np.float64) if want_mag else None
    _load().isp_oracle_fusedmm_backward(n, _ptr(indptr), _ptr(indices), _ptr(values), _ptr(X), d, _ptr(dY), d, d,
                                        EDGE_OPS[op], _ptr(dX), _ptr(mag))
    return dX, mag


REDUCE = {"sum": 0, "mean": 1, "min": 2, "max": 3}


def spmm_reduce(indptr, indices, values, X, reduce, want_mag=True):
    """Y = reduce over each row's stored entries of a_p * X[col_p] for reduce in 'mean', 'min', 'max'.
    Returns (Y fp64, arg int32 | None, mag | None); min / max products are formed in fp32."""
    indptr, indices, values = _csr(indptr, indices, values)
    X = _dense(X)
    n, d = indptr.shape[0] - 1, X.shape[1]
    if indices.size:
        assert indices.max() < X.shape[0] and indices.min() >= 0
    r = REDUCE[reduce]
    assert r in (1, 2, 3)
    Y = np.empty((n, d), dtype=np.float64)
    arg = np.empty((n, d), dtype=np.int32) if r >= 2 else None
    mag = np.empty((n, d), dtype=np.float64) if (want_mag and r == 1) else None
    _load().isp_oracle_spmm_reduce(n, _ptr(indptr), _ptr(indices), _ptr(values), _ptr(X), d, d, r, _ptr(Y),
                                   _ptr(arg), _ptr(mag))
    return Y, arg, mag


def spmm_reduce_backward(n_cols, indptr, indices, values, dY, reduce, arg=None, want_mag=True):
    """dX (n_cols x d, fp64) of spmm_reduce for upstream gradient dY; min / max need the forward's arg."""
    indptr, indices, values = _csr(indptr, indices, values)
    dY = _dense(dY)
    n, d = indptr.shape[0] - 1, dY.shape[1]
    assert dY.shape[0] == n
    r = REDUCE[reduce]
    assert r in (1, 2, 3)
    if r >= 2:
        arg = np.ascontiguousarray(arg, dtype=np.int32)
        assert arg.shape == (n, d)
    dX = np.empty((n_cols, d), dtype=np.float64)
    mag = np.empty((n_cols, d), dtype=np.float64) if want_mag else None
    _load().isp_oracle_spmm_reduce_backward(n, n_cols, _ptr(indptr), _ptr(indices), _ptr(values), _ptr(dY), d, d, r,
                                            _ptr(arg), _ptr(dX), _ptr(mag))
    return dX, mag
