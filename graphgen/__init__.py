"""Seeded synthetic inputs for the SpMM / SDDMM / FusedMM path.

Generates the graphs (Erdos-Renyi, R-MAT), edge values (unit, GCN-normalised, row-mean)
and dense feature matrices the tests and the benchmark run on.  It holds inputs only:
none of the sparse arithmetic lives here, and both the CPU oracle's tests and the GPU
library's tests draw their data from this one module so they see identical bytes.

The heavy lifting is a small C++/OpenMP library (``gen.cpp``) compiled on first use
with g++ and loaded through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.cpp")
_LIB = os.path.join(_HERE, "libgraphgen.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile gen.cpp into libgraphgen.so (g++, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["g++", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c++17", _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


def use_library(path):
    """Point this module at another build of gen.cpp (the sanitizer test loads an instrumented one);
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
    i32p = ctypes.POINTER(ctypes.c_int32)
    i64p = ctypes.POINTER(ctypes.c_int64)
    f32p = ctypes.POINTER(ctypes.c_float)
    lib.gg_rmat_edges.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_uint64,
                                  ctypes.c_double, ctypes.c_double, ctypes.c_double, i32p, i32p]
    lib.gg_rmat_edges.restype = None
    lib.gg_er_edges.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_uint64, i32p, i32p]
    lib.gg_er_edges.restype = None
    lib.gg_permutation.argtypes = [ctypes.c_int64, ctypes.c_uint64, i32p]
    lib.gg_permutation.restype = None
    lib.gg_build_csr.argtypes = [ctypes.c_int64, ctypes.c_int64, i32p, i32p, i32p, ctypes.c_int, ctypes.c_int,
                                 i64p, i32p]
    lib.gg_build_csr.restype = ctypes.c_int64
    lib.gg_values.argtypes = [ctypes.c_int64, i64p, i32p, ctypes.c_int, f32p]
    lib.gg_values.restype = None
    lib.gg_fill_uniform.argtypes = [f32p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_double, ctypes.c_double]
    lib.gg_fill_uniform.restype = None
    lib.gg_fill_normal.argtypes = [f32p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_double, ctypes.c_double]
    lib.gg_fill_normal.restype = None
    lib.gg_max_threads.restype = ctypes.c_int
    return lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


VALUE_MODES = {"unit": 0, "gcn": 1, "rowmean": 2}


def edge_values(indptr: np.ndarray, indices: np.ndarray, mode: str) -> np.ndarray:
    """fp32 edge values for a CSR pattern: 'unit', 'gcn' (1/sqrt(deg_i deg_j)) or 'rowmean' (1/deg_i)."""
    lib = _load()
    n = indptr.shape[0] - 1
    vals = np.empty(indices.shape[0], dtype=np.float32)
    lib.gg_values(n, _p(indptr, ctypes.c_int64), _p(indices, ctypes.c_int32), VALUE_MODES[mode],
                  _p(vals, ctypes.c_float))
    return vals


def uniform(shape, seed: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    lib = _load()
    out = np.empty(shape, dtype=np.float32)
    lib.gg_fill_uniform(_p(out, ctypes.c_float), out.size, seed, lo, hi)
    return out


def normal(shape, seed: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    lib = _load()
    out = np.empty(shape, dtype=np.float32)
    lib.gg_fill_normal(_p(out, ctypes.c_float), out.size, seed, mean, std)
    return out


def csr_from_pairs(n: int, u: np.ndarray, v: np.ndarray, *, symmetrise: bool, self_loops: bool,
                   relabel_seed: int | None):
    """(indptr int64, indices int32): sorted, duplicate-free rows from candidate (u, v) pairs."""
    lib = _load()
    m = u.shape[0]
    relabel = None
    if relabel_seed is not None:
        relabel = np.empty(n, dtype=np.int32)
        lib.gg_permutation(n, relabel_seed, _p(relabel, ctypes.c_int32))
    cap = (2 if symmetrise else 1) * m + n
    indptr = np.empty(n + 1, dtype=np.int64)
    indices = np.empty(cap, dtype=np.int32)
    nnz = lib.gg_build_csr(n, m, _p(u, ctypes.c_int32), _p(v, ctypes.c_int32),
                           _p(relabel, ctypes.c_int32) if relabel is not None else None,
                           int(symmetrise), int(self_loops), _p(indptr, ctypes.c_int64),
                           _p(indices, ctypes.c_int32))
    return indptr, indices[:nnz].copy()


def er_graph(n: int, avg_degree: float, seed: int, *, self_loops: bool = True, symmetrise: bool = False):
    """Directed Erdos-Renyi style graph: n*avg_degree uniformly drawn ordered pairs, deduplicated."""
    lib = _load()
    m = int(round(n * avg_degree))
    u = np.empty(m, dtype=np.int32)
    v = np.empty(m, dtype=np.int32)
    lib.gg_er_edges(n, m, seed, _p(u, ctypes.c_int32), _p(v, ctypes.c_int32))
    return csr_from_pairs(n, u, v, symmetrise=symmetrise, self_loops=self_loops, relabel_seed=None)


def rmat_graph(n: int, m_candidates: int, seed: int, *, abc=(0.57, 0.19, 0.19), symmetrise: bool = True,
               self_loops: bool = True, relabel: bool = True):
    """R-MAT graph on n vertices from m_candidates draws (scale = ceil(log2 n), no noise),
    endpoints >= n rejected, optionally symmetrised / self-looped, vertex ids randomly relabelled so
    hubs do not sit at contiguous low ids."""
    lib = _load()
    scale = max(1, int(np.ceil(np.log2(n))))
    u = np.empty(m_candidates, dtype=np.int32)
    v = np.empty(m_candidates, dtype=np.int32)
    lib.gg_rmat_edges(scale, n, m_candidates, seed, abc[0], abc[1], abc[2], _p(u, ctypes.c_int32),
                      _p(v, ctypes.c_int32))
    return csr_from_pairs(n, u, v, symmetrise=symmetrise, self_loops=self_loops,
                          relabel_seed=(seed + 0x5EED) if relabel else None)


@dataclass
class Workload:
    name: str
    n: int
    d: int
    indptr: np.ndarray  # int64 [n+1]
    indices: np.ndarray  # int32 [nnz]
    values: np.ndarray | None  # fp32 [nnz]; None means all ones
    X: np.ndarray  # fp32 [n, d]
    dY: np.ndarray  # fp32 [n, d]
    ops: tuple = ()
    recipe: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.indices.shape[0])


# Recipes for the five benchmark configurations.  m = number of candidate draws, calibrated
# so the deduplicated graph lands near the stated edge count.  `shrink` divides n and m
# for quick tests while keeping the degree structure.
_CONFIGS = {
    0: dict(name="c0-er4096-d32", kind="er", n=4096, avg_degree=8.0, d=32, values="gcn",
            symmetrise=False, self_loops=True, feat="uniform", ops=("spmm", "spmm_t", "sddmm")),
    1: dict(name="c1-rmat169k-d128", kind="rmat", n=169_343, m=1_390_000, d=128, values="gcn",
            symmetrise=True, self_loops=True, feat="normal", std=1.0, ops=("spmm", "spmm_t")),
    2: dict(name="c2-rmat233k-dense-d128", kind="rmat", n=232_965, m=92_300_000, d=128, values="rowmean",
            symmetrise=True, self_loops=False, feat="normal", std=1.0, ops=("spmm", "spmm_t", "sddmm")),
    3: dict(name="c3-rmat2.4m-d128", kind="rmat", n=2_449_029, m=81_700_000, d=128, values="gcn",
            symmetrise=True, self_loops=True, feat="normal", std=1.0, ops=("spmm", "spmm_t")),
    4: dict(name="c4-rmat1m-d64-fusedmm", kind="rmat", n=1_048_576, m=17_600_000, d=64, values="unit",
            symmetrise=False, self_loops=False, feat="normal", std=0.1, ops=("fusedmm", "fusedmm_bwd")),
}


def config_recipe(k: int, shrink: int = 1) -> dict:
    r = dict(_CONFIGS[k])
    if shrink > 1:
        r["n"] = max(64, r["n"] // shrink)
        if "m" in r:
            r["m"] = max(64, r["m"] // shrink)
        r["name"] += "-shrink%d" % shrink
    return r


def make_config(k: int, *, shrink: int = 1, graph_seed: int = 0, x_seed: int = 1, dy_seed: int = 2,
                d: int | None = None, relabel: bool = True) -> Workload:
    """Build benchmark configuration k (0..4).  Seeds: graph 0, X 1, dY 2 unless overridden.
    relabel=False keeps the R-MAT generator's own vertex ids (hubs at ids with few one-bits): not a
    benchmark configuration, only a point of comparison."""
    r = config_recipe(k, shrink)
    if not relabel:
        r["name"] += "-unrelabelled"
    n = r["n"]
    if r["kind"] == "er":
        indptr, indices = er_graph(n, r["avg_degree"], graph_seed, self_loops=r["self_loops"],
                                   symmetrise=r["symmetrise"])
    else:
        indptr, indices = rmat_graph(n, r["m"], graph_seed, symmetrise=r["symmetrise"],
                                     self_loops=r["self_loops"], relabel=relabel)
    # unit edge values are represented by "no value array" (the kernels then read no values)
    vals = None if r["values"] == "unit" else edge_values(indptr, indices, r["values"])
    dd = d if d is not None else r["d"]
    if r["feat"] == "uniform":
        X = uniform((n, dd), x_seed)
    else:
        X = normal((n, dd), x_seed, 0.0, r["std"])
    dY = uniform((n, dd), dy_seed) if r["feat"] == "uniform" else normal((n, dd), dy_seed, 0.0, 1.0)
    return Workload(name=r["name"], n=n, d=dd, indptr=indptr, indices=indices, values=vals, X=X, dY=dY,
                    ops=r["ops"], recipe=r)


def random_csr(n_rows: int, n_cols: int, nnz_target: int, seed: int, *, sorted_cols: bool = True,
               allow_dup: bool = False, values: str = "normal"):
    """Small general (possibly rectangular, possibly unsorted / duplicated) CSR for edge-case tests."""
    rng = np.random.Generator(np.random.Philox(seed))
    if n_rows == 0 or n_cols == 0 or nnz_target == 0:
        return (np.zeros(n_rows + 1, dtype=np.int64), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float32))
    rows = rng.integers(0, n_rows, size=nnz_target)
    cols = rng.integers(0, n_cols, size=nnz_target).astype(np.int32)
    if not allow_dup:
        key = rows.astype(np.int64) * n_cols + cols
        _, first = np.unique(key, return_index=True)
        first.sort()
        rows, cols = rows[first], cols[first]
    order = np.argsort(rows, kind="stable")
    rows, cols = rows[order], cols[order]
    indptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.add.at(indptr, rows + 1, 1)
    indptr = np.cumsum(indptr)
    if sorted_cols:
        for i in range(n_rows):
            s, e = indptr[i], indptr[i + 1]
            cols[s:e] = np.sort(cols[s:e], kind="stable")
    if values == "normal":
        vals = rng.standard_normal(cols.shape[0]).astype(np.float32)
    else:
        vals = np.ones(cols.shape[0], dtype=np.float32)
    return indptr, cols.astype(np.int32), vals
