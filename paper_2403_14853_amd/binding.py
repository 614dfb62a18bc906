"""ctypes binding of include/isp.h.  Same names as the C entry points, minus the ``isp_`` prefix.

Argument marshalling only.  Device buffers are torch CUDA tensors (allocation plumbing); the
handle object keeps references to every tensor the C library borrows so they outlive it.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libisp.so")
_lib = None

EXPORTED_SYMBOLS = [
    "isp_csr_build_workspace", "isp_csr_build", "isp_csr_transpose_workspace", "isp_csr_transpose_cached",
    "isp_csr_values_changed", "isp_csr_alias_workspace", "isp_csr_alias", "isp_csr_export", "isp_csr_info", "isp_spmm",
    "isp_spmm_static_scratch", "isp_sddmm", "isp_fusedmm", "isp_fusedmm_backward",
    "isp_spmm_reduce", "isp_spmm_reduce_backward", "isp_csr_destroy", "isp_last_error", "isp_version",
]

ISP_TRUSTED = 1
ISP_SCALE_BY_A = 1
ISP_OP_SIGMOID, ISP_OP_DOT, ISP_OP_ONE = 0, 1, 2
EDGE_OPS = {"sigmoid": 0, "dot": 1, "one": 2}
_STATUS = {0: "ISP_OK", 1: "ISP_EINVAL", 2: "ISP_EBADCSR", 3: "ISP_ENOMEM", 4: "ISP_EHIP", 5: "ISP_EUNSUPPORTED"}


class IspError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("%s: %s" % (_STATUS.get(status, status), msg))
        self.status = status
        self.status_name = _STATUS.get(status, str(status))


class CsrInfo(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("n_cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("max_degree", ctypes.c_int64), ("bin_rows", ctypes.c_int64 * 5), ("bin_nnz", ctypes.c_int64 * 5),
                ("hub_threshold", ctypes.c_int32), ("segment_len", ctypes.c_int32), ("block_cost", ctypes.c_int32),
                ("n_row_blocks", ctypes.c_int32), ("n_hub_rows", ctypes.c_int32), ("n_segments", ctypes.c_int32),
                ("is_transpose", ctypes.c_int32), ("has_cached_transpose", ctypes.c_int32),
                ("spmm_mid_threshold", ctypes.c_int32), ("spmm_cut_rows", ctypes.c_int32),
                ("spmm_pieces", ctypes.c_int32), ("spmm_row_blocks", ctypes.c_int32), ("symmetric_pattern", ctypes.c_int32)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libisp.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_2403_14853_amd.build` "
                          "(or __graft_entry__.build())" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, u32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint, ctypes.c_size_t
    P = ctypes.POINTER
    lib.isp_csr_build_workspace.argtypes = [i64, i64, i64, P(sz)]
    lib.isp_csr_build.argtypes = [i64, i64, i64, vp, vp, vp, vp, sz, u32, vp, P(vp)]
    lib.isp_csr_transpose_workspace.argtypes = [vp, P(sz)]
    lib.isp_csr_transpose_cached.argtypes = [vp, vp, sz, vp, P(vp), P(ctypes.c_int)]
    lib.isp_csr_export.argtypes = [vp, P(vp), P(vp), P(vp), P(vp)]
    lib.isp_csr_values_changed.argtypes = [vp, vp]
    lib.isp_csr_alias_workspace.argtypes = [vp, i32, P(sz)]
    lib.isp_csr_alias.argtypes = [vp, i32, vp, sz, P(vp)]
    lib.isp_csr_info.argtypes = [vp, P(CsrInfo)]
    lib.isp_spmm.argtypes = [vp, vp, i64, i32, vp, i64, vp]
    lib.isp_spmm_static_scratch.argtypes = [vp, vp, i64, i32, vp, i64, vp]
    lib.isp_sddmm.argtypes = [vp, vp, i64, vp, i64, i32, u32, vp, vp]
    lib.isp_fusedmm.argtypes = [vp, vp, i64, i32, ctypes.c_int, vp, i64, vp]
    lib.isp_fusedmm_backward.argtypes = [vp, vp, i64, vp, i64, i32, ctypes.c_int, vp, i64, vp]
    lib.isp_spmm_reduce.argtypes = [vp, vp, i64, i32, ctypes.c_int, vp, i64, vp, vp]
    lib.isp_spmm_reduce_backward.argtypes = [vp, vp, i64, i32, ctypes.c_int, vp, vp, i64, vp]
    lib.isp_csr_destroy.argtypes = [vp]
    lib.isp_csr_destroy.restype = None
    for name in EXPORTED_SYMBOLS:
        fn = getattr(lib, name)
        if name in ("isp_last_error", "isp_version"):
            fn.restype = ctypes.c_char_p
        elif name != "isp_csr_destroy":
            fn.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise IspError(status, load_library().isp_last_error().decode())


def _stream(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _dptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _workspace(nbytes: int, device):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class CSR:
    """A library handle plus the tensors it borrows.  Create with :func:`csr_build`."""

    def __init__(self, handle, n_rows, n_cols, nnz, keep, owner=None):
        self._h = handle
        self.n_rows, self.n_cols, self.nnz = n_rows, n_cols, nnz
        self._keep = keep          # tensors the C side points into
        self._owner = owner        # the source CSR for a cached transpose
        self._At = None

    @property
    def handle(self):
        return self._h

    def info(self) -> dict:
        ci = CsrInfo()
        _check(load_library().isp_csr_info(self._h, ctypes.byref(ci)))
        out = {k: getattr(ci, k) for k, _ in CsrInfo._fields_}
        out["bin_rows"] = list(ci.bin_rows)
        out["bin_nnz"] = list(ci.bin_nnz)
        return out

    def export(self):
        """Copies of the handle's CSR arrays as torch tensors: (indptr, indices, values|None, perm|None)."""
        import torch
        lib = load_library()
        p = [ctypes.c_void_p() for _ in range(4)]
        _check(lib.isp_csr_export(self._h, *[ctypes.byref(x) for x in p]))
        dev = self._keep[0].device

        def view(ptr, n, dtype, itemsize):
            if not ptr.value:
                return None
            out = torch.empty(n, dtype=dtype, device=dev)
            if n:
                torch.cuda.synchronize()
                ctypes_copy(out.data_ptr(), ptr.value, n * itemsize)
            return out

        return (view(p[0], self.n_rows + 1, torch.int64, 8), view(p[1], self.nnz, torch.int32, 4),
                view(p[2], self.nnz, torch.float32, 4), view(p[3], self.nnz, torch.int32, 4))

    def destroy(self):
        if self._h is not None and self._owner is None:
            load_library().isp_csr_destroy(self._h)
        self._h = None
        if self._At is not None:
            self._At._h = None
        self._keep = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


_hip = None


def ctypes_copy(dst_ptr: int, src_ptr: int, nbytes: int):
    """Device-to-device copy through the HIP runtime (used only by CSR.export)."""
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
        _hip.hipMemcpy.restype = ctypes.c_int
    rc = _hip.hipMemcpy(dst_ptr, src_ptr, nbytes, 3)  # hipMemcpyDeviceToDevice
    if rc != 0:
        raise RuntimeError("hipMemcpy failed with %d" % rc)


def csr_build_workspace(n_rows, n_cols, nnz) -> int:
    """isp_csr_build_workspace: bytes of device workspace isp_csr_build needs."""
    need = ctypes.c_size_t()
    _check(load_library().isp_csr_build_workspace(int(n_rows), int(n_cols), int(nnz), ctypes.byref(need)))
    return int(need.value)


def csr_transpose_workspace(A: "CSR") -> int:
    """isp_csr_transpose_workspace: bytes of device workspace the first transpose of A needs."""
    need = ctypes.c_size_t()
    _check(load_library().isp_csr_transpose_workspace(A._h, ctypes.byref(need)))
    return int(need.value)


def _own_workspace(workspace, nbytes, device):
    """The caller's uint8 CUDA tensor when given (checked for size), else a fresh allocation."""
    if workspace is None:
        return _workspace(nbytes, device)
    import torch
    assert workspace.is_cuda and workspace.dtype == torch.uint8 and workspace.is_contiguous()
    assert workspace.numel() >= nbytes, "workspace too small: %d < %d bytes" % (workspace.numel(), nbytes)
    return workspace


def csr_build(indptr, indices, values=None, n_cols=None, *, trusted=False, stream=None, workspace=None) -> CSR:
    """isp_csr_build on torch CUDA tensors (indptr int64, indices int32, values fp32 or None).
    workspace: optional uint8 CUDA tensor of at least csr_build_workspace() bytes (kept alive by the handle)."""
    import torch
    lib = load_library()
    assert indptr.is_cuda and indptr.dtype == torch.int64 and indptr.is_contiguous()
    assert indices.dtype == torch.int32 and indices.is_contiguous()
    assert values is None or (values.dtype == torch.float32 and values.is_contiguous())
    n_rows = indptr.numel() - 1
    nnz = indices.numel()
    n_cols = n_rows if n_cols is None else int(n_cols)
    need = ctypes.c_size_t()
    _check(lib.isp_csr_build_workspace(n_rows, n_cols, nnz, ctypes.byref(need)))
    ws = _own_workspace(workspace, need.value, indptr.device)
    h = ctypes.c_void_p()
    _check(lib.isp_csr_build(n_rows, n_cols, nnz, _dptr(indptr), _dptr(indices), _dptr(values), _dptr(ws),
                             ws.numel(), ISP_TRUSTED if trusted else 0, _stream(stream), ctypes.byref(h)))
    return CSR(h, n_rows, n_cols, nnz, [indptr, indices, values, ws])


def csr_transpose_cached(A: CSR, *, stream=None, workspace=None):
    """isp_csr_transpose_cached.  Returns (At, was_cached).
    workspace: optional uint8 CUDA tensor of at least csr_transpose_workspace(A) bytes, used on a cache miss."""
    lib = load_library()
    At_h = ctypes.c_void_p()
    was = ctypes.c_int(0)
    if A._At is not None:
        _check(lib.isp_csr_transpose_cached(A._h, None, 0, _stream(stream), ctypes.byref(At_h), ctypes.byref(was)))
        assert At_h.value == A._At._h.value
        return A._At, bool(was.value)
    need = ctypes.c_size_t()
    _check(lib.isp_csr_transpose_workspace(A._h, ctypes.byref(need)))
    ws = _own_workspace(workspace, need.value, A._keep[0].device)
    _check(lib.isp_csr_transpose_cached(A._h, _dptr(ws), ws.numel(), _stream(stream), ctypes.byref(At_h),
                                        ctypes.byref(was)))
    A._keep.append(ws)
    A._At = CSR(At_h, A.n_cols, A.n_rows, A.nnz, [ws], owner=A)
    return A._At, bool(was.value)


def csr_alias_workspace(A: CSR, max_d: int = 256) -> int:
    """isp_csr_alias_workspace: bytes of device workspace an alias of A needs."""
    need = ctypes.c_size_t()
    _check(load_library().isp_csr_alias_workspace(A._h, int(max_d), ctypes.byref(need)))
    return int(need.value)


def csr_alias(A: CSR, max_d: int = 256, *, workspace=None) -> CSR:
    """isp_csr_alias: a second handle on A's matrix with scratch of its own, whose calls may overlap A's.
    The alias keeps A alive; destroy it (or drop it) before destroying A."""
    lib = load_library()
    ws = _own_workspace(workspace, csr_alias_workspace(A, max_d), A._keep[0].device)
    h = ctypes.c_void_p()
    _check(lib.isp_csr_alias(A._h, int(max_d), _dptr(ws), ws.numel(), ctypes.byref(h)))
    B = CSR(h, A.n_rows, A.n_cols, A.nnz, [A._keep[0], ws, A])
    if A._At is not None:  # the alias's own copy of the cached transpose (a cache hit: no device work)
        At_h = ctypes.c_void_p()
        _check(lib.isp_csr_transpose_cached(h, None, 0, None, ctypes.byref(At_h), None))
        B._At = CSR(At_h, A.n_cols, A.n_rows, A.nnz, [ws], owner=B)
    return B


def csr_values_changed(A: CSR, *, stream=None):
    """isp_csr_values_changed: the caller has rewritten A's values tensor in place; the cached transpose's
    values are gathered again, everything else stays cached."""
    _check(load_library().isp_csr_values_changed(A._h, _stream(stream)))


def _ld(t):
    assert t.dim() == 2 and t.stride(1) == 1 and t.is_cuda
    import torch
    assert t.dtype == torch.float32
    return int(t.stride(0)) if t.shape[0] > 1 else max(int(t.stride(0)), int(t.shape[1]))


def spmm(A: CSR, X, Y, *, stream=None):
    """isp_spmm: Y = A X (Y is overwritten)."""
    d = X.shape[1]
    assert X.shape[0] == A.n_cols and Y.shape == (A.n_rows, d)
    _check(load_library().isp_spmm(A._h, _dptr(X), _ld(X), d, _dptr(Y), _ld(Y), _stream(stream)))
    return Y


def spmm_static_scratch(A: CSR, X, Y, *, stream=None):
    """isp_spmm_static_scratch: isp_spmm with the hub-row partial sums in the library's static device array."""
    d = X.shape[1]
    assert X.shape[0] == A.n_cols and Y.shape == (A.n_rows, d)
    _check(load_library().isp_spmm_static_scratch(A._h, _dptr(X), _ld(X), d, _dptr(Y), _ld(Y), _stream(stream)))
    return Y


def sddmm(A: CSR, U, V, out, *, scale_by_a=False, stream=None):
    """isp_sddmm: out[p] = <U[row(p)], V[col(p)]>."""
    d = U.shape[1]
    assert U.shape[0] == A.n_rows and V.shape == (A.n_cols, d) and out.numel() == A.nnz
    _check(load_library().isp_sddmm(A._h, _dptr(U), _ld(U), _dptr(V), _ld(V), d,
                                    ISP_SCALE_BY_A if scale_by_a else 0, _dptr(out), _stream(stream)))
    return out


def fusedmm(A: CSR, X, Y, *, op=ISP_OP_SIGMOID, stream=None):
    """isp_fusedmm forward; op is ISP_OP_* or one of 'sigmoid', 'dot', 'one'."""
    op = EDGE_OPS.get(op, op)
    d = X.shape[1]
    assert X.shape[0] == A.n_rows and Y.shape == X.shape
    _check(load_library().isp_fusedmm(A._h, _dptr(X), _ld(X), d, op, _dptr(Y), _ld(Y), _stream(stream)))
    return Y


def fusedmm_backward(A: CSR, X, dY, dX, *, op=ISP_OP_SIGMOID, stream=None):
    """isp_fusedmm_backward (needs csr_transpose_cached(A) first)."""
    op = EDGE_OPS.get(op, op)
    d = X.shape[1]
    assert dY.shape == X.shape and dX.shape == X.shape
    _check(load_library().isp_fusedmm_backward(A._h, _dptr(X), _ld(X), _dptr(dY), _ld(dY), d, op, _dptr(dX),
                                               _ld(dX), _stream(stream)))
    return dX


REDUCE = {"sum": 0, "mean": 1, "min": 2, "max": 3}


def spmm_reduce(A: CSR, X, Y, reduce: str, arg=None, *, stream=None):
    """isp_spmm_reduce: reduce in 'sum' | 'mean' | 'min' | 'max'; arg (int32 [n_rows, d], contiguous) for min / max."""
    import torch
    d = X.shape[1]
    assert X.shape[0] == A.n_cols and Y.shape == (A.n_rows, d)
    if arg is not None:
        assert arg.dtype == torch.int32 and arg.is_contiguous() and arg.shape == (A.n_rows, d)
    _check(load_library().isp_spmm_reduce(A._h, _dptr(X), _ld(X), d, REDUCE[reduce], _dptr(Y), _ld(Y), _dptr(arg),
                                          _stream(stream)))
    return Y


def spmm_reduce_backward(A: CSR, dY, dX, reduce: str, arg=None, *, stream=None):
    """isp_spmm_reduce_backward (needs csr_transpose_cached(A) first)."""
    d = dY.shape[1]
    assert dY.shape[0] == A.n_rows and dX.shape == (A.n_cols, d)
    _check(load_library().isp_spmm_reduce_backward(A._h, _dptr(dY), _ld(dY), d, REDUCE[reduce], _dptr(arg),
                                                   _dptr(dX), _ld(dX), _stream(stream)))
    return dX
