"""MI355X-native sparse GNN hot path (SpMM, cached-transpose backward, SDDMM, FusedMM).

Thin ctypes binding over the C-ABI library ``libisp.so`` (see ``include/isp.h``).  The binding
only marshals arguments: every step of the path runs in the library's HIP kernels.  PyTorch is
used for device memory and streams.  There is no CPU fallback: without the compiled library
the import of :mod:`paper_2403_14853_amd.binding` fails loudly.
"""
from .binding import (  # noqa: F401
    CSR, IspError, lib_path, load_library, csr_build, csr_build_workspace, csr_transpose_cached,
    csr_transpose_workspace, csr_values_changed, csr_alias, csr_alias_workspace, spmm, spmm_static_scratch, sddmm, fusedmm,
    fusedmm_backward, spmm_reduce, spmm_reduce_backward, EXPORTED_SYMBOLS,
)
