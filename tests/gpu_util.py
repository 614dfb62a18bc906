"""Helpers for the GPU parity tests: move a generated workload to the device, build handles,
and compare against the oracle with the per-element tolerance."""
import numpy as np
import torch

import paper_2403_14853_amd as isp

REL, ABS = 1e-5, 1e-6  # |gpu - oracle| <= REL * magnitude + ABS, per element


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def build(indptr, indices, values, n_cols=None):
    return isp.csr_build(dev(indptr), dev(indices), dev(values), n_cols=n_cols)


def worst_ratio(gpu, ref, mag):
    """max over elements of |gpu - ref| / (REL * mag + ABS); parity holds when <= 1."""
    g = gpu.detach().cpu().numpy().astype(np.float64).reshape(-1)
    if g.size == 0:
        return 0.0
    r = np.asarray(ref, dtype=np.float64).reshape(-1)
    m = np.asarray(mag, dtype=np.float64).reshape(-1)
    assert np.all(np.isfinite(g)), "non-finite GPU output"
    return float(np.max(np.abs(g - r) / (REL * m + ABS)))


def assert_close(gpu, ref, mag, what=""):
    w = worst_ratio(gpu, ref, mag)
    assert w <= 1.0, "%s: error is %.3g x the tolerance" % (what, w)


def sub_csr(indptr, indices, values, rows):
    """CSR made of the selected rows only (for sampled full-size checks)."""
    rows = np.asarray(rows, dtype=np.int64)
    lens = indptr[rows + 1] - indptr[rows]
    sp = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    pos = np.concatenate([np.arange(indptr[r], indptr[r + 1]) for r in rows]) if len(rows) else np.zeros(0, np.int64)
    pos = pos.astype(np.int64)
    return sp, indices[pos], (None if values is None else values[pos]), pos
