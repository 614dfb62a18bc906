// isp_csr_alias: a second handle on the same matrix whose calls may overlap the first one's.
//
// The kernels of a handle keep the partial sums of hub-row segments (and, in the min / max backward, one mark
// per entry) in that handle's workspace, so two calls on one handle that run at the same time on two streams
// would overwrite each other's partial rows.  An alias shares everything that is only read - the caller's
// CSR arrays, the work partitions, the packed SpMM layout, the cached transpose's arrays - and keeps what a
// call writes in a workspace of its own.
#include <new>
#include "isp_internal.h"

namespace {

struct alias_layout {
  int64_t rows_a, rows_t;   // partial rows for the handle and for its transpose
  size_t off_t, off_flags;  // byte offsets of the transpose's partial rows and of its entry marks
  size_t total;
};

// Partial rows one launch on h may touch: one per hub-row segment and column group (FusedMM wider than 256
// columns stores `groups` groups of 256 columns per segment and launch), one per piece of the packed layout.
int64_t rows_needed(const isp_csr* h, int64_t groups) {
  int64_t r = (int64_t)h->v.n_seg * groups;
  if (h->has_packed && h->info.spmm_pieces > r) r = h->info.spmm_pieces;
  return r > 0 ? r : 1;
}

alias_layout make_alias_layout(const isp_csr* A, int32_t max_d) {
  const int64_t groups = (max_d + ISP_PARTIAL_TILE - 1) / ISP_PARTIAL_TILE;
  alias_layout L;
  L.rows_a = rows_needed(A, groups);
  L.rows_t = A->At ? rows_needed(A->At, groups) : 0;
  size_t off = isp_align((size_t)L.rows_a * ISP_PARTIAL_TILE * sizeof(float));
  L.off_t = off;
  off += isp_align((size_t)L.rows_t * ISP_PARTIAL_TILE * sizeof(float));
  L.off_flags = off;
  if (A->At) off += isp_align((size_t)A->v.nnz + 4);  // (cleared in 32-bit words)
  L.total = off;
  return L;
}

isp_status check_source(const isp_csr* A, int32_t max_d) {
  if (!A) return isp_fail(ISP_EINVAL, "handle is NULL");
  if (A->is_transpose) return isp_fail(ISP_EINVAL, "pass the source handle, not its transpose (the alias carries its own)");
  if (A->source) return isp_fail(ISP_EINVAL, "pass the handle isp_csr_build returned, not an alias of it");
  if (max_d <= 0) return isp_fail(ISP_EINVAL, "max_d must be positive");
  return ISP_OK;
}

}  // namespace

extern "C" isp_status isp_csr_alias_workspace(const isp_csr_t* A, int32_t max_d, size_t* bytes) {
  isp_status st = check_source(A, max_d);
  if (st != ISP_OK) return st;
  if (!bytes) return isp_fail(ISP_EINVAL, "bytes is NULL");
  *bytes = make_alias_layout(A, max_d).total;
  return ISP_OK;
}

extern "C" isp_status isp_csr_alias(const isp_csr_t* A, int32_t max_d, void* workspace, size_t workspace_bytes,
                                    isp_csr_t** out) {
  isp_status st = check_source(A, max_d);
  if (st != ISP_OK) return st;
  if (!out) return isp_fail(ISP_EINVAL, "out is NULL");
  *out = nullptr;
  if ((st = isp_check_device(A)) != ISP_OK) return st;
  const alias_layout L = make_alias_layout(A, max_d);
  if (!workspace) return isp_fail(ISP_EINVAL, "workspace is NULL");
  if (((uintptr_t)workspace & 255) != 0) return isp_fail(ISP_EINVAL, "workspace must be 256-byte aligned");
  if (workspace_bytes < L.total)
    return isp_fail(ISP_EINVAL, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, L.total);
  char* base = static_cast<char*>(workspace);

  isp_csr* B = new (std::nothrow) isp_csr(*A);
  if (!B) return isp_fail(ISP_ENOMEM, "host allocation of the handle failed");
  B->source = A;
  B->source_gen = A->values_gen;
  B->At = nullptr;
  // Every partial row a launch reads was written by that launch before, so the workspace needs no clearing.
  B->v.partials = reinterpret_cast<float*>(base);
  B->vp.partials = B->v.partials;  // (a call runs on one of the two partitions, never on both)
  B->partial_rows = L.rows_a;
  if (A->At) {
    isp_csr* Bt = new (std::nothrow) isp_csr(*A->At);
    if (!Bt) { delete B; return isp_fail(ISP_ENOMEM, "host allocation of the handle failed"); }
    Bt->source = A;
    Bt->source_gen = A->values_gen;
    Bt->At = nullptr;
    Bt->v.partials = reinterpret_cast<float*>(base + L.off_t);
    Bt->vp.partials = Bt->v.partials;
    Bt->partial_rows = L.rows_t;
    // The marks of the min / max backward are written by every call: the alias's own.  What the transpose
    // caches on first use besides (value / row length, the inverse permutation) is a pure function of the
    // shared arrays and stays shared: whichever handle fills it first writes the same numbers any other would.
    Bt->sel_flags = reinterpret_cast<uint8_t*>(base + L.off_flags);
    B->At = Bt;
  }
  *out = B;
  return ISP_OK;
}
