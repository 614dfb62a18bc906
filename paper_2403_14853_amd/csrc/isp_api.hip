// The C ABI (include/isp.h): argument checks, error reporting, dispatch.  No device code here.
#include <stdarg.h>
#include <stdio.h>
#include "isp_internal.h"

namespace {
thread_local char g_err[512] = "";
}

isp_status isp_fail(isp_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

extern "C" {

const char* isp_last_error(void) { return g_err; }
const char* isp_version(void) { return "isp-gfx950 0.1"; }

static isp_status check_shape(int64_t n_rows, int64_t n_cols, int64_t nnz) {
  if (n_rows < 0 || n_cols < 0 || nnz < 0) return isp_fail(ISP_EINVAL, "negative size");
  const int64_t lim = 2147483646;
  if (n_rows > lim || n_cols > lim || nnz > lim)
    return isp_fail(ISP_EUNSUPPORTED, "n_rows, n_cols and nnz must be below 2^31 - 1");
  return ISP_OK;
}

isp_status isp_csr_build_workspace(int64_t n_rows, int64_t n_cols, int64_t nnz, size_t* bytes) {
  if (!bytes) return isp_fail(ISP_EINVAL, "bytes is NULL");
  isp_status st = check_shape(n_rows, n_cols, nnz);
  if (st != ISP_OK) return st;
  *bytes = isp_partition_workspace(n_rows, n_cols, nnz);
  return ISP_OK;
}

isp_status isp_csr_build(int64_t n_rows, int64_t n_cols, int64_t nnz, const int64_t* indptr, const int32_t* indices,
                         const float* values, void* workspace, size_t workspace_bytes, unsigned flags, void* stream,
                         isp_csr_t** out) {
  if (!out) return isp_fail(ISP_EINVAL, "out is NULL");
  *out = nullptr;
  isp_status st = check_shape(n_rows, n_cols, nnz);
  if (st != ISP_OK) return st;
  if (!indptr) return isp_fail(ISP_EINVAL, "indptr is NULL");
  if (nnz > 0 && !indices) return isp_fail(ISP_EINVAL, "indices is NULL");
  if (!workspace) return isp_fail(ISP_EINVAL, "workspace is NULL");
  if (flags & ~ISP_TRUSTED) return isp_fail(ISP_EUNSUPPORTED, "unknown flag bits 0x%x", flags & ~ISP_TRUSTED);
  if (n_rows == 0 && nnz != 0) return isp_fail(ISP_EBADCSR, "nnz must be 0 when n_rows is 0");
  return isp_build_handle(n_rows, n_cols, nnz, indptr, indices, values, workspace, workspace_bytes,
                          !(flags & ISP_TRUSTED), (hipStream_t)stream, out);
}

}  // extern "C"

// The handle's arrays live on the device that was current when it was built.
isp_status isp_check_device(const isp_csr* A) {
  int dev = -1;
  ISP_HIP(hipGetDevice(&dev));
  if (dev != A->device)
    return isp_fail(ISP_EINVAL, "the handle was built on device %d, the current device is %d", A->device, dev);
  if (A->source && A->source_gen != A->source->values_gen)
    return isp_fail(ISP_EINVAL, "isp_csr_values_changed ran on the source handle after this alias was made: "
                    "destroy the alias and make a new one");
  return ISP_OK;
}

isp_status isp_check_dense(const void* p, int64_t ld, int32_t d, int64_t rows, const char* name) {
  if (d <= 0) return isp_fail(ISP_EINVAL, "d must be positive");
  if (rows > 0 && !p) return isp_fail(ISP_EINVAL, "%s is NULL", name);
  if (ld < d) return isp_fail(ISP_EINVAL, "leading dimension of %s (%lld) is smaller than d (%d)", name, (long long)ld, d);
  return ISP_OK;
}

extern "C" {

isp_status isp_csr_transpose_workspace(const isp_csr_t* A, size_t* bytes) {
  if (!A || !bytes) return isp_fail(ISP_EINVAL, "NULL argument");
  *bytes = isp_transpose_workspace_bytes(A->v.n_rows, A->v.n_cols, A->v.nnz, A->v.values != nullptr);
  return ISP_OK;
}

isp_status isp_csr_transpose_cached(isp_csr_t* A, void* workspace, size_t workspace_bytes, void* stream,
                                    const isp_csr_t** At, int* was_cached) {
  if (!A || !At) return isp_fail(ISP_EINVAL, "NULL argument");
  if (A->is_transpose) return isp_fail(ISP_EINVAL, "the handle is itself a cached transpose");
  if (A->At) {  // cache hit: no device work
    *At = A->At;
    if (was_cached) *was_cached = 1;
    return ISP_OK;
  }
  if (was_cached) *was_cached = 0;
  if (A->source)
    return isp_fail(ISP_EINVAL, "an alias takes its transpose from its source handle: call isp_csr_transpose_cached "
                    "on that handle first, then make the alias");
  isp_status st = isp_check_device(A);
  if (st != ISP_OK) return st;
  st = isp_transpose_build(A, workspace, workspace_bytes, (hipStream_t)stream);
  if (st != ISP_OK) return st;
  *At = A->At;
  return ISP_OK;
}

isp_status isp_csr_values_changed(isp_csr_t* A, void* stream) {
  if (!A) return isp_fail(ISP_EINVAL, "handle is NULL");
  if (A->is_transpose) return isp_fail(ISP_EINVAL, "pass the source handle, not its transpose");
  if (A->source) return isp_fail(ISP_EINVAL, "pass the handle isp_csr_build returned, not an alias of it");
  isp_status st = isp_check_device(A);
  if (st != ISP_OK) return st;
  ++A->values_gen;  // aliases made before this call are refused from now on
  // everything derived from the values, in stream order: the packed SpMM layout's copy, the transposed values
  // (and what the mean backward keeps of them), the transpose's own packed copy
  if ((st = isp_refresh_packed_values(A, (hipStream_t)stream)) != ISP_OK) return st;
  if ((st = isp_transpose_refresh_values(A, (hipStream_t)stream)) != ISP_OK) return st;
  return A->At ? isp_refresh_packed_values(A->At, (hipStream_t)stream) : ISP_OK;
}

isp_status isp_csr_export(const isp_csr_t* A, const int64_t** indptr, const int32_t** indices, const float** values,
                          const int32_t** perm) {
  if (!A) return isp_fail(ISP_EINVAL, "handle is NULL");
  if (indptr) *indptr = A->v.indptr;
  if (indices) *indices = A->v.indices;
  if (values) *values = A->v.values;
  if (perm) *perm = A->perm;
  return ISP_OK;
}

isp_status isp_csr_info(const isp_csr_t* A, isp_csr_info_t* info) {
  if (!A || !info) return isp_fail(ISP_EINVAL, "NULL argument");
  *info = A->info;
  return ISP_OK;
}

isp_status isp_spmm(const isp_csr_t* A, const float* X, int64_t ldx, int32_t d, float* Y, int64_t ldy, void* stream) {
  if (!A) return isp_fail(ISP_EINVAL, "handle is NULL");
  isp_status st;
  if ((st = isp_check_device(A)) != ISP_OK) return st;
  if ((st = isp_check_dense(X, ldx, d, A->v.nnz > 0 ? A->v.n_cols : 0, "X")) != ISP_OK) return st;
  if ((st = isp_check_dense(Y, ldy, d, A->v.n_rows, "Y")) != ISP_OK) return st;
  return isp_spmm_launch(A, X, ldx, d, Y, ldy, (hipStream_t)stream);
}

isp_status isp_sddmm(const isp_csr_t* A, const float* U, int64_t ldu, const float* V, int64_t ldv, int32_t d,
                     unsigned flags, float* out, void* stream) {
  if (!A) return isp_fail(ISP_EINVAL, "handle is NULL");
  if (flags & ~ISP_SCALE_BY_A) return isp_fail(ISP_EUNSUPPORTED, "unknown flag bits 0x%x", flags & ~ISP_SCALE_BY_A);
  isp_status st;
  if ((st = isp_check_device(A)) != ISP_OK) return st;
  const int64_t live = A->v.nnz > 0 ? 1 : 0;
  if ((st = isp_check_dense(U, ldu, d, live * A->v.n_rows, "U")) != ISP_OK) return st;
  if ((st = isp_check_dense(V, ldv, d, live * A->v.n_cols, "V")) != ISP_OK) return st;
  if (A->v.nnz > 0 && !out) return isp_fail(ISP_EINVAL, "out is NULL");
  return isp_sddmm_launch(A, U, ldu, V, ldv, d, (flags & ISP_SCALE_BY_A) != 0, out, (hipStream_t)stream);
}

static isp_status check_fused(const isp_csr_t* A, int32_t d, int op) {
  if (!A) return isp_fail(ISP_EINVAL, "handle is NULL");
  if (op != ISP_OP_SIGMOID && op != ISP_OP_DOT && op != ISP_OP_ONE)
    return isp_fail(ISP_EUNSUPPORTED, "unknown edge op %d", op);
  if (A->v.n_rows != A->v.n_cols) return isp_fail(ISP_EINVAL, "FusedMM needs a square matrix");
  if (d > 4 * ISP_PARTIAL_TILE) return isp_fail(ISP_EUNSUPPORTED, "FusedMM supports d <= %d", 4 * ISP_PARTIAL_TILE);
  return isp_check_device(A);
}

isp_status isp_fusedmm(const isp_csr_t* A, const float* X, int64_t ldx, int32_t d, int op, float* Y, int64_t ldy,
                       void* stream) {
  isp_status st;
  if ((st = check_fused(A, d, op)) != ISP_OK) return st;
  if ((st = isp_check_dense(X, ldx, d, A->v.n_rows, "X")) != ISP_OK) return st;
  if ((st = isp_check_dense(Y, ldy, d, A->v.n_rows, "Y")) != ISP_OK) return st;
  return isp_fusedmm_launch(A, X, ldx, d, op, Y, ldy, (hipStream_t)stream);
}

isp_status isp_fusedmm_backward(isp_csr_t* A, const float* X, int64_t ldx, const float* dY, int64_t lddy, int32_t d,
                                int op, float* dX, int64_t lddx, void* stream) {
  isp_status st;
  if ((st = check_fused(A, d, op)) != ISP_OK) return st;
  if (!A->At) return isp_fail(ISP_EINVAL, "call isp_csr_transpose_cached on the handle first");
  if ((st = isp_check_dense(X, ldx, d, A->v.n_rows, "X")) != ISP_OK) return st;
  if ((st = isp_check_dense(dY, lddy, d, A->v.n_rows, "dY")) != ISP_OK) return st;
  if ((st = isp_check_dense(dX, lddx, d, A->v.n_rows, "dX")) != ISP_OK) return st;
  return isp_fusedmm_bwd_launch(A, X, ldx, dY, lddy, d, op, dX, lddx, (hipStream_t)stream);
}

isp_status isp_spmm_reduce(const isp_csr_t* A, const float* X, int64_t ldx, int32_t d, int reduce, float* Y,
                           int64_t ldy, int32_t* arg, void* stream) {
  if (reduce == ISP_REDUCE_SUM) return isp_spmm(A, X, ldx, d, Y, ldy, stream);
  if (!A) return isp_fail(ISP_EINVAL, "handle is NULL");
  if (reduce != ISP_REDUCE_MEAN && reduce != ISP_REDUCE_MIN && reduce != ISP_REDUCE_MAX)
    return isp_fail(ISP_EUNSUPPORTED, "unknown reduction %d", reduce);
  isp_status st;
  if ((st = isp_check_device(A)) != ISP_OK) return st;
  if ((st = isp_check_dense(X, ldx, d, A->v.nnz > 0 ? A->v.n_cols : 0, "X")) != ISP_OK) return st;
  if ((st = isp_check_dense(Y, ldy, d, A->v.n_rows, "Y")) != ISP_OK) return st;
  if (reduce != ISP_REDUCE_MEAN && A->v.n_rows > 0 && !arg) return isp_fail(ISP_EINVAL, "arg is NULL");
  return isp_spmm_reduce_launch(A, X, ldx, d, reduce, Y, ldy, arg, (hipStream_t)stream);
}

isp_status isp_spmm_reduce_backward(isp_csr_t* A, const float* dY, int64_t lddy, int32_t d, int reduce,
                                    const int32_t* arg, float* dX, int64_t lddx, void* stream) {
  if (!A) return isp_fail(ISP_EINVAL, "handle is NULL");
  if (A->is_transpose) return isp_fail(ISP_EINVAL, "pass the source handle, not its transpose");
  if (!A->At) return isp_fail(ISP_EINVAL, "call isp_csr_transpose_cached on the handle first");
  if (reduce == ISP_REDUCE_SUM) return isp_spmm(A->At, dY, lddy, d, dX, lddx, stream);
  if (reduce != ISP_REDUCE_MEAN && reduce != ISP_REDUCE_MIN && reduce != ISP_REDUCE_MAX)
    return isp_fail(ISP_EUNSUPPORTED, "unknown reduction %d", reduce);
  isp_status st;
  if ((st = isp_check_device(A)) != ISP_OK) return st;
  if ((st = isp_check_dense(dY, lddy, d, A->v.nnz > 0 ? A->v.n_rows : 0, "dY")) != ISP_OK) return st;
  if ((st = isp_check_dense(dX, lddx, d, A->v.n_cols, "dX")) != ISP_OK) return st;
  if (reduce != ISP_REDUCE_MEAN && A->v.nnz > 0 && !arg) return isp_fail(ISP_EINVAL, "arg is NULL");
  return isp_spmm_reduce_bwd_launch(A, dY, lddy, d, reduce, arg, dX, lddx, (hipStream_t)stream);
}

void isp_csr_destroy(isp_csr_t* A) {
  if (!A) return;
  if (A->is_transpose) return;  // owned by its source handle
  delete A->At;
  delete A;
}

}  // extern "C"
