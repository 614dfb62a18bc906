/*
 * isp.h -- C ABI of the MI355X (gfx950) sparse GNN hot path.
 *
 * Operations (iSpLib, arXiv 2403.14853):
 *   SpMM   Y = A X, sum reduction, A in CSR, X dense row-major fp32      (abstract; Sections 1, 3.4, 3.5)
 *   SpMM backward dX = A^T dY through a CSR transpose that is built once
 *          and kept in A's handle                                        (Section 3.3, cache-enabled backprop)
 *   SDDMM  one dot product per stored entry of A (gives dA of SpMM)       (Section 1)
 *   FusedMM SDDMM -> edge function -> SpMM in one pass, edge matrix never
 *          written; sigmoid instance, forward and backward               (Section 1(a))
 *
 * General conventions
 *   - Every array pointer is a DEVICE pointer on the current HIP device unless its name starts
 *     with h_.  The caller allocates and owns every buffer, including workspaces, and must keep
 *     them alive and unmodified while a handle that refers to them lives.  The library never
 *     allocates or frees device memory.
 *   - CSR: indptr int64[n_rows+1], indices int32[nnz], values fp32[nnz] or NULL (all ones).
 *     Columns inside a row may be unsorted and may repeat; a repeated column is a separate
 *     stored entry (SpMM adds them, SDDMM emits one output per stored entry).
 *   - Dense matrices are fp32 row-major; ld* is the distance between rows in elements (>= d).  Any ld and
 *     alignment is accepted; rows that start on 128-byte lines (ld a multiple of 32, base pointer aligned)
 *     gather fastest.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).  Compute calls are
 *     asynchronous on it.  isp_csr_build and a cache-missing isp_csr_transpose_cached
 *     synchronise the stream once, to read a few counters back.
 *   - Outputs are overwritten (Y = A X, not +=).  n_rows = 0 and nnz = 0 are valid.
 *   - Every function returns a status; nothing throws or aborts across this boundary.  After a
 *     failure isp_last_error() returns a thread-local message.
 *   - A handle belongs to the HIP device that was current when it was built; using it with another device
 *     current yields ISP_EINVAL.
 *   - Calls that use the same handle (or a handle and its cached transpose) on different streams
 *     at the same time race on the handle's scratch (hub-row partial sums); serialise them.
 *   - Results are run-to-run bitwise deterministic: no floating-point atomics are used.
 *   - Environment variables (tuning and tests only; none is needed).  All are read when isp_csr_build runs and
 *     are kept in the handle; no compute call reads the environment.  (The partition sizes of a cached transpose
 *     are read when it is built, by the first isp_csr_transpose_cached call and its workspace query; the other
 *     settings it inherits from its source.)
 *       ISP_BLOCK_COST, ISP_HUB_THRESHOLD, ISP_SEGMENT_LEN, ISP_BANDS, ISP_MIN_PIECE, ISP_MID_THRESHOLD,
 *       ISP_PACKED_BLOCK:
 *                              sizes of the work partition (clamped to what the kernels' tables hold)
 *       ISP_NO_GROUPED         run every operation on the general kernels
 *       ISP_SPMM_LPG, ISP_SPMM_TILE   lanes per group / feature columns per launch of the tuned SpMM
 *       ISP_SDDMM_ONE_PASS     SDDMM keeps 128-column rows in one pass
 *       ISP_NO_MIRROR          the FusedMM backward always runs its two passes, also on symmetric patterns
 *       ISP_FUSED_W            4 / 8: the tuned SDDMM / FusedMM kernels give a lane one / two float4 at every width above 32
 *       ISP_WIDE_GROUPS        most 256-column groups a split row stores per launch of a FusedMM pass wider than 256
 *     isp_csr_build_workspace reads the partition sizes too, so set them before both calls or not at all.
 */
#ifndef ISP_H
#define ISP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct isp_csr isp_csr_t; /* opaque; host-side struct owned by the library */

typedef enum {
  ISP_OK = 0,
  ISP_EINVAL = 1,       /* NULL pointer, negative size, d <= 0, ld < d, workspace too small or misaligned */
  ISP_EBADCSR = 2,      /* indptr not monotone / indptr[0] != 0 / indptr[n] != nnz / column out of range */
  ISP_ENOMEM = 3,       /* host allocation failed */
  ISP_EHIP = 4,         /* a HIP runtime call failed; text in isp_last_error() */
  ISP_EUNSUPPORTED = 5  /* size beyond what the index types hold, or an unknown op / flag */
} isp_status;

/* flags of isp_csr_build */
#define ISP_TRUSTED 1u /* skip the structural validation pass (the caller vouches for the CSR) */
/* flags of isp_sddmm */
#define ISP_SCALE_BY_A 1u /* multiply each dot product by the entry's value */
/* op of isp_fusedmm / isp_fusedmm_backward: the edge function s = f(z) applied to z = <x_i, x_j> */
#define ISP_OP_SIGMOID 0 /* f(z) = 1 / (1 + exp(-z)) */
#define ISP_OP_DOT 1     /* f(z) = z */
#define ISP_OP_ONE 2     /* f(z) = 1: plain aggregation through the fused path */

/* Summary of a handle's row classes and work partition (all counts are rows unless named). */
typedef struct {
  int64_t n_rows, n_cols, nnz;
  int64_t max_degree;
  int64_t bin_rows[5]; /* degree 0 | 1..4 | 5..32 | 33..hub_threshold | > hub_threshold (hub) */
  int64_t bin_nnz[5];
  int32_t hub_threshold;  /* rows longer than this are split by nnz (64..512, by size)*/
  int32_t segment_len;    /* most nonzeros a hub segment holds                     */
  int32_t block_cost;     /* target (nnz + rows) per wavefront work item            */
  int32_t n_row_blocks;   /* wavefront work items made of whole short rows          */
  int32_t n_hub_rows;
  int32_t n_segments;     /* wavefront work items made of hub-row segments          */
  int32_t is_transpose;   /* 1 for a handle returned by isp_csr_transpose_cached    */
  int32_t has_cached_transpose;
  /* the packed layout the tuned SpMM runs on (large matrices with many columns; all 0 without it): rows
     longer than spmm_mid_threshold are cut into column-band pieces that share work items                 */
  int32_t spmm_mid_threshold;
  int32_t spmm_cut_rows;
  int32_t spmm_pieces;
  int32_t spmm_row_blocks; /* work items of that layout (whole short rows, or several pieces)              */
  /* 1 once the cached transpose exists and its offsets and indices equal the handle's own element for element
     (a symmetric pattern with ascending rows): the FusedMM backward then runs as one pass over the matrix     */
  int32_t symmetric_pattern;
} isp_csr_info_t;

/* Bytes of device workspace isp_csr_build needs for a matrix of this shape (upper bound). */
isp_status isp_csr_build_workspace(int64_t n_rows, int64_t n_cols, int64_t nnz, size_t* bytes);

/*
 * Wrap the caller's CSR arrays in a handle and prepare the work partition: rows are classed by
 * degree; short rows are grouped into contiguous row blocks of about equal (nnz + rows); hub rows
 * (degree > hub threshold) are cut into segments of bounded length, at column-band boundaries first,
 * which are scheduled in column order (Section 1(b): balanced scheduling; Section 3.5: CSR operand).
 * For large matrices with many columns (8 Mi .. 256 Mi entries, >= 64 Ki columns) the tuned SpMM also gets a packed
 * layout of its own: rows longer than 256 entries are cut into column-band pieces of 64 entries or more, and
 * the pieces, scheduled in column order, share work items with each other; that layout keeps a reordered copy
 * of the index and value arrays in the workspace (isp_csr_values_changed refreshes the values).
 * Integer work and copies only.  Rows with ascending columns schedule best; any order is accepted.
 *   indptr/indices/values: borrowed device arrays (values may be NULL).
 *   workspace: device memory, 256-byte aligned, >= isp_csr_build_workspace() bytes; borrowed
 *              until isp_csr_destroy.
 *   flags: 0 or ISP_TRUSTED.  Without ISP_TRUSTED a malformed CSR yields ISP_EBADCSR and no handle.
 * Synchronises `stream` once.  n_rows, n_cols < 2^31 - 1 and nnz < 2^31 - 1, else ISP_EUNSUPPORTED.
 */
isp_status isp_csr_build(int64_t n_rows, int64_t n_cols, int64_t nnz, const int64_t* indptr,
                         const int32_t* indices, const float* values, void* workspace,
                         size_t workspace_bytes, unsigned flags, void* stream, isp_csr_t** out);

/* Bytes of device workspace the first isp_csr_transpose_cached call on A needs. */
isp_status isp_csr_transpose_workspace(const isp_csr_t* A, size_t* bytes);

/*
 * A^T as a CSR handle, built on the first call and kept inside A (Section 3.3): later calls
 * return the stored handle, do no device work and ignore workspace.  The transpose is the
 * stable one: entries of a column keep their order of appearance in A, so the result is unique:
 *   t_indptr  int64[n_cols+1], t_indices int32[nnz] (source rows), perm int32[nnz] (position in
 *   A of each transposed entry), t_values[q] = values[perm[q]] (absent when A has no values).
 * These arrays live in `workspace` (256-byte aligned, borrowed until isp_csr_destroy(A)).
 *   *At: handle owned by A (never destroy it yourself).  *was_cached: 1 on a cache hit (may be NULL).
 * A cache miss synchronises `stream` once.
 */
isp_status isp_csr_transpose_cached(isp_csr_t* A, void* workspace, size_t workspace_bytes,
                                    void* stream, const isp_csr_t** At, int* was_cached);

/*
 * Tell the handle that the caller has overwritten A's values array in place (same pointer, same structure),
 * as happens every epoch when the edge values are trained from the SDDMM gradients.  What Section 3.3 caches
 * stays cached - A^T's structure, its permutation and both work partitions - and only the transposed values
 * are gathered again: t_values[q] = values[perm[q]], one asynchronous pass on `stream`; if a mean-reduction
 * backward has run on the handle, the per-entry values it keeps (value / row length) are recomputed right
 * behind it on the same stream.  Everything happens in stream order, so the call may be captured into a HIP
 * graph (every replay refreshes), and graphs captured earlier read the refreshed arrays.  What a graph cannot
 * see is a change of the cache's bookkeeping on the host: a graph captured BEFORE the first mean backward of a
 * handle contains that first call's fill pass and keeps running it on every replay - correct, only redundant.
 * A no-op for a handle without values or without a cached transpose.  A must be the source handle, not its
 * transpose.
 */
isp_status isp_csr_values_changed(isp_csr_t* A, void* stream);

/* Device pointers of a handle's CSR arrays (perm is NULL for a handle that is not a transpose;
 * values is NULL when absent).  Any out pointer may be NULL.  For inspection and tests. */
isp_status isp_csr_export(const isp_csr_t* A, const int64_t** indptr, const int32_t** indices,
                          const float** values, const int32_t** perm);

/* Fill *info (host struct) with the handle's shape, degree classes and partition sizes. */
isp_status isp_csr_info(const isp_csr_t* A, isp_csr_info_t* info);

/*
 * Overlapping calls on one matrix (Section 1(b): the work partition, and Section 3.3: the cached transpose,
 * are built once and shared).  The compute calls keep the partial sums of hub-row segments, and the min / max
 * backward its per-entry marks, in the handle's workspace, so two calls on ONE handle must not run at the same
 * time.  An alias is a second handle on the same matrix that keeps exactly that scratch in a workspace of its
 * own and shares everything else - the caller's arrays, both work partitions, the packed SpMM layout, the
 * cached transpose and its permutation: calls on A, on the alias and on other aliases may overlap freely
 * (different streams or threads); calls on one alias must still follow each other.  Results are bit-identical
 * to A's.
 *   max_d: the widest feature width the alias will be used with (sizes the partial rows of FusedMM beyond 256
 *     columns; wider calls still work, one 256-column group per launch).
 *   workspace: device memory, 256-byte aligned, isp_csr_alias_workspace bytes, borrowed until the alias is
 *     destroyed; it needs no clearing.  Size: 1 KiB per hub-row segment or row piece (isp_csr_info: n_segments,
 *     spmm_pieces) of A and as much again for its cached transpose, plus one byte per stored entry when the
 *     transpose exists - about 2 GiB for 124 M entries in 2.4 M rows.
 *   The alias takes over A's cached transpose as it is at this call: build it on A first if the alias is to
 *     run backward calls (isp_csr_transpose_cached on the alias returns it, or ISP_EINVAL if A had none).
 *   Destroy the alias (isp_csr_destroy) before A.  After isp_csr_values_changed(A) every alias made before is
 *     refused with ISP_EINVAL: make a new one (host work only, nothing is copied or launched).
 * Errors: ISP_EINVAL (NULL or unaligned arguments, workspace too small, A is a transpose or an alias).
 */
isp_status isp_csr_alias_workspace(const isp_csr_t* A, int32_t max_d, size_t* bytes);
isp_status isp_csr_alias(const isp_csr_t* A, int32_t max_d, void* workspace, size_t workspace_bytes,
                         isp_csr_t** out);

/*
 * SpMM, sum reduction: Y[i, 0:d] = sum over stored entries p of row i of values[p] * X[indices[p], 0:d]
 * (abstract; Sections 1, 3.4).  X has A.n_cols rows, Y has A.n_rows rows.  Backward dX = A^T dY is the
 * same call on the handle from isp_csr_transpose_cached (Section 3.3).  X and Y must not overlap.
 */
isp_status isp_spmm(const isp_csr_t* A, const float* X, int64_t ldx, int32_t d, float* Y, int64_t ldy,
                    void* stream);

/*
 * isp_spmm for callers that cannot allocate device memory or hand over scratch: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * results; the difference is where the partial sums of the hub-row segments live.  isp_spmm keeps them in the
 * workspace given to isp_csr_build; this call keeps them in a fixed 32 MiB array inside the library's device
 * image (one per GPU, present from the library's first use on that GPU until the process ends) and makes no
 * allocation of any kind.  Limits and rules:
 *   - a handle that needs more than 32,768 partial rows - one per hub-row segment, or one per row piece where
 *     the handle has the packed SpMM layout (isp_csr_info: n_segments, spmm_pieces) - is rejected with
 *     ISP_EUNSUPPORTED and nothing is launched;
 *   - the array is shared by every handle and every call on that GPU: calls of this function that overlap
 *     on one GPU (different streams or threads) race, whichever handles they use; calls on one stream are safe;
 *   - nothing in the array needs clearing between calls (each launch writes every partial row it later reads).
 */
isp_status isp_spmm_static_scratch(const isp_csr_t* A, const float* X, int64_t ldx, int32_t d, float* Y,
                                   int64_t ldy, void* stream);

/*
 * SDDMM (Section 1): out[p] = <U[i, 0:d], V[indices[p], 0:d]> for every stored entry p of every
 * row i, in A's CSR order; with ISP_SCALE_BY_A multiplied by values[p].  U has n_rows rows, V has
 * n_cols rows, out has nnz elements.  With U = dY and V = X this is dA of Y = A X.
 */
isp_status isp_sddmm(const isp_csr_t* A, const float* U, int64_t ldu, const float* V, int64_t ldv,
                     int32_t d, unsigned flags, float* out, void* stream);

/*
 * FusedMM forward (Section 1(a): SDDMM, an edge function and SpMM as one operation), A square:
 *   s_p = f(<X[i], X[j]>), j = indices[p];  Y[i] = sum_p values[p] * s_p * X[j],
 * f chosen by op (ISP_OP_SIGMOID, ISP_OP_DOT, ISP_OP_ONE).  The per-edge scores are never written to
 * memory.  d <= 1024; beyond 256 columns d must be a multiple of 4 and the rows 16-byte aligned (base pointers
 * and leading dimensions), else ISP_EUNSUPPORTED.  Up to 256 columns run on the tuned kernels; wider rows on a
 * slower general path (whole rows per lane group; the rows long enough to be split keep one partial row per 256
 * columns, normally all in one launch, in several when the scratch is too small for that).
 */
isp_status isp_fusedmm(const isp_csr_t* A, const float* X, int64_t ldx, int32_t d, int op, float* Y,
                       int64_t ldy, void* stream);

/*
 * FusedMM backward: dX for upstream gradient dY of the forward above.  With g = dY and
 * dz_p = values[p] <g_i, x_j> f'(z_p)   (s_p (1 - s_p) for the sigmoid):
 *   dX[i] = sum_{p in row i} dz_p x_j  +  sum_{p: indices[p] = i} (values[p] s_p g_r + dz_p x_r),
 * r = row of p.  The second sum runs over row i of the cached transpose, so
 * isp_csr_transpose_cached(A) must have succeeded before; otherwise ISP_EINVAL.  When the transpose's offsets
 * and indices turn out equal to A's own (a symmetric pattern with ascending rows; the values may differ) both
 * sums run over the same neighbours and the tuned kernels take them in one pass over A, gathering x_j and g_j
 * once for both (two gathered rows per entry instead of three).
 */
isp_status isp_fusedmm_backward(isp_csr_t* A, const float* X, int64_t ldx, const float* dY, int64_t lddy,
                                int32_t d, int op, float* dX, int64_t lddx, void* stream);

/* reduce of isp_spmm_reduce / isp_spmm_reduce_backward */
#define ISP_REDUCE_SUM 0
#define ISP_REDUCE_MEAN 1
#define ISP_REDUCE_MIN 2
#define ISP_REDUCE_MAX 3

/*
 * SpMM with the other reductions of the paper's matmul (Sections 3.4, 3.5: 'sum', 'mean', 'min', 'max').
 *   sum : same as isp_spmm.
 *   mean: Y[i] = (sum_p values[p] X[indices[p]]) / (stored entries of row i); empty row -> 0.
 *   min / max: Y[i,k] = min / max over the stored entries p of row i of values[p] * X[indices[p], k], product
 *         and comparison in fp32; arg[i,k] = position p (index into indices / values) of the first entry that
 *         attains it; empty row -> Y = 0, arg = -1.  arg is int32, n_rows x d, row-major, dense (leading
 *         dimension d), required for min / max, ignored otherwise.
 * sum has the tuned kernels; mean reuses them, and min / max have a kernel of the same design, when width and
 * alignment allow (d and the leading dimensions multiples of 4, 16-byte aligned pointers); other shapes run
 * on the generic path.
 */
isp_status isp_spmm_reduce(const isp_csr_t* A, const float* X, int64_t ldx, int32_t d, int reduce, float* Y,
                           int64_t ldy, int32_t* arg, void* stream);

/*
 * Backward of isp_spmm_reduce with respect to X, through the cached transpose (Section 3.3), which must
 * have been built (isp_csr_transpose_cached) - otherwise ISP_EINVAL.  dX is n_cols x d and is overwritten.
 *   sum : dX = A^T dY.   mean: dX[j] = sum_{p in column j} (values[p] / len(row(p))) dY[row(p)]; the first
 *         mean call on a handle (and the first after isp_csr_values_changed) computes values[p] / len(row(p))
 *         for every entry, on `stream`, into a part of the transpose workspace that the transposition itself
 *         no longer needs; later calls read it.  (A first call made while `stream` is being captured into a
 *         HIP graph records that pass in the graph and leaves the cache unmarked, so every replay - and the
 *         next call outside the capture - computes it again; the same holds for the min / max bookkeeping.)
 *   min / max: dX[j,k] = sum over entries p in column j with arg[row(p),k] == p of values[p] dY[row(p),k];
 *         arg is the array the forward call filled; positions outside [0, nnz) name no entry.  Each call
 *         first marks the entries arg names (one byte per entry, in spare transpose workspace) and passes
 *         over the others.
 */
isp_status isp_spmm_reduce_backward(isp_csr_t* A, const float* dY, int64_t lddy, int32_t d, int reduce,
                                    const int32_t* arg, float* dX, int64_t lddx, void* stream);

/* Free the host-side handle and its cached transpose handle.  Never touches caller buffers.  NULL ok. */
void isp_csr_destroy(isp_csr_t* A);

/* Message of the calling thread's most recent failure ("" if none).  Static storage. */
const char* isp_last_error(void);

/* Library version string, e.g. "isp-gfx950 0.1". */
const char* isp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ISP_H */
