// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "isp.h"

#define ISP_WAVE 64
#define ISP_WG 256                 // threads per workgroup in the row-streaming kernels
#define ISP_WAVES_PER_WG (ISP_WG / ISP_WAVE)
#define ISP_PARTIAL_TILE 256       // floats per hub-segment partial row (one column tile)

// Device-side view of a CSR with its work partition.  Passed to kernels by value.
struct isp_view {
  int64_t n_rows, n_cols, nnz;
  const int64_t* indptr;
  const int32_t* indices;
  const float* values;     // may be NULL
  // work items: [0, n_blocks) are row blocks [blk_row[b], blk_row[b+1]) made of whole short rows;
  // [n_blocks, n_blocks + n_seg) are segments of hub rows.  Segments are numbered row by row in order of
  // position (that number also names the segment's partial row); they are scheduled in seg_order.
  const int32_t* blk_row;  // n_blocks + 1
  int32_t n_blocks;
  const int32_t* hub_rows; // n_hub row ids, ascending
  const int32_t* hub_seg_ptr;  // n_hub + 1: first segment of each hub row
  const int32_t* seg_hub;  // n_seg: index into hub_rows of each segment
  const int32_t* seg_begin;  // n_seg: position of each segment's first nonzero; a segment ends where the
                             // row's next one begins, the row's last one at the end of the row
  const int32_t* seg_order;  // n_seg: work item n_blocks + k processes segment seg_order[k] (in order of first column)
  const int4* item_desc;     // n_blocks + n_seg: what each work item covers, resolved at build time so that a
                             // wavefront starts with one 16-byte load instead of a chain through the tables
                             // above: (first entry, end, first row | segment, end row or -1 = skip | hub row)
  int32_t n_hub, n_seg;
  int32_t hub_t, seg_len;
  float* partials;         // n_seg * ISP_PARTIAL_TILE floats
  const float* inv_len;    // 1 / (stored entries of the row), 0 for an empty row; indexed by the rows of the
                           // handle's matrix (also in the view of a derived matrix)
  // Views of a derived matrix (packed SpMM layout) only: rows [n_real_rows, n_rows) are pieces of the handle's
  // long rows; piece k = row n_real_rows + k adds into partial row piece_slot[k], and hub_rows / hub_seg_ptr /
  // n_hub list the cut rows with their partial rows for the fix-up.  Ordinary views: n_real_rows = n_rows.
  int64_t n_real_rows;
  const int32_t* piece_slot;
};

// Tuning and debugging overrides.  They come from the environment and are resolved ONCE, when a handle is
// built (the cached transpose inherits its source's): the compute entry points read the handle, never the
// environment.  include/isp.h lists the variables.
struct isp_tuning {
  bool no_grouped;      // ISP_NO_GROUPED: every op runs on the generic kernels
  bool sddmm_one_pass;  // ISP_SDDMM_ONE_PASS: SDDMM never splits 128-column rows into two 64-column passes
  int spmm_lpg;         // ISP_SPMM_LPG: lanes per group of the grouped SpMM (0 = chosen by shape)
  int spmm_tile;        // ISP_SPMM_TILE: feature columns per launch of the grouped SpMM (0 = chosen by shape)
  bool no_mirror;       // ISP_NO_MIRROR: the FusedMM backward never takes the one-pass form of symmetric patterns
  int fused_w;          // ISP_FUSED_W: 4 / 8 = the grouped SDDMM / FusedMM kernels give a lane one / two float4 at every width above 32 (0 = chosen by width and graph)
  int wide_groups;      // ISP_WIDE_GROUPS: most column groups a hub segment stores per launch of a wide FusedMM pass (0 = as many as fit)
};
isp_tuning isp_read_tuning();
// Wavefront slots of the current device at the occupancy the row-streaming kernels run at (compute units x 4
// SIMDs x 4 waves); the device is asked once per process and device.
int isp_wave_slots();

struct isp_csr {
  isp_view v;
  // Packed SpMM layout (csr_build.hip): a derived matrix whose rows are the short rows of v's matrix followed by
  // column-band pieces of its long rows, in its own copy of the index / value arrays (in the build workspace).
  // Only the tuned SpMM reads it.  Without it vp == v.
  isp_view vp;
  int64_t partial_rows;           // partial rows (ISP_PARTIAL_TILE floats each) v.partials has room for
  bool has_packed;
  int packed_block_cost, packed_row_cost;  // of vp's partition (bounds of its blocks: see csr_build.hip)
  float* packed_values_rw;        // vp.values, writable, NULL without values
  const int32_t* packed_src_pos;  // position in v's arrays of every entry of the derived matrix
  isp_tuning tune;
  const int32_t* perm;     // transposes only
  float* t_values_rw;      // transposes only: the values array (in the workspace), writable
  float* mean_values;      // transposes only: nnz floats of workspace the transposition no longer needs, for
                           // value / (length of the entry's source row), filled on first use
  float* mean_values_packed;  // the same values in the order of the packed SpMM layout's entries (NULL without it)
  bool mean_values_valid;  // false until filled
  bool mean_values_used;   // a mean backward has run on this handle: isp_csr_values_changed refills the array
  uint8_t* sel_flags;      // transposes only: nnz bytes of the same spare workspace; the min / max backward
                           // marks there which entries its arg array names
  int32_t* inv_perm;       // transposes only, same spare workspace: inv_perm[perm[q]] = q, filled on first use
  bool inv_perm_valid;
  isp_csr_info_t info;
  int device;
  isp_csr* At;             // cached transpose (owned), or NULL
  bool is_transpose;
  // Alias handles (alias.hip): a copy of another handle ("the source") with scratch of its own.  source is
  // NULL for a built handle and for its cached transpose.  values_gen counts isp_csr_values_changed calls on
  // a built handle; an alias remembers in source_gen the count it was made at and is refused once they differ.
  const isp_csr* source;
  uint64_t values_gen, source_gen;
  bool mirror_aligned;     // set with the cached transpose: A^T's offsets and indices equal A's own element for
                           // element (a symmetric pattern, rows ascending), so entry p of A^T is the mirror of
                           // entry p of A and one pass over A can serve both
};

// ---- error plumbing --------------------------------------------------------------------------
isp_status isp_fail(isp_status st, const char* fmt, ...);
#define ISP_HIP(call)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return isp_fail(ISP_EHIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)
#define ISP_LAUNCH_CHECK() ISP_HIP(hipGetLastError())

static inline size_t isp_align(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- argument checks shared by the entry points (isp_api.hip) -----------------------------------
// The handle's device must be the current one, and an alias must be as recent as its source's values.
isp_status isp_check_device(const isp_csr* A);
isp_status isp_check_dense(const void* p, int64_t ld, int32_t d, int64_t rows, const char* name);

// ---- device scans (scan.hip) -----------------------------------------------------------------
// Exclusive prefix sums; out has n + 1 entries (out[n] = total).  tmp must hold
// isp_scan_tmp_bytes(n) bytes.  in and out may not alias.
size_t isp_scan_tmp_bytes(int64_t n);
isp_status isp_scan_i32_to_i64(const int32_t* in, int64_t* out, int64_t n, void* tmp, hipStream_t s);
isp_status isp_scan_i32_to_i32(const int32_t* in, int32_t* out, int64_t n, void* tmp, hipStream_t s);

// ---- partition (csr_build.hip) ---------------------------------------------------------------
size_t isp_partition_workspace(int64_t n_rows, int64_t n_cols, int64_t nnz);
isp_status isp_build_handle(int64_t n_rows, int64_t n_cols, int64_t nnz, const int64_t* indptr,
                            const int32_t* indices, const float* values, void* ws, size_t ws_bytes,
                            bool validate, hipStream_t s, isp_csr** out);
// Copy A's (rewritten) values into the packed SpMM layout's own value array again.
isp_status isp_refresh_packed_values(isp_csr* A, hipStream_t s);

// ---- transpose (transpose.hip) ---------------------------------------------------------------
size_t isp_transpose_workspace_bytes(int64_t n_rows, int64_t n_cols, int64_t nnz, bool has_values);
isp_status isp_transpose_build(isp_csr* A, void* ws, size_t ws_bytes, hipStream_t s);
// Gather the cached transpose's values again from A's (rewritten) values.
isp_status isp_transpose_refresh_values(isp_csr* A, hipStream_t s);
// Values of A's cached transpose divided by the lengths of their source rows of A (what the backward of the
// mean reduction multiplies dY's rows by): computed on s at the first call and after the values changed,
// kept in the transpose workspace afterwards.
isp_status isp_transpose_mean_values(isp_csr* A, hipStream_t s, const float** out, const float** out_packed);
// Position q in A's cached transpose of every stored entry p of A (the inverse of perm): computed on s at the
// first call, kept in the transpose workspace afterwards.
isp_status isp_transpose_inverse_perm(isp_csr* A, hipStream_t s, const int32_t** out);

// ---- compute (spmm.hip, sddmm.hip, fusedmm.hip) ------------------------------------------------
isp_status isp_spmm_launch(const isp_csr* A, const float* X, int64_t ldx, int32_t d, float* Y, int64_t ldy,
                           hipStream_t s);
// Grouped fast path of SpMM; *done = false (nothing launched) when the operands do not qualify.
// mean_mode 0: plain sum; 1: rows divided by their length.  values_override (optional): nnz values used in
// place of A's own, in the order of A's entries; values_override_packed: the same values in the order of the
// packed layout's entries, without which an override keeps the launch on A's ordinary partition.
isp_status isp_spmm_grouped_launch(const isp_csr* A, const float* X, int64_t ldx, int32_t d, float* Y, int64_t ldy,
                                   int mean_mode, const float* values_override, hipStream_t s, bool* done,
                                   const float* values_override_packed = nullptr);
isp_status isp_sddmm_launch(const isp_csr* A, const float* U, int64_t ldu, const float* V, int64_t ldv,
                            int32_t d, bool scale, float* out, hipStream_t s);
isp_status isp_fusedmm_launch(const isp_csr* A, const float* X, int64_t ldx, int32_t d, int op, float* Y,
                              int64_t ldy, hipStream_t s);
isp_status isp_fusedmm_bwd_launch(const isp_csr* A, const float* X, int64_t ldx, const float* G, int64_t ldg,
                                  int32_t d, int op, float* dX, int64_t lddx, hipStream_t s);
isp_status isp_spmm_reduce_launch(const isp_csr* A, const float* X, int64_t ldx, int32_t d, int reduce, float* Y,
                                  int64_t ldy, int32_t* arg, hipStream_t s);
isp_status isp_spmm_reduce_bwd_launch(isp_csr* A, const float* dY, int64_t lddy, int32_t d, int reduce,
                                      const int32_t* arg, float* dX, int64_t lddx, hipStream_t s);
