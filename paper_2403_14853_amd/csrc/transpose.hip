// Stable CSR transpose, built once per graph and cached in the source handle (paper Section 3.3:
// cache-enabled backpropagation; the cached expression is read as A^T in CSR form).
//
// "Stable" = entries of one column keep their order of appearance in A, which makes the result
// unique and lets it be compared bit for bit.  It is computed as a least-significant-digit radix
// sort of the column indices (digits of up to 8 bits) that carries source position, source row and value as
// payload; every pass is a stable counting sort: per-tile digit histograms -> exclusive scan over
// (digit, tile) -> scatter with ranks taken in source order.  Integer work only, no atomics on
// anything order-dependent.
#include "isp_internal.h"

namespace {

constexpr int RS_THREADS = 256;
constexpr int RS_WAVES = RS_THREADS / ISP_WAVE;
constexpr int RS_ROUNDS = 16;                       // keys per lane
constexpr int RS_WAVE_KEYS = RS_ROUNDS * ISP_WAVE;  // contiguous keys owned by one wave
constexpr int RS_TILE = RS_WAVE_KEYS * RS_WAVES;    // keys per workgroup
constexpr int RS_RADIX = 256;

// Row that owns the first entry of every sort tile: the smallest r with indptr[r + 1] > tile * RS_TILE.
__global__ void __launch_bounds__(256) k_tile_rows(const int64_t* __restrict__ indptr, int64_t n_rows, int n_tiles,
                                                   int32_t* __restrict__ tile_row) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_tiles) return;
  const int64_t q = (int64_t)t * RS_TILE;
  int64_t lo = 0, hi = n_rows - 1;  // q < nnz = indptr[n_rows], so the answer exists
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (indptr[mid + 1] > q) hi = mid; else lo = mid + 1;
  }
  tile_row[t] = (int32_t)lo;
}

// Per-tile digit histogram; table is digit-major: table[digit * n_tiles + tile].
__global__ void __launch_bounds__(RS_THREADS) k_radix_hist(const int32_t* __restrict__ keys, int64_t n, int shift,
                                                           int mask, int n_tiles, int32_t* __restrict__ table) {
  __shared__ int hist[RS_RADIX];
  hist[threadIdx.x] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * RS_TILE;
  for (int i = threadIdx.x; i < RS_TILE; i += RS_THREADS) {
    const int64_t q = base + i;
    if (q < n) atomicAdd(&hist[(keys[q] >> shift) & mask], 1);
  }
  __syncthreads();
  table[(int64_t)threadIdx.x * n_tiles + blockIdx.x] = hist[threadIdx.x];
}

// Stable scatter of one pass; the records travel as four parallel arrays (column key, source position,
// source row, value), so the last pass leaves perm, the source rows and the values of A^T where they
// belong and nothing has to be gathered afterwards.
// Wave w of a workgroup owns the contiguous keys [tile + w * RS_WAVE_KEYS, +RS_WAVE_KEYS) and walks them
// 64 at a time in source order, so a key's rank among equal digits = (equal digits in earlier tiles:
// scanned table) + (in earlier waves of the tile) + (earlier rounds of this wave) + (lower lanes of this
// round).  The tile is first put in digit order in LDS and written out from there, which turns the
// scattered 4-byte stores into contiguous runs per digit.
// FIRST: the input is the CSR itself: keys = indices, source position = index, value = values (val_in), and
// the source rows are rebuilt per tile from the row offsets: every row that starts inside the tile marks its
// first position in LDS, a running maximum spreads the marks (tile_row = the row owning the tile's first entry).
template <bool FIRST, bool HAS_VAL>
__global__ void __launch_bounds__(RS_THREADS) k_radix_scatter(
    const int32_t* __restrict__ keys_in, const int32_t* __restrict__ src_in, const int32_t* __restrict__ row_in,
    const int32_t* __restrict__ val_in, const int64_t* __restrict__ indptr, int64_t n_rows,
    const int32_t* __restrict__ tile_row, int64_t n, int shift, int mask, int n_tiles,
    const int32_t* __restrict__ table_scanned, int32_t* __restrict__ keys_out, int32_t* __restrict__ src_out,
    int32_t* __restrict__ row_out, int32_t* __restrict__ val_out) {
  __shared__ volatile int wave_cnt[RS_WAVES][RS_RADIX];
  __shared__ int wave_base[RS_WAVES][RS_RADIX];  // tile-local sorted position of each wave's first key of a digit
  __shared__ int delta[RS_RADIX];                // output position minus tile-local position, per digit
  __shared__ int wave_tot[RS_WAVES];
  __shared__ int buf[RS_TILE];
  const int lane = threadIdx.x & (ISP_WAVE - 1), w = threadIdx.x / ISP_WAVE;
  for (int i = threadIdx.x; i < RS_WAVES * RS_RADIX; i += RS_THREADS) (&wave_cnt[0][0])[i] = 0;
  const int64_t tile_base = (int64_t)blockIdx.x * RS_TILE;
  const int tile_count = (int)((n - tile_base < RS_TILE) ? n - tile_base : RS_TILE);
  if (FIRST) {
    for (int i = threadIdx.x; i < RS_TILE; i += RS_THREADS) buf[i] = 0;
    __syncthreads();
    const int r_first = tile_row[blockIdx.x];
    if (threadIdx.x == 0) buf[0] = r_first;
    // rows after r_first that start inside the tile (of several empty rows sharing a start, the last one -
    // the owner of the entry there - wins)
    for (int64_t r = (int64_t)r_first + 1 + threadIdx.x; r < n_rows; r += RS_THREADS) {
      const int64_t o = indptr[r] - tile_base;
      if (o >= tile_count) break;
      atomicMax(&buf[o], (int)r);
    }
    __syncthreads();
    // running maximum over the tile: thread t owns positions [16 t, 16 t + 16)
    int loc[RS_ROUNDS], run = 0;
#pragma unroll
    for (int k = 0; k < RS_ROUNDS; ++k) {
      const int v = buf[threadIdx.x * RS_ROUNDS + k];
      run = v > run ? v : run;
      loc[k] = run;
    }
    int inc = run;
#pragma unroll
    for (int o = 1; o < ISP_WAVE; o <<= 1) {
      const int t = __shfl_up(inc, o);
      if (lane >= o && t > inc) inc = t;
    }
    if (lane == ISP_WAVE - 1) wave_tot[w] = inc;
    __syncthreads();
    int before = __shfl_up(inc, 1);  // maximum over the lower lanes of this wave
    if (lane == 0) before = 0;
    for (int ww = 0; ww < w; ++ww) before = wave_tot[ww] > before ? wave_tot[ww] : before;
#pragma unroll
    for (int k = 0; k < RS_ROUNDS; ++k) buf[threadIdx.x * RS_ROUNDS + k] = loc[k] > before ? loc[k] : before;
  }
  __syncthreads();
  const int64_t wbase = tile_base + (int64_t)w * RS_WAVE_KEYS;
  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  int key[RS_ROUNDS], src[RS_ROUNDS], row[RS_ROUNDS], val[RS_ROUNDS], pos[RS_ROUNDS];
#pragma unroll
  for (int r = 0; r < RS_ROUNDS; ++r) {
    const int64_t q = wbase + r * ISP_WAVE + lane;
    const bool valid = q < n;
    key[r] = valid ? keys_in[q] : 0;
    if (FIRST) {
      src[r] = (int32_t)q;
      row[r] = valid ? buf[w * RS_WAVE_KEYS + r * ISP_WAVE + lane] : 0;
      val[r] = (HAS_VAL && valid) ? val_in[q] : 0;
    } else {
      src[r] = valid ? src_in[q] : 0;
      row[r] = valid ? row_in[q] : 0;
      val[r] = (HAS_VAL && valid) ? val_in[q] : 0;
    }
  }
#pragma unroll
  for (int r = 0; r < RS_ROUNDS; ++r) {
    const bool valid = wbase + r * ISP_WAVE + lane < n;
    const int dg = (key[r] >> shift) & mask;
    unsigned long long m = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const unsigned long long bal = __ballot((dg >> b) & 1);
      m &= ((dg >> b) & 1) ? bal : ~bal;
    }
    // m = valid lanes of this round holding the same digit as this lane
    const int before = valid ? wave_cnt[w][dg] : 0;
    pos[r] = before + __popcll(m & lt_mask);
    if (valid && (m & lt_mask) == 0) wave_cnt[w][dg] = before + __popcll(m);  // lowest lane of the group
  }
  __syncthreads();
  {  // thread t owns digit t: exclusive scan of the tile's digit counts -> where each digit starts in the tile
    const int dg = threadIdx.x;
    int cnt[RS_WAVES], tot = 0;
#pragma unroll
    for (int ww = 0; ww < RS_WAVES; ++ww) { cnt[ww] = wave_cnt[ww][dg]; tot += cnt[ww]; }
    int inc = tot;
#pragma unroll
    for (int o = 1; o < ISP_WAVE; o <<= 1) {
      const int t = __shfl_up(inc, o);
      if (lane >= o) inc += t;
    }
    if (lane == ISP_WAVE - 1) wave_tot[w] = inc;
    __syncthreads();
    int start = inc - tot;
    for (int ww = 0; ww < w; ++ww) start += wave_tot[ww];
    delta[dg] = table_scanned[(int64_t)dg * n_tiles + blockIdx.x] - start;
    int run = start;
#pragma unroll
    for (int ww = 0; ww < RS_WAVES; ++ww) { wave_base[ww][dg] = run; run += cnt[ww]; }
  }
  __syncthreads();
  // keys: into digit order in LDS, then out; remember both positions for the other arrays
#pragma unroll
  for (int r = 0; r < RS_ROUNDS; ++r) {
    const bool valid = wbase + r * ISP_WAVE + lane < n;
    const int dg = (key[r] >> shift) & mask;
    pos[r] = valid ? wave_base[w][dg] + pos[r] : -1;
    if (valid) buf[pos[r]] = key[r];
  }
  __syncthreads();
  int dst[RS_ROUNDS];
#pragma unroll
  for (int k = 0; k < RS_ROUNDS; ++k) {
    const int i = k * RS_THREADS + threadIdx.x;
    dst[k] = -1;
    if (i < tile_count) {
      const int kk = buf[i];
      dst[k] = delta[(kk >> shift) & mask] + i;
      keys_out[dst[k]] = kk;
    }
  }
  auto move = [&](const int (&v)[RS_ROUNDS], int32_t* __restrict__ out) {
    __syncthreads();  // everyone has read the previous array out of buf
#pragma unroll
    for (int r = 0; r < RS_ROUNDS; ++r)
      if (pos[r] >= 0) buf[pos[r]] = v[r];
    __syncthreads();
#pragma unroll
    for (int k = 0; k < RS_ROUNDS; ++k)
      if (dst[k] >= 0) out[dst[k]] = buf[k * RS_THREADS + threadIdx.x];
  };
  move(src, src_out);
  move(row, row_out);
  if (HAS_VAL) move(val, val_out);
}

// Row offsets of A^T from the sorted column keys: an offset changes where the sorted column changes;
// empty columns get the next offset.
__global__ void __launch_bounds__(256) k_col_offsets(const int32_t* __restrict__ skey, int64_t nnz, int64_t n_cols,
                                                     int64_t* __restrict__ t_indptr) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= nnz) return;
  const int32_t c = skey[q];
  const int32_t prev = q > 0 ? skey[q - 1] : -1;
  // (the clamp only matters for an unvalidated CSR with a column >= n_cols)
  const int64_t c_hi = c < n_cols ? (int64_t)c : n_cols - 1;
  for (int64_t cc = (int64_t)prev + 1; cc <= c_hi; ++cc) t_indptr[cc] = q;
  if (q == nnz - 1)
    for (int64_t cc = (int64_t)c + 1; cc <= n_cols; ++cc) t_indptr[cc] = nnz;
}

// t_values[q] = values[perm[q]]
__global__ void __launch_bounds__(256) k_gather_values(const int32_t* __restrict__ perm, const float* __restrict__ values,
                                                       int64_t nnz, float* __restrict__ t_values) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q < nnz) t_values[q] = values[perm[q]];
}

// mean_values[q] = t_values[q] / len_A(t_indices[q])  (t_values absent: 1 / len), as one fp32 product with
// the reciprocal lengths the build keeps
__global__ void __launch_bounds__(256) k_mean_values(const int32_t* __restrict__ t_indices,
                                                     const float* __restrict__ t_values,
                                                     const float* __restrict__ inv_len, int64_t nnz,
                                                     float* __restrict__ mean_values) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q < nnz) mean_values[q] = (t_values ? t_values[q] : 1.f) * inv_len[t_indices[q]];
}

__global__ void __launch_bounds__(256) k_inverse_perm(const int32_t* __restrict__ perm, int64_t nnz,
                                                      int32_t* __restrict__ inv_perm) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q < nnz) inv_perm[perm[q]] = (int32_t)q;
}

// *differs becomes 1 when A^T's offsets and indices are not, element for element, A's own: otherwise the pattern
// is symmetric with every row's columns ascending, and entry p of A^T is the mirror (j, i) of entry p = (i, j)
// of A.  (*differs is zeroed before.)
__global__ void __launch_bounds__(256) k_compare_pattern(const int64_t* __restrict__ indptr, const int64_t* __restrict__ t_indptr,
                                                         int64_t n, const int32_t* __restrict__ indices,
                                                         const int32_t* __restrict__ t_indices, int64_t nnz,
                                                         int* __restrict__ differs) {
  bool bad = false;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nnz + n + 1; i += (int64_t)gridDim.x * blockDim.x) {
    if (i < nnz) bad |= indices[i] != t_indices[i];
    else bad |= indptr[i - nnz] != t_indptr[i - nnz];
  }
  if (__any(bad) && (threadIdx.x & (ISP_WAVE - 1)) == 0) *differs = 1;  // (plain store of the same value from any wave)
}

__global__ void k_zero_int(int* p) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0;
}

__global__ void __launch_bounds__(256) k_fill_i64(int64_t* __restrict__ a, int64_t n, int64_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) a[i] = v;
}

struct t_layout {
  size_t t_indptr, t_indices, perm, t_values, set[2][4], tile_row, table, table_scanned, scan_tmp, part, total;
  int64_t n_tiles;
};

t_layout make_layout(int64_t n_rows, int64_t n_cols, int64_t nnz, bool has_values) {
  t_layout L;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += isp_align(bytes); return o; };
  L.n_tiles = (nnz + RS_TILE - 1) / RS_TILE;
  const size_t e = (size_t)(nnz + 1) * 4;
  L.t_indptr = take((size_t)(n_cols + 1) * 8);
  L.t_indices = take(e);
  L.perm = take(e);
  L.t_values = take(has_values ? e : 0);
  // two sets of record arrays (key, source position, source row, value) that the passes alternate between
  for (int k = 0; k < 2; ++k)
    for (int a = 0; a < 4; ++a) L.set[k][a] = take(a == 3 && !has_values ? 0 : e);
  L.tile_row = take((size_t)(L.n_tiles + 1) * 4);
  const int64_t tbl = (int64_t)RS_RADIX * L.n_tiles;
  L.table = take((size_t)(tbl + 1) * 4);
  L.table_scanned = take((size_t)(tbl + 1) * 4);
  L.scan_tmp = take(isp_scan_tmp_bytes(tbl + 1));
  L.part = take(isp_partition_workspace(n_cols, n_rows, nnz));  // (A^T: n_cols rows, n_rows columns)
  L.total = off;
  return L;
}

}  // namespace

size_t isp_transpose_workspace_bytes(int64_t n_rows, int64_t n_cols, int64_t nnz, bool has_values) {
  return make_layout(n_rows, n_cols, nnz, has_values).total;
}

isp_status isp_transpose_build(isp_csr* A, void* ws, size_t ws_bytes, hipStream_t s) {
  const isp_view& v = A->v;
  const int64_t nnz = v.nnz, n_cols = v.n_cols, n_rows = v.n_rows;
  const bool has_values = v.values != nullptr;
  const t_layout L = make_layout(n_rows, n_cols, nnz, has_values);
  if (!ws) return isp_fail(ISP_EINVAL, "transpose workspace is NULL");
  if (ws_bytes < L.total) return isp_fail(ISP_EINVAL, "transpose workspace too small: %zu < %zu bytes", ws_bytes, L.total);
  if (((uintptr_t)ws & 255) != 0) return isp_fail(ISP_EINVAL, "workspace must be 256-byte aligned");
  char* base = (char*)ws;
  int64_t* t_indptr = (int64_t*)(base + L.t_indptr);
  int32_t* t_indices = (int32_t*)(base + L.t_indices);
  int32_t* perm = (int32_t*)(base + L.perm);
  float* t_values = has_values ? (float*)(base + L.t_values) : nullptr;
  int32_t* tile_row = (int32_t*)(base + L.tile_row);
  int32_t* table = (int32_t*)(base + L.table);
  int32_t* table_scanned = (int32_t*)(base + L.table_scanned);
  void* scan_tmp = base + L.scan_tmp;

  if (nnz == 0) {
    k_fill_i64<<<(unsigned)((n_cols + 1 + 255) / 256), 256, 0, s>>>(t_indptr, n_cols + 1, 0);
    ISP_LAUNCH_CHECK();
  } else {
    int bits = 1;
    while (bits < 31 && ((int64_t)1 << bits) < n_cols) ++bits;
    const int n_pass = (bits + 7) / 8;  // digits of at most 8 bits (5-, 6- and 7-bit digits measured slower)
    const int n_tiles = (int)L.n_tiles;
    k_tile_rows<<<(n_tiles + 255) / 256, 256, 0, s>>>(v.indptr, n_rows, n_tiles, tile_row);
    ISP_LAUNCH_CHECK();
    const int32_t* in[4] = {v.indices, nullptr, nullptr, (const int32_t*)v.values};
    for (int pass = 0; pass < n_pass; ++pass) {
      // digits of about equal width: pass p takes bits [p * bits / n_pass, (p + 1) * bits / n_pass)
      const int shift = pass * bits / n_pass;
      const int mask = (1 << ((pass + 1) * bits / n_pass - shift)) - 1;
      k_radix_hist<<<n_tiles, RS_THREADS, 0, s>>>(in[0], nnz, shift, mask, n_tiles, table);
      ISP_LAUNCH_CHECK();
      isp_status st = isp_scan_i32_to_i32(table, table_scanned, (int64_t)RS_RADIX * n_tiles, scan_tmp, s);
      if (st != ISP_OK) return st;
      int32_t* out[4];
      for (int a = 0; a < 4; ++a) out[a] = (int32_t*)(base + L.set[pass & 1][a]);
      if (pass == n_pass - 1) {  // the last pass writes A^T's arrays; its keys still go to the set (for the offsets)
        out[1] = perm;
        out[2] = t_indices;
        out[3] = (int32_t*)t_values;
      }
#define ISP_GO(F, HV)                                                                                             \
  k_radix_scatter<F, HV><<<n_tiles, RS_THREADS, 0, s>>>(in[0], in[1], in[2], in[3], v.indptr, n_rows, tile_row, nnz, shift, mask, \
                                                        n_tiles, table_scanned, out[0], out[1], out[2], out[3])
      if (pass == 0) { if (has_values) ISP_GO(true, true); else ISP_GO(true, false); }
      else { if (has_values) ISP_GO(false, true); else ISP_GO(false, false); }
#undef ISP_GO
      ISP_LAUNCH_CHECK();
      for (int a = 0; a < 4; ++a) in[a] = out[a];
    }
    k_col_offsets<<<(unsigned)((nnz + 255) / 256), 256, 0, s>>>(in[0], nnz, n_cols, t_indptr);
    ISP_LAUNCH_CHECK();
  }
  // Is the pattern symmetric (A^T's structure identical to A's)?  The flag lives in the sort's histogram table,
  // which is free by now, and is read back with the counters of the partition build below.
  int* differs = (int*)table;
  const bool square = n_rows == n_cols && nnz > 0;
  if (square) {
    k_zero_int<<<1, 64, 0, s>>>(differs);
    ISP_LAUNCH_CHECK();
    k_compare_pattern<<<2048, 256, 0, s>>>(v.indptr, t_indptr, n_rows, v.indices, t_indices, nnz, differs);
    ISP_LAUNCH_CHECK();
  }
  isp_csr* At = nullptr;
  isp_status st = isp_build_handle(n_cols, n_rows, nnz, t_indptr, t_indices, t_values, base + L.part,
                                   ws_bytes - L.part, false, s, &At);
  if (st != ISP_OK) return st;
  int h_differs = 1;
  if (square) {
    ISP_HIP(hipMemcpyAsync(&h_differs, differs, sizeof(int), hipMemcpyDeviceToHost, s));
    ISP_HIP(hipStreamSynchronize(s));
  }
  A->mirror_aligned = At->mirror_aligned = (h_differs == 0);
  A->info.symmetric_pattern = At->info.symmetric_pattern = A->mirror_aligned ? 1 : 0;
  At->tune = A->tune;  // (resolved when A was built)
  At->perm = perm;
  At->t_values_rw = t_values;
  // the record arrays of the sort are free from here on; one of them later holds the mean reduction's values
  At->mean_values = (float*)(base + L.set[0][1]);
  At->mean_values_packed = At->has_packed ? (float*)(base + L.set[1][2]) : nullptr;
  At->mean_values_valid = false;
  At->mean_values_used = false;
  At->sel_flags = (uint8_t*)(base + L.set[1][1]);
  At->inv_perm = (int32_t*)(base + L.set[0][2]);
  At->inv_perm_valid = false;
  At->is_transpose = true;
  At->info.is_transpose = 1;
  A->At = At;
  A->info.has_cached_transpose = 1;
  return ISP_OK;
}

namespace {
// While s is being captured into a HIP graph the kernels enqueued here run only when the graph is replayed:
// the fill is then part of every replay and the cache is not marked filled.
bool stream_is_capturing(hipStream_t s) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return st == hipStreamCaptureStatusActive;
}

}  // namespace

// (and, where A^T has the packed SpMM layout, the same values in the order of that layout's entries)
static isp_status fill_mean_values(isp_csr* A, hipStream_t s) {
  isp_csr* At = A->At;
  const unsigned grid = (unsigned)((A->v.nnz + 255) / 256);
  k_mean_values<<<grid, 256, 0, s>>>(At->v.indices, At->v.values, A->v.inv_len, A->v.nnz, At->mean_values);
  ISP_LAUNCH_CHECK();
  if (At->mean_values_packed) {
    k_gather_values<<<grid, 256, 0, s>>>(At->packed_src_pos, At->mean_values, A->v.nnz, At->mean_values_packed);
    ISP_LAUNCH_CHECK();
  }
  return ISP_OK;
}

isp_status isp_transpose_mean_values(isp_csr* A, hipStream_t s, const float** out, const float** out_packed) {
  isp_csr* At = A->At;
  if (!At || !At->mean_values) return isp_fail(ISP_EINVAL, "no cached transpose");
  if (!At->mean_values_valid && A->v.nnz > 0) {
    isp_status st = fill_mean_values(A, s);
    if (st != ISP_OK) return st;
    At->mean_values_valid = !stream_is_capturing(s);
  }
  At->mean_values_used = true;
  *out = At->mean_values;
  *out_packed = At->mean_values_packed;
  return ISP_OK;
}

isp_status isp_transpose_inverse_perm(isp_csr* A, hipStream_t s, const int32_t** out) {
  isp_csr* At = A->At;
  if (!At || !At->inv_perm) return isp_fail(ISP_EINVAL, "no cached transpose");
  if (!At->inv_perm_valid && A->v.nnz > 0) {
    k_inverse_perm<<<(unsigned)((A->v.nnz + 255) / 256), 256, 0, s>>>(At->perm, A->v.nnz, At->inv_perm);
    ISP_LAUNCH_CHECK();
    At->inv_perm_valid = !stream_is_capturing(s);
  }
  *out = At->inv_perm;
  return ISP_OK;
}

// Everything derived from A's values is brought up to date on s itself, in stream order: a call recorded into a
// HIP graph refreshes on every replay, and a graph that was captured while the mean reduction's values were
// valid (and therefore holds no pass that computes them) reads refreshed ones after an eager call.
isp_status isp_transpose_refresh_values(isp_csr* A, hipStream_t s) {
  isp_csr* At = A->At;
  if (!At || !A->v.values || !At->t_values_rw || A->v.nnz == 0) return ISP_OK;
  const unsigned grid = (unsigned)((A->v.nnz + 255) / 256);
  k_gather_values<<<grid, 256, 0, s>>>(At->perm, A->v.values, A->v.nnz, At->t_values_rw);
  ISP_LAUNCH_CHECK();
  if (At->mean_values_used) {  // a mean backward has run (or was captured): its values follow at once
    isp_status st = fill_mean_values(A, s);
    if (st != ISP_OK) return st;
    // (valid stays as it is: during a capture the refill runs with the replays, like the fill itself)
  }
  return ISP_OK;
}
