// CSR ingest: structural validation, degree classes and the wavefront work partition.
//
// Rows are classed by degree (0 | 1..4 | 5..32 | 33..hub_t | hub).  Short rows are grouped
// into contiguous row blocks of about block_cost units, one unit per nonzero plus one per row
// (a row's output write costs about as much as one gathered input row).  Hub rows
// (degree > hub_t) never share a block; each is cut into segments of at most seg_len nonzeros whose
// partial sums are combined later in a fixed order.  A hub row is cut first where its (sorted) columns
// cross the boundaries of column bands, so that a segment gathers dense rows from one band only, and the
// segments are scheduled in order of their first column: the whole chip then works on one band of the
// dense operand at a time and the L2 caches hold that band's frequently used rows instead of a sample
// of all of them.
// Everything here is integer work and runs once per graph (balanced scheduling: paper Section 1(b); CSR
// operand: Section 3.5).
#include <stdlib.h>
#include <new>
#include "isp_internal.h"

namespace {

struct build_counters {
  unsigned long long bin_rows[5];
  unsigned long long bin_nnz[5];
  unsigned long long max_degree;
  int err;            // bit 0: indptr malformed, bit 1: column index out of range
  int n_blocks, n_hub, n_seg;
};

struct partition_params {
  int block_cost, hub_t, seg_len;
  int row_cost;   // cost units of a row besides its entries (1; 2 in the derived matrix, which allows larger blocks)
  int bands;      // column bands of the finest cut (a power of two); 1 = no band cuts
  int min_piece;  // a hub row is cut into at most degree / min_piece bands
};

constexpr int MAX_BANDS = 64;  // one piece per lane

int env_int(const char* name, int dflt, int lo, int hi) {
  const char* s = getenv(name);
  if (!s || !*s) return dflt;
  long v = strtol(s, nullptr, 10);
  if (v < lo) v = lo;
  if (v > hi) v = hi;
  return (int)v;
}

partition_params get_params(int64_t n_rows, int64_t n_cols, int64_t nnz) {
  partition_params p;
  p.row_cost = 1;
  const int64_t slots = isp_wave_slots();  // 4,096 on an MI355X (256 compute units)
  // Upper limits = what the grouped kernels' per-wave LDS tables hold (block_cost + hub_t <= 768
  // entries, block_cost <= 256 rows, seg_len <= 768 entries).  The environment overrides exist for
  // tuning and for tests that want many small work items.
  // Small matrices get smaller row blocks, about as many as the chip has wavefront slots (compute units x 16):
  // a wavefront's work is a chain of dependent memory round trips, and a short chain on every slot
  // finishes sooner than a long one on a few (4,096 rows x 9 entries: 16 -> 7 us per SpMM).
  int64_t auto_cost = (nnz + n_rows + slots - 1) / slots;
  auto_cost = auto_cost < 16 ? 16 : (auto_cost > 256 ? 256 : auto_cost);
  p.block_cost = env_int("ISP_BLOCK_COST", (int)auto_cost, 16, 256);
  // ... and shorter hub segments, for the same reason and because the segments are the heavy items that the
  // launch hands out last: a quarter of the per-slot share, between 80 and 512 entries, rows of more than two
  // segments' worth being hubs (2.4 M entries: segments of 157 instead of 512, 0.512 -> 0.468 ms for four
  // SpMMs; 0.6 M entries: 0.167 -> 0.155 ms; from 8 M entries up the sizes are 512 / 512 as before).
  // With many columns a column band of the dense operand is far larger than an L2, and finer pieces of the
  // hub rows (segments of at most 384, pieces from 192 entries) keep more of each segment's gathers inside its
  // band (2.4 M columns: 5.30 -> 5.19 ms per SpMM, the other kernels 1-3 %); with few columns a band's popular
  // rows fit an L2 anyway and the longer segments win (233 k columns: SDDMM 3.21 vs 3.32 ms).
  // Measured again with the present kernels (segments 256 .. 512, smallest pieces 64 .. 256, on the three large
  // benchmark graphs): segments of at most 320 and pieces from 128 entries are best or within 1 % of it for every
  // kernel on every one of them (233 k columns: SpMM 2.68 -> 2.59 ms, SDDMM 2.71 -> 2.60 ms; 2.4 M columns:
  // FusedMM 5.59 -> 5.41 ms; 1 M columns: FusedMM backward 1.36 -> 1.32 ms).
  const int seg_cap = 320;
  int64_t auto_seg = (nnz + n_rows + slots - 1) / slots / 4;
  auto_seg = auto_seg < 80 ? 80 : (auto_seg > seg_cap ? seg_cap : auto_seg);
  const int auto_hub = 2 * auto_seg > 512 ? 512 : (int)(2 * auto_seg);
  p.hub_t = env_int("ISP_HUB_THRESHOLD", auto_hub, 8, 512);
  p.seg_len = env_int("ISP_SEGMENT_LEN", (int)auto_seg, 8, 768);
  int b = env_int("ISP_BANDS", 32, 1, MAX_BANDS);
  while (b & (b - 1)) b &= b - 1;  // round down to a power of two
  p.bands = b;
  // (the lower limit bounds the number of segments, hence the partial-sum rows the workspace must hold)
  const int mp_lo = p.seg_len / 8 > 4 ? p.seg_len / 8 : 4;
  int mp = p.seg_len / 2 < 128 ? p.seg_len / 2 : 128;
  if (mp < mp_lo) mp = mp_lo;
  p.min_piece = env_int("ISP_MIN_PIECE", mp, mp_lo, 1 << 20);
  return p;
}

}  // namespace

isp_tuning isp_read_tuning() {
  isp_tuning t;
  t.no_grouped = getenv("ISP_NO_GROUPED") != nullptr;
  t.sddmm_one_pass = getenv("ISP_SDDMM_ONE_PASS") != nullptr;
  const int lpg = env_int("ISP_SPMM_LPG", 0, 0, 64);
  t.spmm_lpg = (lpg == 4 || lpg == 8 || lpg == 16 || lpg == 32 || lpg == 64) ? lpg : 0;
  const int tile = env_int("ISP_SPMM_TILE", 0, 0, 256);
  t.spmm_tile = (tile == 64 || tile == 128 || tile == 256) ? tile : 0;
  t.wide_groups = env_int("ISP_WIDE_GROUPS", 0, 0, 4);
  t.no_mirror = getenv("ISP_NO_MIRROR") != nullptr;
  const int fw = env_int("ISP_FUSED_W", 0, 0, 8);
  t.fused_w = (fw == 4 || fw == 8) ? fw : 0;
  return t;
}

int isp_wave_slots() {
  constexpr int MAX_DEV = 64;
  static int cached[MAX_DEV] = {};  // 0 = not asked yet (racing first calls store the same number)
  constexpr int fallback = 256 * 16;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return fallback; }
  if (dev >= 0 && dev < MAX_DEV && cached[dev]) return cached[dev];
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
    (void)hipGetLastError();
    return fallback;
  }
  const int slots = cus * 16;  // 4 SIMDs per compute unit x the 4 waves per SIMD the kernels are built for
  if (dev >= 0 && dev < MAX_DEV) cached[dev] = slots;
  return slots;
}

namespace {

__global__ void k_zero_counters(build_counters* c) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *c = build_counters{};
}

// Pieces of a hub row: its entries [a, b) cut where the columns cross band boundaries.  A row of degree
// deg is cut into br = the largest power of two <= min(bands, deg / min_piece) coarse bands, each made of
// bands / br fine bands of width ceil(n_cols / bands).  The whole wavefront calls this with the same row
// (a, b wave-uniform): lane j < br gets piece j as [*first, *last), the other lanes an empty piece.  Every
// lane finds one cut position by binary search, which assumes ascending columns; on a row that is not
// sorted the positions are made monotone, so they are still valid cuts (inside the row, in order) and only
// the scheduling benefit is lost, never correctness.
__device__ inline void wave_hub_pieces(const int32_t* __restrict__ indices, int64_t a, int64_t b, int64_t n_cols,
                                       const partition_params& pp, int lane, int64_t* first, int64_t* last) {
  const int64_t deg = b - a;
  int br = 1;
  while (br * 2 <= pp.bands && (int64_t)(br * 2) * pp.min_piece <= deg) br *= 2;
  const int64_t bw = (n_cols + pp.bands - 1) / pp.bands;
  const int step = pp.bands / br;
  // cut j = first position whose column is >= j * step * bw; cut 0 = a, cuts >= br = b
  int64_t lo = a, hi = b;
  if (lane == 0) hi = a;
  if (lane >= br) lo = b;
  const int64_t target = (int64_t)lane * step * bw;
  while (__any(lo < hi)) {
    if (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if ((int64_t)indices[mid] < target) lo = mid + 1; else hi = mid;
    }
  }
  int64_t cut = lo;
#pragma unroll
  for (int o = 1; o < ISP_WAVE; o <<= 1) {  // running maximum over the lanes: monotone cuts
    const int64_t t = __shfl_up(cut, o);
    if (lane >= o && t > cut) cut = t;
  }
  int64_t next = __shfl_down(cut, 1);
  if (lane == ISP_WAVE - 1) next = b;  // (the last lane has no neighbour; it holds a piece only with 64 bands)
  *first = lane < br ? cut : b;
  *last = lane < br ? next : b;
}

__device__ inline int degree_bin(long long deg, int hub_t) {
  if (deg <= 0) return 0;
  if (deg > hub_t) return 4;
  if (deg <= 4) return 1;
  if (deg <= 32) return 2;
  return 3;
}

// Per row: degree, class, cost, segment count; indptr checks.  Grid-stride; the class histogram,
// maximum degree and segment total are reduced per workgroup before a handful of integer atomics.
__global__ void __launch_bounds__(256) k_row_pass(const int64_t* __restrict__ indptr,
                                                  const int32_t* __restrict__ indices, int64_t n_rows, int64_t n_cols,
                                                  int64_t nnz, partition_params pp, int32_t* __restrict__ cost,
                                                  int32_t* __restrict__ hubflag, int32_t* __restrict__ nseg,
                                                  float* __restrict__ inv_len, build_counters* __restrict__ ctr) {
  __shared__ unsigned long long s_rows[5], s_nnz[5], s_max;
  __shared__ int s_err, s_seg;
  if (threadIdx.x < 5) { s_rows[threadIdx.x] = 0; s_nnz[threadIdx.x] = 0; }
  if (threadIdx.x == 0) { s_max = 0; s_err = 0; s_seg = 0; }
  __syncthreads();
  unsigned long long my_rows[5] = {0, 0, 0, 0, 0}, my_nnz[5] = {0, 0, 0, 0, 0}, my_max = 0;
  int my_err = 0, my_seg = 0;
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  // every wavefront walks whole chunks of 64 rows (one per lane), so that it can turn to a hub row together
  for (int64_t base = (int64_t)blockIdx.x * blockDim.x + (threadIdx.x - lane); base < n_rows;
       base += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i = base + lane;
    const bool valid = i < n_rows;
    const int64_t a = valid ? indptr[i] : 0, b = valid ? indptr[i + 1] : 0;
    long long deg = b - a;
    if (valid && (deg < 0 || a < 0 || b > nnz || (i == 0 && a != 0) || (i == n_rows - 1 && b != nnz))) { my_err = 1; deg = 0; }
    const bool hub = deg > pp.hub_t;
    int ns = 0;
    for (unsigned long long hm = __ballot(hub); hm; hm &= hm - 1) {  // the chunk's hub rows, one at a time
      const int src = __ffsll((long long)hm) - 1;
      const int64_t ha = __shfl(a, src), hb = __shfl(b, src);
      int64_t first, last;
      wave_hub_pieces(indices, ha, hb, n_cols, pp, lane, &first, &last);
      int cnt = (int)((last - first + pp.seg_len - 1) / pp.seg_len);
#pragma unroll
      for (int o = 1; o < ISP_WAVE; o <<= 1) cnt += __shfl_xor(cnt, o);
      if (lane == src) ns = cnt;
    }
    if (!valid) continue;
    cost[i] = hub ? 0 : (int32_t)deg + pp.row_cost;
    hubflag[i] = hub ? 1 : 0;
    nseg[i] = ns;
    inv_len[i] = deg > 0 ? 1.f / (float)deg : 0.f;
    const int bin = degree_bin(deg, pp.hub_t);
#pragma unroll
    for (int k = 0; k < 5; ++k) {
      my_rows[k] += (bin == k);
      my_nnz[k] += (bin == k) ? (unsigned long long)deg : 0ull;
    }
    my_max = (unsigned long long)deg > my_max ? (unsigned long long)deg : my_max;
    my_seg += ns;
  }
#pragma unroll
  for (int k = 0; k < 5; ++k) {
    if (my_rows[k]) atomicAdd(&s_rows[k], my_rows[k]);
    if (my_nnz[k]) atomicAdd(&s_nnz[k], my_nnz[k]);
  }
  if (my_max) atomicMax(&s_max, my_max);
  if (my_err) atomicOr(&s_err, 1);
  if (my_seg) atomicAdd(&s_seg, my_seg);
  __syncthreads();
  if (threadIdx.x < 5) {
    if (s_rows[threadIdx.x]) atomicAdd(&ctr->bin_rows[threadIdx.x], s_rows[threadIdx.x]);
    if (s_nnz[threadIdx.x]) atomicAdd(&ctr->bin_nnz[threadIdx.x], s_nnz[threadIdx.x]);
  }
  if (threadIdx.x == 0) {
    if (s_max) atomicMax(&ctr->max_degree, s_max);
    if (s_err) atomicOr(&ctr->err, 1);
    if (s_seg) atomicAdd(&ctr->n_seg, s_seg);
  }
}

// Column indices must lie in [0, n_cols).
__global__ void __launch_bounds__(256) k_check_indices(const int32_t* __restrict__ indices, int64_t nnz, int64_t n_cols,
                                                       build_counters* __restrict__ ctr) {
  bool bad = false;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * blockDim.x) {
    const int32_t c = indices[p];
    bad |= (c < 0 || c >= n_cols);
  }
  if (__any(bad) && (threadIdx.x & (ISP_WAVE - 1)) == 0) atomicOr(&ctr->err, 2);
}

// Block boundaries forced by hub rows: a hub row starts a block and so does the row after it.
// force_row (if inside the matrix) also starts a block: the derived matrix of the packed SpMM layout keeps
// blocks of whole rows and blocks of row pieces apart that way.
__global__ void __launch_bounds__(256) k_mark_rows(const int32_t* __restrict__ hubflag, int64_t n_rows,
                                                   int64_t force_row, int32_t* __restrict__ mark) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_rows) return;
  mark[i] = (i == 0 || i == force_row || hubflag[i] || hubflag[i - 1]) ? 1 : 0;
}

// Balanced boundaries: block b starts at the first row whose cumulative short-row cost reaches b * block_cost.
__global__ void __launch_bounds__(256) k_mark_balanced(const int64_t* __restrict__ cum_cost, int64_t n_rows,
                                                       int64_t n_bal, int block_cost, int32_t* __restrict__ mark) {
  const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= n_bal) return;
  const int64_t target = b * (int64_t)block_cost;
  int64_t lo = 0, hi = n_rows;  // first i in [0, n_rows] with cum_cost[i] >= target
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (cum_cost[mid] >= target) hi = mid; else lo = mid + 1;
  }
  if (lo < n_rows) mark[lo] = 1;
}

__global__ void __launch_bounds__(256) k_compact(const int64_t* __restrict__ indptr, const int32_t* __restrict__ indices,
                                                 int64_t n_cols, partition_params pp,
                                                 const int32_t* __restrict__ mark, const int32_t* __restrict__ mpos,
                                                 const int32_t* __restrict__ hubflag, const int32_t* __restrict__ hpos,
                                                 const int32_t* __restrict__ segbase,
                                                 int64_t n_rows, int32_t* __restrict__ blk_row,
                                                 int32_t* __restrict__ hub_rows, int32_t* __restrict__ hub_seg_ptr,
                                                 int32_t* __restrict__ seg_hub, int32_t* __restrict__ seg_begin,
                                                 int32_t* __restrict__ seg_key, build_counters* __restrict__ ctr,
                                                 int64_t max_blocks, int64_t max_hub, int64_t max_seg) {
  // The bounds only bite for a malformed indptr (the host then reports ISP_EBADCSR); they keep
  // every write inside the workspace in that case too.
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  if (i == 0) {
    const int nb = mpos[n_rows], nh = hpos[n_rows];
    if (nb <= max_blocks) blk_row[nb] = (int32_t)n_rows;
    if (nh <= max_hub) hub_seg_ptr[nh] = segbase[n_rows];
    ctr->n_blocks = nb;
    ctr->n_hub = nh;
  }
  const bool valid = i < n_rows;  // (no early exit: the wavefront handles its hub rows together)
  if (valid && mark[i] && mpos[i] < max_blocks) blk_row[mpos[i]] = (int32_t)i;
  const bool hub = valid && hubflag[i];
  const int h = hub ? hpos[i] : 0, s0 = hub ? segbase[i] : 0;
  const int64_t a = hub ? indptr[i] : 0, b = hub ? indptr[i + 1] : 0;
  if (hub && h < max_hub) {
    hub_rows[h] = (int32_t)i;
    hub_seg_ptr[h] = s0;
  }
  for (unsigned long long hm = __ballot(hub); hm; hm &= hm - 1) {
    const int src = __ffsll((long long)hm) - 1;
    const int64_t ha = __shfl(a, src), hb = __shfl(b, src);
    const int hh = __shfl(h, src), hs0 = __shfl(s0, src);
    int64_t first, last;
    wave_hub_pieces(indices, ha, hb, n_cols, pp, lane, &first, &last);
    // the row's segments, in order of position: piece by piece (lane by lane), each piece in runs of seg_len
    const int cnt = (int)((last - first + pp.seg_len - 1) / pp.seg_len);
    int inc = cnt;
#pragma unroll
    for (int o = 1; o < ISP_WAVE; o <<= 1) {
      const int t = __shfl_up(inc, o);
      if (lane >= o) inc += t;
    }
    int64_t s = (int64_t)hs0 + inc - cnt;
    for (int64_t q = first; q < last; q += pp.seg_len, ++s) {
      if (s >= max_seg) continue;
      seg_hub[s] = hh;
      seg_begin[s] = (int32_t)q;
      seg_key[s] = indices[q];
    }
  }
}

// ---- schedule order of the segments: stable radix sort (8-bit digits) by first column -----------------
constexpr int SO_TILE = 256;
constexpr int SO_RADIX = 256;

__global__ void __launch_bounds__(SO_TILE) k_seg_hist(const int32_t* __restrict__ key, int n_seg, int shift, int n_tiles,
                                                      int32_t* __restrict__ table) {
  __shared__ int hist[SO_RADIX];
  hist[threadIdx.x] = 0;
  __syncthreads();
  const int s = blockIdx.x * SO_TILE + threadIdx.x;
  if (s < n_seg) atomicAdd(&hist[(key[s] >> shift) & (SO_RADIX - 1)], 1);
  __syncthreads();
  table[threadIdx.x * n_tiles + blockIdx.x] = hist[threadIdx.x];
}

// val_in == NULL: the payload is the element's index (first pass)
__global__ void __launch_bounds__(SO_TILE) k_seg_scatter(const int32_t* __restrict__ key_in,
                                                         const int32_t* __restrict__ val_in, int n_seg, int shift,
                                                         int n_tiles, const int32_t* __restrict__ table_scanned,
                                                         int32_t* __restrict__ key_out, int32_t* __restrict__ val_out) {
  __shared__ int digits[SO_TILE];
  const int s = blockIdx.x * SO_TILE + threadIdx.x;
  const int key = s < n_seg ? key_in[s] : 0;
  const int dg = s < n_seg ? (key >> shift) & (SO_RADIX - 1) : -1;
  digits[threadIdx.x] = dg;
  __syncthreads();
  if (dg < 0) return;
  int rank = 0;  // earlier elements of this tile with the same digit
  for (int t = 0; t < (int)threadIdx.x; ++t) rank += (digits[t] == dg);
  const int dst = table_scanned[dg * n_tiles + blockIdx.x] + rank;
  key_out[dst] = key;
  val_out[dst] = val_in ? val_in[s] : s;
}

// What work item `item` covers, written once per handle (see isp_view::item_desc).
__global__ void __launch_bounds__(256) k_item_desc(const int64_t* __restrict__ indptr, const int32_t* __restrict__ blk_row,
                                                   int n_blocks, const int32_t* __restrict__ hub_rows,
                                                   const int32_t* __restrict__ hub_seg_ptr,
                                                   const int32_t* __restrict__ seg_hub,
                                                   const int32_t* __restrict__ seg_begin,
                                                   const int32_t* __restrict__ seg_order, int n_seg, int hub_t,
                                                   int4* __restrict__ desc) {
  const int item = blockIdx.x * blockDim.x + threadIdx.x;
  if (item >= n_blocks + n_seg) return;
  int4 q;
  if (item < n_blocks) {
    const int row = blk_row[item], row_last = blk_row[item + 1];
    const int64_t p = indptr[row], p_end = indptr[row_last];
    const bool skip = (row_last == row + 1) && (p_end - p > hub_t);
    q = make_int4((int)p, (int)p_end, row, skip ? -1 : row_last);
  } else {
    const int s = seg_order[item - n_blocks];
    const int h = seg_hub[s];
    const int hr = hub_rows[h];
    const int64_t p_end = (s + 1 < hub_seg_ptr[h + 1]) ? (int64_t)seg_begin[s + 1] : indptr[hr + 1];
    q = make_int4(seg_begin[s], (int)p_end, s, hr);
  }
  desc[item] = q;
}

// ---- the derived matrix of the packed SpMM layout ------------------------------------------------------
// Rows longer than mid_t ("cut rows") are cut into column-band pieces exactly like hub rows, but with a lower
// threshold and smaller pieces, and the pieces - far too short to be work items of their own - become the rows
// of a derived CSR that is appended, in schedule order (by first column), to a copy of the short rows:
//   rows [0, n)        : the matrix's own rows, the cut ones left empty
//   rows [n, n + n_pc) : the pieces, piece k being segment seg_order[k] of the cut partition
// The derived matrix has short rows only, so the ordinary row blocks pack several pieces into every
// full-sized work item; a piece's sum goes to the partial row of its segment and the fixed-order fix-up adds a
// cut row's pieces as it does a hub row's segments.

// lengths of the short part's rows (0 for a cut row)
__global__ void __launch_bounds__(256) k_short_len(const int64_t* __restrict__ indptr, const int32_t* __restrict__ hubflag,
                                                   int64_t n_rows, int32_t* __restrict__ len) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_rows) len[i] = hubflag[i] ? 0 : (int32_t)(indptr[i + 1] - indptr[i]);
}

// lengths of the pieces in schedule order
__global__ void __launch_bounds__(256) k_piece_len(const int64_t* __restrict__ indptr, const int32_t* __restrict__ hub_rows,
                                                   const int32_t* __restrict__ hub_seg_ptr,
                                                   const int32_t* __restrict__ seg_hub,
                                                   const int32_t* __restrict__ seg_begin,
                                                   const int32_t* __restrict__ seg_order, int n_seg,
                                                   int32_t* __restrict__ len) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n_seg) return;
  const int s = seg_order[k];
  const int h = seg_hub[s];
  const int64_t end = (s + 1 < hub_seg_ptr[h + 1]) ? (int64_t)seg_begin[s + 1] : indptr[hub_rows[h] + 1];
  len[k] = (int32_t)(end - seg_begin[s]);
}

// row offsets of the derived matrix: the short part's scan, then the pieces' scan behind it
__global__ void __launch_bounds__(256) k_join_offsets(const int64_t* __restrict__ short_scan, int64_t n_rows,
                                                      const int64_t* __restrict__ piece_scan, int64_t n_seg,
                                                      int64_t* __restrict__ indptr2) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_rows) indptr2[i] = short_scan[i];
  else if (i <= n_rows + n_seg) indptr2[i] = short_scan[n_rows] + piece_scan[i - n_rows];
}

// Copy of the short rows' entries.  One thread per stored entry of the source matrix; the workgroup's tile of
// consecutive entries spans a narrow range of rows, found once per tile, in which each thread then searches.
constexpr int CP_TILE = 1024;
__global__ void __launch_bounds__(256) k_copy_short(const int64_t* __restrict__ indptr, const int32_t* __restrict__ indices,
                                                    const float* __restrict__ values,
                                                    const int32_t* __restrict__ hubflag, int64_t n_rows, int64_t nnz,
                                                    const int64_t* __restrict__ indptr2, int32_t* __restrict__ indices2,
                                                    float* __restrict__ values2, int32_t* __restrict__ src_pos) {
  __shared__ int64_t s_lo, s_hi;
  const int64_t p0 = (int64_t)blockIdx.x * CP_TILE;
  if (threadIdx.x < 2) {  // last row starting at or before the tile's first / last entry
    const int64_t target = threadIdx.x == 0 ? p0 : (p0 + CP_TILE - 1 < nnz ? p0 + CP_TILE - 1 : nnz - 1);
    int64_t lo = 0, hi = n_rows;  // invariant: indptr[lo] <= target < indptr[hi]
    while (hi - lo > 1) {
      const int64_t mid = (lo + hi) >> 1;
      if (indptr[mid] <= target) lo = mid; else hi = mid;
    }
    if (threadIdx.x == 0) s_lo = lo; else s_hi = lo;
  }
  __syncthreads();
  for (int64_t p = p0 + threadIdx.x; p < p0 + CP_TILE && p < nnz; p += blockDim.x) {
    int64_t lo = s_lo, hi = s_hi + 1;  // the entry's row: last one with indptr[row] <= p
    while (hi - lo > 1) {
      const int64_t mid = (lo + hi) >> 1;
      if (indptr[mid] <= p) lo = mid; else hi = mid;
    }
    if (hubflag[lo]) continue;  // a cut row: its entries are copied piece by piece
    const int64_t q = indptr2[lo] + (p - indptr[lo]);
    indices2[q] = indices[p];
    if (values2) values2[q] = values[p];
    src_pos[q] = (int32_t)p;
  }
}

// Copy of the pieces' entries: one wavefront per piece, both sides contiguous.
__global__ void __launch_bounds__(256) k_copy_pieces(const int32_t* __restrict__ indices, const float* __restrict__ values,
                                                     const int32_t* __restrict__ seg_begin,
                                                     const int32_t* __restrict__ seg_order, int n_seg, int64_t n_rows,
                                                     const int64_t* __restrict__ indptr2, int32_t* __restrict__ indices2,
                                                     float* __restrict__ values2, int32_t* __restrict__ src_pos) {
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  const int k = blockIdx.x * (blockDim.x / ISP_WAVE) + (threadIdx.x >> 6);
  if (k >= n_seg) return;
  const int64_t src = seg_begin[seg_order[k]];
  const int64_t q0 = indptr2[n_rows + k], q1 = indptr2[n_rows + k + 1];
  for (int64_t q = q0 + lane; q < q1; q += ISP_WAVE) {
    const int64_t p = src + (q - q0);
    indices2[q] = indices[p];
    if (values2) values2[q] = values[p];
    src_pos[q] = (int32_t)p;
  }
}

__global__ void __launch_bounds__(256) k_regather_values(const int32_t* __restrict__ src_pos, const float* __restrict__ values,
                                                         int64_t nnz, float* __restrict__ values2) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q < nnz) values2[q] = values[src_pos[q]];
}

// ---- workspace layout ------------------------------------------------------------------------------------
struct ws_layout {
  size_t counters, cost, hubflag, nseg, cum_cost, mark, mpos, hpos, segbase, scan_tmp;
  size_t blk_row, hub_rows, hub_seg_ptr, seg_hub, seg_begin, seg_key[2], seg_order[2], so_table, so_scanned, so_tmp;
  size_t inv_len, item_desc, partials, total;
  int64_t max_blocks, max_hub, max_seg;
};

// The tables of one partition of a matrix with n_rows rows and nnz entries, laid out from offset `start`.
ws_layout make_layout(int64_t n_rows, int64_t nnz, const partition_params& pp, size_t start = 0,
                      bool with_partials = true) {
  ws_layout L;
  size_t off = start;
  auto take = [&](size_t bytes) { size_t o = off; off += isp_align(bytes); return o; };
  const int64_t n_bal = (nnz + (int64_t)pp.row_cost * n_rows) / pp.block_cost + 2;
  int64_t max_hub = nnz / ((int64_t)pp.hub_t + 1);
  if (max_hub > n_rows) max_hub = n_rows;
  int64_t max_blocks = n_bal + 2 * max_hub + 3;
  if (max_blocks > n_rows + 1) max_blocks = n_rows + 1;
  // a row of degree deg has at most deg / min_piece pieces, and a piece of len entries at most
  // len / seg_len + 1 segments
  const int64_t max_seg = nnz / pp.seg_len + (pp.bands > 1 ? nnz / pp.min_piece : 0) + max_hub + 1;
  L.max_blocks = max_blocks; L.max_hub = max_hub; L.max_seg = max_seg;
  L.counters = take(sizeof(build_counters));
  L.cost = take((size_t)(n_rows + 1) * 4);
  L.hubflag = take((size_t)(n_rows + 1) * 4);
  L.nseg = take((size_t)(n_rows + 1) * 4);
  L.cum_cost = take((size_t)(n_rows + 1) * 8);
  L.mark = take((size_t)(n_rows + 1) * 4);
  L.mpos = take((size_t)(n_rows + 1) * 4);
  L.hpos = take((size_t)(n_rows + 1) * 4);
  L.segbase = take((size_t)(n_rows + 1) * 4);
  L.scan_tmp = take(isp_scan_tmp_bytes(n_rows + 1));
  L.blk_row = take((size_t)(max_blocks + 1) * 4);
  L.hub_rows = take((size_t)(max_hub + 1) * 4);
  L.hub_seg_ptr = take((size_t)(max_hub + 2) * 4);
  L.seg_hub = take((size_t)(max_seg + 1) * 4);
  L.seg_begin = take((size_t)(max_seg + 1) * 4);
  for (int k = 0; k < 2; ++k) {
    L.seg_key[k] = take((size_t)(max_seg + 1) * 4);
    L.seg_order[k] = take((size_t)(max_seg + 1) * 4);
  }
  const int64_t so_tbl = (int64_t)SO_RADIX * ((max_seg + SO_TILE - 1) / SO_TILE + 1);
  L.so_table = take((size_t)(so_tbl + 1) * 4);
  L.so_scanned = take((size_t)(so_tbl + 1) * 4);
  L.so_tmp = take(isp_scan_tmp_bytes(so_tbl + 1));
  L.inv_len = take((size_t)(n_rows + 1) * 4);
  L.item_desc = take((size_t)(max_blocks + max_seg + 2) * 16);
  // (a derived matrix has no hub rows of its own, hence no partial rows)
  L.partials = take(with_partials ? (size_t)(max_seg + 1) * ISP_PARTIAL_TILE * sizeof(float) : 256);
  L.total = off;
  return L;
}

// The packed SpMM layout's share of the workspace, behind the matrix's ordinary partition.
struct packed_layout {
  ws_layout cut;      // the cut partition of the matrix itself (its partial rows are the pieces' partial rows)
  size_t indptr2, indices2, values2, src_pos, len_tmp, scan64, scan_tmp;
  size_t part2_start; // the derived matrix's partition starts here (laid out once its row count is known)
  size_t total;
};

// Block cost of the derived matrix.  Its rows cost two units besides their entries, so a block of B units holds
// at most B / 2 rows and B may reach twice the ordinary 256 within the kernels' 256-row tables; its entries
// (fewer than B plus the longest row) must fit their 768-entry tables.
// One and a half times the ordinary block where the longest row leaves room for it (config 3: 384 units next to
// rows of up to 384 entries; measured 4.75 ms per SpMM against 4.81 at 256 and 4.76 at 512, where the segments
// have to shrink to 256 entries): every work item starts with a chain of dependent loads before its first
// gather, and fewer, larger items pay it less often.
int derived_block_cost(const partition_params& p1, int mid_t) {
  const int longest = mid_t > p1.seg_len ? mid_t : p1.seg_len;
  int dflt = p1.block_cost * 3 / 2;
  if (dflt > 768 - longest) dflt = 768 - longest;
  if (dflt < 16) dflt = 16;
  return env_int("ISP_PACKED_BLOCK", dflt, 16, 512);
}

partition_params cut_params(const partition_params& p1, int mid_t) {
  partition_params c = p1;
  c.hub_t = mid_t;
  const int room = 768 - derived_block_cost(p1, mid_t);  // longest row the derived matrix may have
  // (the ordinary partition's segment length also bounds the pieces here: 320 against 384 measured 4.65 / 4.64 ms
  // per SpMM on 2.4 M columns, 0.345 / 0.357 ms on 1 M columns at d = 64)
  if (c.seg_len > room) c.seg_len = room;
  // pieces of 64 entries or more, on up to 32 bands (measured on 2.4 M columns: smaller pieces fetch less but
  // pay it back in partial rows)
  c.min_piece = env_int("ISP_MIN_PIECE", 64, c.seg_len / 8 > 4 ? c.seg_len / 8 : 4, 1 << 20);
  return c;
}

partition_params derived_params(const partition_params& p1, const partition_params& cut) {
  partition_params d = p1;
  d.hub_t = cut.hub_t > cut.seg_len ? cut.hub_t : cut.seg_len;  // no row of the derived matrix is longer
  d.seg_len = d.hub_t;
  d.bands = 1;
  d.row_cost = 2;
  d.block_cost = derived_block_cost(p1, cut.hub_t);
  return d;
}

packed_layout make_packed_layout(int64_t n_rows, int64_t nnz, bool has_values, const partition_params& p1, int mid_t,
                                 size_t start) {
  packed_layout P;
  const partition_params pc = cut_params(p1, mid_t);
  P.cut = make_layout(n_rows, nnz, pc, start);
  size_t off = P.cut.total;
  auto take = [&](size_t bytes) { size_t o = off; off += isp_align(bytes); return o; };
  const int64_t n2 = n_rows + P.cut.max_seg;
  P.indptr2 = take((size_t)(n2 + 2) * 8);
  P.indices2 = take((size_t)(nnz + 1) * 4);
  P.values2 = has_values ? take((size_t)(nnz + 1) * 4) : 0;
  P.src_pos = take((size_t)(nnz + 1) * 4);
  const int64_t longest = n_rows > P.cut.max_seg ? n_rows : P.cut.max_seg;
  P.len_tmp = take((size_t)(longest + 2) * 4);
  P.scan64 = take((size_t)(n_rows + P.cut.max_seg + 4) * 8);  // the two scans, one behind the other
  P.scan_tmp = take(isp_scan_tmp_bytes(longest + 1));
  P.part2_start = off;
  // upper bound of the derived matrix's partition
  P.total = make_layout(n2, nnz, derived_params(p1, pc), off, false).total;
  return P;
}

// Rows above this length are cut for the packed SpMM layout; 0 = no packed layout.  Chosen for large
// matrices whose dense operand is far larger than an L2 (64 Ki columns or more): there the pieces of
// mid-sized rows (too short to be work items, hence packed) gather from one band at a time like the hub
// segments do.  Measured on 233 k columns / 115 M entries: 2.50 against 2.60 ms per SpMM; on 169 k columns /
// 2.4 M entries it loses (0.125 against 0.113 ms: too few items per band), hence the lower size limit.
// ISP_MID_THRESHOLD overrides (0 disables).
// The layout costs workspace - a second copy of the entries, their source positions and one partial row per
// piece: up to about 36 bytes per stored entry - so beyond 256 Mi entries it is left out as well.
int mid_threshold(int64_t n_rows, int64_t n_cols, int64_t nnz, const partition_params& p1) {
  const int dflt = (nnz >= ((int64_t)8 << 20) && nnz <= ((int64_t)256 << 20) && n_cols >= (1 << 16)) ? 256 : 0;
  int t = env_int("ISP_MID_THRESHOLD", dflt, 0, 512);
  if (t > 0 && t < 8) t = 8;
  // the derived matrix's rows (short rows, pieces) must fit the grouped kernels' tables next to a block
  if (t > 0) {
    const partition_params c = cut_params(p1, t), dd = derived_params(p1, c);
    if (c.seg_len < 8 || dd.block_cost + dd.hub_t > 768 || dd.block_cost / dd.row_cost > 256) t = 0;
  }
  // ... and its rows (the matrix's rows plus one per piece) must stay countable in 32 bits
  if (t > 0 && n_rows + make_layout(n_rows, nnz, cut_params(p1, t)).max_seg >= 2147483646) t = 0;
  return t;
}

// One partition of a CSR matrix: every table the kernels read, in the workspace region laid out by L.
struct partition_out {
  int32_t *blk_row, *hub_rows, *hub_seg_ptr, *seg_hub, *seg_begin, *hubflag;
  const int32_t* seg_order;
  int4* item_desc;
  float* partials;
  float* inv_len;
  build_counters h;
};

isp_status build_partition(int64_t n_rows, int64_t n_cols, int64_t nnz, const int64_t* indptr, const int32_t* indices,
                           const partition_params& pp, char* base, const ws_layout& L, bool validate,
                           int64_t force_row, hipStream_t s, partition_out* out) {
  build_counters* ctr = (build_counters*)(base + L.counters);
  int32_t* cost = (int32_t*)(base + L.cost);
  int32_t* hubflag = (int32_t*)(base + L.hubflag);
  int32_t* nseg = (int32_t*)(base + L.nseg);
  int64_t* cum_cost = (int64_t*)(base + L.cum_cost);
  int32_t* mark = (int32_t*)(base + L.mark);
  int32_t* mpos = (int32_t*)(base + L.mpos);
  int32_t* hpos = (int32_t*)(base + L.hpos);
  int32_t* segbase = (int32_t*)(base + L.segbase);
  void* scan_tmp = base + L.scan_tmp;
  int32_t* blk_row = (int32_t*)(base + L.blk_row);
  int32_t* hub_rows = (int32_t*)(base + L.hub_rows);
  int32_t* hub_seg_ptr = (int32_t*)(base + L.hub_seg_ptr);
  int32_t* seg_hub = (int32_t*)(base + L.seg_hub);
  int32_t* seg_begin = (int32_t*)(base + L.seg_begin);
  int32_t* seg_key[2] = {(int32_t*)(base + L.seg_key[0]), (int32_t*)(base + L.seg_key[1])};
  int32_t* seg_ord[2] = {(int32_t*)(base + L.seg_order[0]), (int32_t*)(base + L.seg_order[1])};
  const int32_t* seg_order = seg_ord[0];

  k_zero_counters<<<1, 64, 0, s>>>(ctr);
  ISP_LAUNCH_CHECK();
  const unsigned row_grid = (unsigned)((n_rows + 255) / 256);
  if (n_rows > 0) {
    k_row_pass<<<row_grid < 2048 ? row_grid : 2048, 256, 0, s>>>(indptr, indices, n_rows, n_cols, nnz, pp, cost,
                                                                 hubflag, nseg, (float*)(base + L.inv_len), ctr);
    ISP_LAUNCH_CHECK();
  }
  if (validate && nnz > 0) {
    k_check_indices<<<2048, 256, 0, s>>>(indices, nnz, n_cols, ctr);
    ISP_LAUNCH_CHECK();
  }
  isp_status st;
  if ((st = isp_scan_i32_to_i64(cost, cum_cost, n_rows, scan_tmp, s)) != ISP_OK) return st;
  if (n_rows > 0) {
    k_mark_rows<<<row_grid, 256, 0, s>>>(hubflag, n_rows, force_row, mark);
    ISP_LAUNCH_CHECK();
    // total short-row cost <= nnz + n_rows, so this many targets cover it
    const int64_t n_bal = (nnz + (int64_t)pp.row_cost * n_rows) / pp.block_cost + 1;
    k_mark_balanced<<<(unsigned)((n_bal + 255) / 256), 256, 0, s>>>(cum_cost, n_rows, n_bal, pp.block_cost, mark);
    ISP_LAUNCH_CHECK();
  }
  if ((st = isp_scan_i32_to_i32(mark, mpos, n_rows, scan_tmp, s)) != ISP_OK) return st;
  if ((st = isp_scan_i32_to_i32(hubflag, hpos, n_rows, scan_tmp, s)) != ISP_OK) return st;
  if ((st = isp_scan_i32_to_i32(nseg, segbase, n_rows, scan_tmp, s)) != ISP_OK) return st;
  k_compact<<<row_grid > 0 ? row_grid : 1, 256, 0, s>>>(indptr, indices, n_cols, pp, mark, mpos, hubflag, hpos, segbase,
                                                       n_rows, blk_row, hub_rows, hub_seg_ptr, seg_hub, seg_begin,
                                                       seg_key[0], ctr, L.max_blocks, L.max_hub, L.max_seg);
  ISP_LAUNCH_CHECK();
  build_counters& h = out->h;
  ISP_HIP(hipMemcpyAsync(&h, ctr, sizeof(h), hipMemcpyDeviceToHost, s));
  ISP_HIP(hipStreamSynchronize(s));
  if (h.err & 1) return isp_fail(ISP_EBADCSR, "indptr is not a monotone offset array from 0 to nnz");
  if (h.err & 2) return isp_fail(ISP_EBADCSR, "a column index lies outside [0, n_cols)");
  if (h.n_blocks > L.max_blocks || h.n_hub > L.max_hub || h.n_seg > L.max_seg)
    return isp_fail(ISP_EINVAL, "internal: partition exceeds its bounds (%d/%lld blocks, %d/%lld hubs, %d/%lld segs)",
                    h.n_blocks, (long long)L.max_blocks, h.n_hub, (long long)L.max_hub, h.n_seg, (long long)L.max_seg);
  if (h.n_seg > 0) {  // schedule order: by first column, equal ones in order of position (stable)
    const int n_tiles = (h.n_seg + SO_TILE - 1) / SO_TILE;
    int32_t* table = (int32_t*)(base + L.so_table);
    int32_t* scanned = (int32_t*)(base + L.so_scanned);
    int bits = 1;  // the keys are columns (< n_cols)
    while (bits < 31 && ((int64_t)1 << bits) < n_cols) ++bits;
    const int n_pass = (bits + 7) / 8;
    for (int pass = 0; pass < n_pass; ++pass) {
      const int32_t* kin = seg_key[pass & 1];
      const int32_t* vin = pass == 0 ? nullptr : seg_ord[pass & 1];
      k_seg_hist<<<n_tiles, SO_TILE, 0, s>>>(kin, h.n_seg, 8 * pass, n_tiles, table);
      ISP_LAUNCH_CHECK();
      if ((st = isp_scan_i32_to_i32(table, scanned, (int64_t)SO_RADIX * n_tiles, base + L.so_tmp, s)) != ISP_OK) return st;
      k_seg_scatter<<<n_tiles, SO_TILE, 0, s>>>(kin, vin, h.n_seg, 8 * pass, n_tiles, scanned, seg_key[(pass + 1) & 1],
                                                seg_ord[(pass + 1) & 1]);
      ISP_LAUNCH_CHECK();
    }
    seg_order = seg_ord[n_pass & 1];
  }

  int4* item_desc = (int4*)(base + L.item_desc);
  if (h.n_blocks + h.n_seg > 0) {
    k_item_desc<<<(unsigned)((h.n_blocks + h.n_seg + 255) / 256), 256, 0, s>>>(indptr, blk_row, h.n_blocks, hub_rows,
                                                                             hub_seg_ptr, seg_hub, seg_begin, seg_order,
                                                                             h.n_seg, pp.hub_t, item_desc);
    ISP_LAUNCH_CHECK();
  }
  out->blk_row = blk_row; out->hub_rows = hub_rows; out->hub_seg_ptr = hub_seg_ptr; out->seg_hub = seg_hub;
  out->seg_begin = seg_begin; out->hubflag = hubflag; out->seg_order = seg_order; out->item_desc = item_desc;
  out->partials = (float*)(base + L.partials);
  out->inv_len = (float*)(base + L.inv_len);
  return ISP_OK;
}

void fill_view(isp_view& v, int64_t n_rows, int64_t n_cols, int64_t nnz, const int64_t* indptr, const int32_t* indices,
               const float* values, const partition_out& po, const partition_params& pp) {
  v.n_rows = n_rows; v.n_cols = n_cols; v.nnz = nnz;
  v.indptr = indptr; v.indices = indices; v.values = values;
  v.blk_row = po.blk_row; v.n_blocks = po.h.n_blocks;
  v.hub_rows = po.hub_rows; v.hub_seg_ptr = po.hub_seg_ptr; v.seg_hub = po.seg_hub;
  v.seg_begin = po.seg_begin; v.seg_order = po.seg_order; v.item_desc = po.item_desc;
  v.n_hub = po.h.n_hub; v.n_seg = po.h.n_seg;
  v.hub_t = pp.hub_t; v.seg_len = pp.seg_len;
  v.partials = po.partials;
  v.inv_len = po.inv_len;
  v.n_real_rows = n_rows;
  v.piece_slot = nullptr;
}

// The packed SpMM layout of the handle's matrix (see above), into A->vp.  A->v must be filled.
isp_status build_packed(isp_csr* A, const partition_params& p1, int mid_t, char* base, const packed_layout& P,
                        size_t ws_bytes, hipStream_t s) {
  const isp_view& v = A->v;
  const int64_t n = v.n_rows, nnz = v.nnz;
  const partition_params pc = cut_params(p1, mid_t);
  partition_out cut;
  isp_status st = build_partition(n, v.n_cols, nnz, v.indptr, v.indices, pc, base, P.cut, false, -1, s, &cut);
  if (st != ISP_OK) return st;
  const int n_pc = cut.h.n_seg;
  if (cut.h.n_hub == 0) return ISP_OK;  // nothing to cut: the ordinary partition serves
  int64_t* indptr2 = (int64_t*)(base + P.indptr2);
  int32_t* indices2 = (int32_t*)(base + P.indices2);
  float* values2 = v.values ? (float*)(base + P.values2) : nullptr;
  int32_t* src_pos = (int32_t*)(base + P.src_pos);
  int32_t* len_tmp = (int32_t*)(base + P.len_tmp);
  int64_t* short_scan = (int64_t*)(base + P.scan64);
  int64_t* piece_scan = short_scan + (n + 2);
  void* scan_tmp = base + P.scan_tmp;
  k_short_len<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(v.indptr, cut.hubflag, n, len_tmp);
  ISP_LAUNCH_CHECK();
  if ((st = isp_scan_i32_to_i64(len_tmp, short_scan, n, scan_tmp, s)) != ISP_OK) return st;
  k_piece_len<<<(unsigned)((n_pc + 255) / 256), 256, 0, s>>>(v.indptr, cut.hub_rows, cut.hub_seg_ptr, cut.seg_hub,
                                                           cut.seg_begin, cut.seg_order, n_pc, len_tmp);
  ISP_LAUNCH_CHECK();
  if ((st = isp_scan_i32_to_i64(len_tmp, piece_scan, n_pc, scan_tmp, s)) != ISP_OK) return st;
  const int64_t n2 = n + n_pc;
  k_join_offsets<<<(unsigned)((n2 + 1 + 255) / 256), 256, 0, s>>>(short_scan, n, piece_scan, n_pc, indptr2);
  ISP_LAUNCH_CHECK();
  k_copy_short<<<(unsigned)((nnz + CP_TILE - 1) / CP_TILE), 256, 0, s>>>(v.indptr, v.indices, v.values, cut.hubflag, n, nnz,
                                                                       indptr2, indices2, values2, src_pos);
  ISP_LAUNCH_CHECK();
  k_copy_pieces<<<(unsigned)((n_pc + 3) / 4), 256, 0, s>>>(v.indices, v.values, cut.seg_begin, cut.seg_order, n_pc, n,
                                                         indptr2, indices2, values2, src_pos);
  ISP_LAUNCH_CHECK();
  // the derived matrix's own partition: row blocks only, none straddling the first piece row
  const partition_params pd = derived_params(p1, pc);
  const ws_layout L2 = make_layout(n2, nnz, pd, P.part2_start, false);
  if (L2.total > ws_bytes) return isp_fail(ISP_EINVAL, "internal: packed layout exceeds the workspace (%zu > %zu)", L2.total, ws_bytes);
  partition_out d2;
  if ((st = build_partition(n2, v.n_cols, nnz, indptr2, indices2, pd, base, L2, false, n, s, &d2)) != ISP_OK) return st;
  if (d2.h.n_hub != 0 || d2.h.n_seg != 0)
    return isp_fail(ISP_EINVAL, "internal: the derived matrix has %d rows above its hub threshold", d2.h.n_hub);
  isp_view& vp = A->vp;
  fill_view(vp, n2, v.n_cols, nnz, indptr2, indices2, values2, d2, pd);
  // the pieces' sums go to the cut partition's partial rows and are added by its hub tables
  vp.hub_rows = cut.hub_rows; vp.hub_seg_ptr = cut.hub_seg_ptr; vp.n_hub = cut.h.n_hub;
  vp.partials = cut.partials;
  vp.inv_len = v.inv_len;
  vp.n_real_rows = n;
  vp.piece_slot = cut.seg_order;
  A->has_packed = true;
  A->packed_block_cost = pd.block_cost;
  A->packed_row_cost = pd.row_cost;
  A->packed_values_rw = values2;
  A->packed_src_pos = src_pos;
  A->info.spmm_mid_threshold = mid_t;
  A->info.spmm_cut_rows = cut.h.n_hub;
  A->info.spmm_pieces = n_pc;
  A->info.spmm_row_blocks = d2.h.n_blocks;
  return ISP_OK;
}

}  // namespace

size_t isp_partition_workspace(int64_t n_rows, int64_t n_cols, int64_t nnz) {
  const partition_params p1 = get_params(n_rows, n_cols, nnz);
  const ws_layout L = make_layout(n_rows, nnz, p1);
  const int mid_t = mid_threshold(n_rows, n_cols, nnz, p1);
  if (mid_t == 0) return L.total;
  return make_packed_layout(n_rows, nnz, true, p1, mid_t, L.total).total;
}

isp_status isp_refresh_packed_values(isp_csr* A, hipStream_t s) {
  if (!A->has_packed || !A->packed_values_rw || !A->v.values || A->v.nnz == 0) return ISP_OK;
  k_regather_values<<<(unsigned)((A->v.nnz + 255) / 256), 256, 0, s>>>(A->packed_src_pos, A->v.values, A->v.nnz,
                                                                      A->packed_values_rw);
  ISP_LAUNCH_CHECK();
  return ISP_OK;
}

isp_status isp_build_handle(int64_t n_rows, int64_t n_cols, int64_t nnz, const int64_t* indptr,
                            const int32_t* indices, const float* values, void* ws, size_t ws_bytes, bool validate,
                            hipStream_t s, isp_csr** out) {
  const partition_params pp = get_params(n_rows, n_cols, nnz);
  const ws_layout L = make_layout(n_rows, nnz, pp);
  const int mid_t = mid_threshold(n_rows, n_cols, nnz, pp);
  packed_layout P{};
  size_t need = L.total;
  if (mid_t > 0) {
    P = make_packed_layout(n_rows, nnz, values != nullptr, pp, mid_t, L.total);
    need = P.total;
  }
  if (ws_bytes < need) return isp_fail(ISP_EINVAL, "workspace too small: %zu < %zu bytes", ws_bytes, need);
  if (((uintptr_t)ws & 255) != 0) return isp_fail(ISP_EINVAL, "workspace must be 256-byte aligned");
  char* base = (char*)ws;
  partition_out po;
  isp_status st = build_partition(n_rows, n_cols, nnz, indptr, indices, pp, base, L, validate, -1, s, &po);
  if (st != ISP_OK) return st;

  int device = 0;
  ISP_HIP(hipGetDevice(&device));
  isp_csr* A = new (std::nothrow) isp_csr();
  if (!A) return isp_fail(ISP_ENOMEM, "host allocation of the handle failed");
  A->device = device;
  A->tune = isp_read_tuning();
  fill_view(A->v, n_rows, n_cols, nnz, indptr, indices, values, po, pp);
  A->vp = A->v;
  A->partial_rows = L.max_seg + 1;
  A->has_packed = false; A->packed_values_rw = nullptr; A->packed_src_pos = nullptr;
  A->perm = nullptr; A->t_values_rw = nullptr; A->At = nullptr; A->is_transpose = false; A->mirror_aligned = false;
  A->mean_values = nullptr; A->mean_values_packed = nullptr; A->mean_values_valid = false; A->mean_values_used = false;
  A->sel_flags = nullptr; A->inv_perm = nullptr; A->inv_perm_valid = false;
  A->source = nullptr; A->values_gen = 0; A->source_gen = 0;
  isp_csr_info_t& I = A->info;
  const build_counters& h = po.h;
  I.n_rows = n_rows; I.n_cols = n_cols; I.nnz = nnz; I.max_degree = (int64_t)h.max_degree;
  for (int b = 0; b < 5; ++b) { I.bin_rows[b] = (int64_t)h.bin_rows[b]; I.bin_nnz[b] = (int64_t)h.bin_nnz[b]; }
  I.hub_threshold = pp.hub_t; I.segment_len = pp.seg_len; I.block_cost = pp.block_cost;
  I.n_row_blocks = h.n_blocks; I.n_hub_rows = h.n_hub; I.n_segments = h.n_seg;
  I.is_transpose = 0; I.has_cached_transpose = 0;
  I.spmm_mid_threshold = 0; I.spmm_cut_rows = 0; I.spmm_pieces = 0; I.spmm_row_blocks = 0; I.symmetric_pattern = 0;
  if (mid_t > 0 && nnz > 0) {
    st = build_packed(A, pp, mid_t, base, P, ws_bytes, s);
    if (st != ISP_OK) { delete A; return st; }
  }
  *out = A;
  return ISP_OK;
}
