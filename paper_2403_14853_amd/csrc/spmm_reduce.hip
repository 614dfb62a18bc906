// Sparse-dense product with the other reductions the paper's matmul offers (Section 3.4, 3.5):
// mean, min, max - and their backward through the cached transpose.  The sum reduction has the tuned
// kernels; mean reuses them when the operands qualify (rows divided by their length), min / max have a
// grouped forward kernel of the same design for float4-aligned operands, and everything else runs on the
// generic row-streaming skeleton (one nonzero per wave iteration, any width and alignment).
//   mean : Y[i] = (sum_p a_p x_j) / len_i
//   min / max : Y[i,k] = min / max_p a_p x_jk (product and comparison in fp32), arg[i,k] = position p of
//               the first entry attaining it; empty row -> 0 and -1
//   backward mean    : dX[j] = sum_{p in column j} (a_p / len_row(p)) dY[row(p)]
//   backward min/max : dX[j,k] = sum_{p in column j, arg[row(p),k] == p} a_p dY[row(p),k]
// Both backward forms are row passes over the cached transpose (whose perm gives p), so no
// floating-point atomics are needed and results are deterministic.
#include "row_stream.h"
#include "group_stream.h"

namespace {
using namespace isp_dev;

constexpr int R_MEAN = 1, R_MIN = 2, R_MAX = 3;
constexpr int ARG_OFF = ISP_PARTIAL_TILE / 2;  // hub partial rows: values in [0,128), arg bits in [128,256)

// ---- forward -----------------------------------------------------------------------------------
template <int VEC_, int MODE, bool HAS_VAL_>
struct reduce_fwd_policy {
  static constexpr int VEC = VEC_, T = 1, NG = 1, U = 8;
  static constexpr bool HAS_VAL = HAS_VAL_, ACCUMULATE = false, NEEDS_PERM = false, HAS_FINISH = true;
  struct args { const float* src[1]; int64_t ld[1]; int32_t* arg; int d; const int32_t* perm; };
  struct row_state { int where[VEC]; };
  __device__ static inline void row_begin(const args&, row_state& rs, int, const int (&)[1], const bool (&)[1]) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) rs.where[v] = -1;
  }
  __device__ static inline void edge(const args&, row_state& rs, float a, const float (&x)[1][1][VEC],
                                     float (&acc)[1][VEC], const bool (&)[1], const edge_info& ei) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      if (MODE == R_MEAN) {
        acc[0][v] = fmaf(a, x[0][0][v], acc[0][v]);
      } else {
        const float t = __fmul_rn(a, x[0][0][v]);  // one rounded fp32 multiply, never fused
        const bool take = rs.where[v] < 0 || (MODE == R_MIN ? t < acc[0][v] : t > acc[0][v]);
        acc[0][v] = take ? t : acc[0][v];
        rs.where[v] = take ? (int)ei.pos : rs.where[v];
      }
    }
  }
  __device__ static inline void finish(const args& pa, row_state& rs, float (&acc)[1][VEC], int out_row, bool is_seg,
                                       int64_t row_len, float* side, const int (&col)[1], const bool (&on)[1],
                                       int k0) {
    if (MODE == R_MEAN) {
      if (!is_seg) {  // segments hold plain partial sums; the fix-up divides
        const float inv = row_len > 0 ? 1.f / (float)row_len : 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[0][v] *= inv;
      }
    } else if (on[0]) {
      // an empty row never saw row_begin: its position is -1 by definition
      const bool empty = !is_seg && row_len == 0;
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        const int w = empty ? -1 : rs.where[v];
        if (is_seg) side[ARG_OFF + col[0] - k0 + v] = __int_as_float(w);
        else pa.arg[(int64_t)out_row * pa.d + col[0] + v] = w;
      }
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) rs.where[v] = -1;
  }
};

template <int VEC, int MODE, bool HAS_VAL>
__global__ void __launch_bounds__(ISP_WG) k_reduce_fwd(isp_view A, const int64_t* __restrict__ indptr,
                                                       const int32_t* __restrict__ indices,
                                                       const float* __restrict__ values, const float* __restrict__ X,
                                                       int64_t ldx, int d, int k0, float* __restrict__ Y, int64_t ldy,
                                                       int32_t* __restrict__ arg) {
  using P = reduce_fwd_policy<VEC, MODE, HAS_VAL>;
  typename P::args pa;
  pa.src[0] = X; pa.ld[0] = ldx; pa.arg = arg; pa.d = d; pa.perm = nullptr;
  stream_item<P>(A, indptr, indices, values, pa, d, k0, Y, ldy);
}

// ---- grouped forward of min / max ---------------------------------------------------------------------
// The grouped SpMM's work items, LDS staging, step tables and two-buffer pipeline (group_stream.h) with the
// accumulation replaced by a running (value, position) pair per column.  A group of LPG lanes covers a slice
// of 4 * LPG columns and G = 64 / LPG entries share a gather; group g meets entries g, g + G, ... of a row in
// ascending position, so "replace only if strictly better" keeps the first entry within a group, and the
// groups' pairs are combined with ties going to the smaller position: the first entry of the row that
// attains the extremum, as the definition asks.  Hub segments leave (value, position) halves in their
// partial rows exactly as the generic kernel does, and the same fix-up combines them in segment order.
// Needs float4 lanes and 32-bit gather offsets; a launch covers at most 128 columns (the partial rows).
template <int MODE>
__device__ inline bool mm_better(float t, float best) { return MODE == R_MIN ? t < best : t > best; }

template <int LPG, int MODE, bool HAS_VAL, bool SPARSE_ROWS>
__global__ void __launch_bounds__(ISP_WG) k_minmax_grouped(isp_view A, const int64_t* __restrict__ indptr,
                                                           const int32_t* __restrict__ indices,
                                                           const float* __restrict__ values,
                                                           const float* __restrict__ X, int64_t ldx, int d, int k_base,
                                                           int n_slices, float* __restrict__ Y, int64_t ldy,
                                                           int32_t* __restrict__ arg) {
  constexpr int G = ISP_WAVE / LPG;
  constexpr int U = GS_U;
  __shared__ gs_lds lds;
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  const int w = threadIdx.x >> 6;
  const int slice = __builtin_amdgcn_readfirstlane((int)(blockIdx.x % n_slices));
  const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x / n_slices) * ISP_WAVES_PER_WG + w);
  if (item >= A.n_blocks + A.n_seg) return;
  const item_range it = locate_item(A, indptr, item);
  if (it.skip) return;
  gs_wave_lds& L = lds.w[w];
  int n_live = 0;  // non-empty rows of a row block
  const int n_steps = gs_prepare<G, HAS_VAL, SPARSE_ROWS>(it, indptr, indices, values, L, lane, &n_live);  // multiple of U

  const int g = lane / LPG, q = lane % LPG;
  const int col = k_base + (slice * LPG + q) * 4;
  const bool lane_on = col < d;
  const unsigned lane_byte = lane_on ? (unsigned)col * 4u : 0u;
  const unsigned pitch_byte = (unsigned)ldx * 4u;
  const int p0 = (int)it.p;  // position of the item's first entry (nnz < 2^31)

  float best[4];
  int where[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) { best[v] = 0.f; where[v] = -1; }
  const bool listed = SPARSE_ROWS && !it.is_seg;
  auto store_row = [&](int row) {  // this lane's four columns of one finished row (or segment)
    if (it.is_seg) {
      float* pr = A.partials + (int64_t)row * ISP_PARTIAL_TILE + (col - k_base);
      float wb[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) wb[v] = __int_as_float(where[v]);
      store_vec<4>(pr, best);
      store_vec<4>(pr + ARG_OFF, wb);
    } else {
      store_vec<4>(Y + (int64_t)row * ldy + col, best);
      *reinterpret_cast<int4*>(arg + (int64_t)row * d + col) = make_int4(where[0], where[1], where[2], where[3]);
    }
  };
  if (listed && lane_on) {  // empty rows (listed behind the non-empty ones): value 0, position -1
    const int n_empty = it.row_last - it.row - n_live;
    for (int i = g; i < n_empty; i += G) store_row(it.row + (int)L.ss[n_live + 1 + i]);
  }
  int k_done = 0;
  int r_next = listed ? (int)L.ss[0] : 0;

  auto finish_row = [&]() {
    const int row = it.row + __builtin_amdgcn_readfirstlane(r_next);
    ++k_done;
    r_next = listed ? (int)L.ss[k_done] : k_done;
#pragma unroll
    for (int o = LPG; o < ISP_WAVE; o <<= 1) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float ob = __shfl_xor(best[v], o);
        const int ow = __shfl_xor(where[v], o);
        const bool take = ow >= 0 && (where[v] < 0 || mm_better<MODE>(ob, best[v]) || (ob == best[v] && ow < where[v]));
        best[v] = take ? ob : best[v];
        where[v] = take ? ow : where[v];
      }
    }
    if (g == 0 && lane_on) store_row(row);
#pragma unroll
    for (int v = 0; v < 4; ++v) { best[v] = 0.f; where[v] = -1; }
  };
  auto issue = [&](int s0, unsigned (&dsc)[U], float (&x)[U][4], float (&a)[U]) {
    const uint4 pk = *reinterpret_cast<const uint4*>(L.step + s0);
    const unsigned raw[4] = {(unsigned)__builtin_amdgcn_readfirstlane(pk.x), (unsigned)__builtin_amdgcn_readfirstlane(pk.y),
                             (unsigned)__builtin_amdgcn_readfirstlane(pk.z), (unsigned)__builtin_amdgcn_readfirstlane(pk.w)};
    int2 e[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      dsc[u] = (raw[u >> 1] >> ((u & 1) * 16)) & 0xffffu;
      e[u] = L.ent[gs_off(dsc[u]) + g];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool act = g < gs_cnt(dsc[u]) && lane_on;
      a[u] = __int_as_float(e[u].y);
      const int cj = act ? e[u].x : 0;  // dead lanes gather row 0; what they fetch is never used
      const unsigned off = __umul24((unsigned)cj, pitch_byte) + lane_byte;
      load_vec<4>(reinterpret_cast<const float*>(reinterpret_cast<const char*>(X) + off), x[u]);
    }
  };
  auto consume = [&](const unsigned (&dsc)[U], const float (&x)[U][4], const float (&a)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (g < gs_cnt(dsc[u]) && lane_on) {
        const int pos = p0 + gs_off(dsc[u]) + g;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float t = __fmul_rn(a[u], x[u][v]);  // one rounded fp32 multiply, never fused
          const bool take = where[v] < 0 || mm_better<MODE>(t, best[v]);
          best[v] = take ? t : best[v];
          where[v] = take ? pos : where[v];
        }
      }
      if (dsc[u] & GS_LAST) finish_row();
    }
  };

  const int n_groups = n_steps / U;
  if (n_groups == 0) return;
  unsigned dA[U], dB[U];
  float xA[U][4], xB[U][4], aA[U], aB[U];
  issue(0, dA, xA, aA);
  int gi = 0;
  while (gi + 2 < n_groups) {
    issue((gi + 1) * U, dB, xB, aB);
    consume(dA, xA, aA);
    issue((gi + 2) * U, dA, xA, aA);
    consume(dB, xB, aB);
    gi += 2;
  }
  if (gi + 1 < n_groups) {
    issue((gi + 1) * U, dB, xB, aB);
    consume(dA, xA, aA);
    consume(dB, xB, aB);
  } else {
    consume(dA, xA, aA);
  }
}

// One wave per hub row: combine the segments' partial results in segment order.
template <int VEC, int MODE>
__global__ void __launch_bounds__(ISP_WG) k_reduce_fixup(isp_view A, int d, int k0, float* __restrict__ Y, int64_t ldy,
                                                         int32_t* __restrict__ arg) {
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  const int h = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * ISP_WAVES_PER_WG + (threadIdx.x >> 6)));
  if (h >= A.n_hub) return;
  const int s0 = A.hub_seg_ptr[h], s1 = A.hub_seg_ptr[h + 1];
  const int row = A.hub_rows[h];
  const int rel = lane * VEC;
  if (k0 + rel >= d) return;
  float best[VEC];
  int where[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) { best[v] = 0.f; where[v] = -1; }
  auto combine = [&](const float (&t)[VEC], const float (&wbits)[VEC]) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      if (MODE == R_MEAN) {
        best[v] += t[v];
      } else {
        const bool take = where[v] < 0 || (MODE == R_MIN ? t[v] < best[v] : t[v] > best[v]);
        best[v] = take ? t[v] : best[v];
        where[v] = take ? __float_as_int(wbits[v]) : where[v];
      }
    }
  };
  int s = s0;
  for (; s + 8 <= s1; s += 8) {  // eight segments' partial rows in flight, combined in segment order
    float t[8][VEC], wb[8][VEC];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float* pr = A.partials + (int64_t)(s + u) * ISP_PARTIAL_TILE + rel;
      load_vec<VEC>(pr, t[u]);
      if (MODE != R_MEAN) load_vec<VEC>(pr + ARG_OFF, wb[u]);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) combine(t[u], wb[u]);
  }
  for (; s < s1; ++s) {
    const float* pr = A.partials + (int64_t)s * ISP_PARTIAL_TILE + rel;
    float t[VEC], wb[VEC];
    load_vec<VEC>(pr, t);
    if (MODE != R_MEAN) load_vec<VEC>(pr + ARG_OFF, wb);
    combine(t, wb);
  }
  if (MODE == R_MEAN) {
    const int64_t len = A.indptr[row + 1] - A.indptr[row];
    const float inv = len > 0 ? 1.f / (float)len : 0.f;
#pragma unroll
    for (int v = 0; v < VEC; ++v) best[v] *= inv;
  }
#pragma unroll
  for (int v = 0; v < VEC; ++v) {
    Y[(int64_t)row * ldy + k0 + rel + v] = best[v];
    if (MODE != R_MEAN) arg[(int64_t)row * d + k0 + rel + v] = where[v];
  }
}

// ---- backward (row passes over the cached transpose) ---------------------------------------------
// mean: entry (j <- i) contributes (a / len_A(i)) dY[i]; len_A from the source matrix's row offsets.
template <int VEC_, bool HAS_VAL_>
struct mean_bwd_policy {
  static constexpr int VEC = VEC_, T = 1, NG = 1, U = 8;
  static constexpr bool HAS_VAL = HAS_VAL_, ACCUMULATE = false, NEEDS_PERM = false, HAS_FINISH = false;
  struct args { const float* src[1]; int64_t ld[1]; const int64_t* src_indptr; const int32_t* perm; };
  struct row_state {};
  __device__ static inline void row_begin(const args&, row_state&, int, const int (&)[1], const bool (&)[1]) {}
  __device__ static inline void edge(const args& pa, row_state&, float a, const float (&x)[1][1][VEC],
                                     float (&acc)[1][VEC], const bool (&)[1], const edge_info& ei) {
    const int64_t len = pa.src_indptr[ei.col + 1] - pa.src_indptr[ei.col];
    const float w = a / (float)len;  // len >= 1: the entry itself lies in that row
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[0][v] = fmaf(w, x[0][0][v], acc[0][v]);
  }
};

// min / max: gathers dY[i] and arg[i] (as bit patterns); the entry contributes where arg equals its
// position p = perm[q] in the source matrix.  An entry that no column of its row selected (live[q] == 0,
// marked from arg before the pass) is passed over without gathering anything: in a row of many entries at
// most d of them are selected.
template <int VEC_, bool HAS_VAL_>
struct select_bwd_policy {
  static constexpr int VEC = VEC_, T = 1, NG = 2, U = 4;
  static constexpr bool HAS_VAL = HAS_VAL_, ACCUMULATE = false, NEEDS_PERM = true, HAS_FINISH = false, HAS_SKIP = true;
  struct args { const float* src[2]; int64_t ld[2]; const int32_t* perm; const uint8_t* live; };
  struct row_state {};
  __device__ static inline void row_begin(const args&, row_state&, int, const int (&)[1], const bool (&)[1]) {}
  __device__ static inline void edge(const args&, row_state&, float a, const float (&x)[2][1][VEC],
                                     float (&acc)[1][VEC], const bool (&)[1], const edge_info& ei) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const bool mine = __float_as_int(x[1][0][v]) == ei.perm;
      acc[0][v] = mine ? fmaf(a, x[0][0][v], acc[0][v]) : acc[0][v];
    }
  }
};

template <class P>
__global__ void __launch_bounds__(ISP_WG) k_reduce_bwd(isp_view At, const int64_t* __restrict__ indptr,
                                                       const int32_t* __restrict__ indices,
                                                       const float* __restrict__ values, typename P::args pa, int d,
                                                       int k0, float* __restrict__ dX, int64_t lddx) {
  stream_item<P>(At, indptr, indices, values, pa, d, k0, dX, lddx);
}

// live[q] = 1 for every entry q of the transpose whose source position p = perm[q] arg names (positions
// outside [0, nnz) - the -1 of empty rows, or anything a caller's array may hold - are ignored); live was
// zeroed before.  A row's columns name positions inside that row, so the lookups in inv_perm stay local.
__global__ void __launch_bounds__(256) k_mark_selected(const int32_t* __restrict__ arg, int64_t n, int64_t nnz,
                                                       const int32_t* __restrict__ inv_perm,
                                                       uint8_t* __restrict__ live) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  const int32_t p = arg[t];
  if (p >= 0 && p < nnz) live[inv_perm[p]] = 1;
}

__global__ void __launch_bounds__(256) k_zero_u32(uint32_t* __restrict__ a, int64_t n) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) a[t] = 0u;
}

template <int VEC>
__global__ void __launch_bounds__(ISP_WG) k_sum_fixup(isp_view A, int d, int k0, float* __restrict__ Y, int64_t ldy) {
  hub_fixup<VEC, 1, false>(A, d, k0, Y, ldy);
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

unsigned item_grid(const isp_view& v) { return (unsigned)((v.n_blocks + v.n_seg + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG); }
unsigned hub_grid(const isp_view& v) { return (unsigned)((v.n_hub + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG); }

template <int VEC, int MODE>
isp_status fwd_tile(const isp_csr* A, const float* X, int64_t ldx, int d, int k0, float* Y, int64_t ldy, int32_t* arg,
                    hipStream_t s) {
  const isp_view& v = A->v;
  if (v.n_blocks + v.n_seg > 0) {
    if (v.values) k_reduce_fwd<VEC, MODE, true><<<item_grid(v), ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, X, ldx, d, k0, Y, ldy, arg);
    else k_reduce_fwd<VEC, MODE, false><<<item_grid(v), ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, X, ldx, d, k0, Y, ldy, arg);
    ISP_LAUNCH_CHECK();
  }
  if (v.n_hub > 0) {
    k_reduce_fixup<VEC, MODE><<<hub_grid(v), ISP_WG, 0, s>>>(v, d, k0, Y, ldy, arg);
    ISP_LAUNCH_CHECK();
  }
  return ISP_OK;
}

template <int LPG, int MODE>
isp_status minmax_grouped_tile(const isp_csr* A, const float* X, int64_t ldx, int d, int k_base, int n_slices, float* Y,
                               int64_t ldy, int32_t* arg, hipStream_t s) {
  const isp_view& v = A->v;
  const int n_items = v.n_blocks + v.n_seg;
  if (n_items > 0) {
    const unsigned grid = (unsigned)((n_items + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG) * (unsigned)n_slices;
    const bool sparse_rows = A->info.bin_rows[0] * 16 > A->info.n_rows;  // (as the grouped SpMM chooses)
#define ISP_GO(HV, SR)                                                                                             \
  k_minmax_grouped<LPG, MODE, HV, SR><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, X, ldx, d, k_base, \
                                                              n_slices, Y, ldy, arg)
    if (v.values) { if (sparse_rows) ISP_GO(true, true); else ISP_GO(true, false); }
    else { if (sparse_rows) ISP_GO(false, true); else ISP_GO(false, false); }
#undef ISP_GO
    ISP_LAUNCH_CHECK();
  }
  if (v.n_hub > 0) {
    k_reduce_fixup<2, MODE><<<hub_grid(v), ISP_WG, 0, s>>>(v, d, k_base, Y, ldy, arg);
    ISP_LAUNCH_CHECK();
  }
  return ISP_OK;
}

template <int MODE>
isp_status fwd_all(const isp_csr* A, const float* X, int64_t ldx, int d, float* Y, int64_t ldy, int32_t* arg,
                   hipStream_t s) {
  const isp_view& av = A->v;
  if constexpr (MODE != R_MEAN) {
    // grouped kernel: float4 lanes, 32-bit gather offsets, the partition within the LDS tables' limits
    const bool a32 = av.n_cols < (1 << 24) && ldx * 4 < (1 << 24) &&
                     ((uint64_t)av.n_cols * (uint64_t)ldx + (uint64_t)d) * 4u < ((uint64_t)1 << 32);
    const bool ok = av.nnz > 0 && a32 && d % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && aligned(X, 16) &&
                    aligned(Y, 16) && aligned(arg, 16) && A->info.block_cost <= GS_MAX_ROWS &&
                    A->info.block_cost + av.hub_t <= GS_MAX_ENT && av.seg_len <= GS_MAX_ENT && !A->tune.no_grouped;
    if (ok) {
      // 128 columns per launch (a hub partial row holds 128 values and 128 positions), one slice: the two
      // 64-column slices that pay for the sum on large graphs cost more here than they save, the loop doing
      // four compare-and-select steps per entry instead of four multiply-adds (config 3: 7.09 vs 6.05 ms)
      isp_status st = ISP_OK;
      for (int k_base = 0; k_base < d && st == ISP_OK; k_base += 2 * ISP_WAVE) {
        const int w = d - k_base < 2 * ISP_WAVE ? d - k_base : 2 * ISP_WAVE;
        if (w <= 32) st = minmax_grouped_tile<8, MODE>(A, X, ldx, d, k_base, 1, Y, ldy, arg, s);
        else if (w <= 64) st = minmax_grouped_tile<16, MODE>(A, X, ldx, d, k_base, 1, Y, ldy, arg, s);
        else st = minmax_grouped_tile<32, MODE>(A, X, ldx, d, k_base, 1, Y, ldy, arg, s);
      }
      return st;
    }
  }
  // min / max keep (value, position) pairs in the hub partial rows, so their column tiles stop at 128
  const bool v2 = d % 2 == 0 && ldx % 2 == 0 && ldy % 2 == 0 && aligned(X, 8) && aligned(Y, 8) && d > ISP_WAVE;
  isp_status st = ISP_OK;
  for (int k0 = 0; k0 < d && st == ISP_OK; k0 += (v2 ? 2 : 1) * ISP_WAVE)
    st = v2 ? fwd_tile<2, MODE>(A, X, ldx, d, k0, Y, ldy, arg, s) : fwd_tile<1, MODE>(A, X, ldx, d, k0, Y, ldy, arg, s);
  return st;
}

template <class P, int VEC>
isp_status bwd_tile(const isp_csr* At, const typename P::args& pa, int d, int k0, float* dX, int64_t lddx,
                    hipStream_t s) {
  const isp_view& v = At->v;
  if (v.n_blocks + v.n_seg > 0) {
    k_reduce_bwd<P><<<item_grid(v), ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, pa, d, k0, dX, lddx);
    ISP_LAUNCH_CHECK();
  }
  if (v.n_hub > 0) {
    k_sum_fixup<VEC><<<hub_grid(v), ISP_WG, 0, s>>>(v, d, k0, dX, lddx);
    ISP_LAUNCH_CHECK();
  }
  return ISP_OK;
}

template <int VEC, bool HV>
isp_status mean_bwd(const isp_csr* A, const float* dY, int64_t lddy, int d, int k0, float* dX, int64_t lddx,
                    hipStream_t s) {
  using P = mean_bwd_policy<VEC, HV>;
  typename P::args pa{{dY}, {lddy}, A->v.indptr, nullptr};
  return bwd_tile<P, VEC>(A->At, pa, d, k0, dX, lddx, s);
}

template <int VEC, bool HV>
isp_status select_bwd(const isp_csr* A, const float* dY, int64_t lddy, const int32_t* arg, int d, int k0, float* dX,
                      int64_t lddx, hipStream_t s) {
  using P = select_bwd_policy<VEC, HV>;
  typename P::args pa{{dY, reinterpret_cast<const float*>(arg)}, {lddy, (int64_t)d}, A->At->perm, A->At->sel_flags};
  return bwd_tile<P, VEC>(A->At, pa, d, k0, dX, lddx, s);
}

}  // namespace

isp_status isp_spmm_reduce_launch(const isp_csr* A, const float* X, int64_t ldx, int32_t d, int reduce, float* Y,
                                  int64_t ldy, int32_t* arg, hipStream_t s) {
  if (reduce == R_MEAN) {  // the tuned kernel divides each finished row by its length
    bool done = false;
    const isp_status st = isp_spmm_grouped_launch(A, X, ldx, d, Y, ldy, 1, nullptr, s, &done);
    if (done || st != ISP_OK) return st;
    return fwd_all<R_MEAN>(A, X, ldx, d, Y, ldy, arg, s);
  }
  if (reduce == R_MIN) return fwd_all<R_MIN>(A, X, ldx, d, Y, ldy, arg, s);
  return fwd_all<R_MAX>(A, X, ldx, d, Y, ldy, arg, s);
}

isp_status isp_spmm_reduce_bwd_launch(isp_csr* A, const float* dY, int64_t lddy, int32_t d, int reduce,
                                      const int32_t* arg, float* dX, int64_t lddx, hipStream_t s) {
  const isp_csr* At = A->At;
  if (reduce == R_MEAN && At->v.nnz > 0) {
    // the tuned kernels on A^T with every value divided by its source row's length (computed once per handle)
    const float *mv = nullptr, *mv_packed = nullptr;
    isp_status st = isp_transpose_mean_values(A, s, &mv, &mv_packed);
    if (st != ISP_OK) return st;
    bool done = false;
    st = isp_spmm_grouped_launch(At, dY, lddy, d, dX, lddx, 0, mv, s, &done, mv_packed);
    if (done || st != ISP_OK) return st;
  }
  const bool hv = At->v.values != nullptr;
  const bool v2 = d % 2 == 0 && lddy % 2 == 0 && lddx % 2 == 0 && aligned(dY, 8) && aligned(dX, 8) &&
                  aligned(arg, 8) && d > ISP_WAVE;
  isp_status st = ISP_OK;
  if (reduce != R_MEAN && At->v.nnz > 0) {  // which entries of A does arg name at all (any column)?
    const int64_t nnz = At->v.nnz, words = (nnz + 3) / 4, n_arg = A->v.n_rows * (int64_t)d;
    const int32_t* inv_perm = nullptr;
    st = isp_transpose_inverse_perm(A, s, &inv_perm);
    if (st != ISP_OK) return st;
    k_zero_u32<<<(unsigned)((words + 255) / 256), 256, 0, s>>>(reinterpret_cast<uint32_t*>(At->sel_flags), words);
    ISP_LAUNCH_CHECK();
    if (n_arg > 0) {
      k_mark_selected<<<(unsigned)((n_arg + 255) / 256), 256, 0, s>>>(arg, n_arg, nnz, inv_perm, At->sel_flags);
      ISP_LAUNCH_CHECK();
    }
  }
  for (int k0 = 0; k0 < d && st == ISP_OK; k0 += (v2 ? 2 : 1) * ISP_WAVE) {
    if (reduce == R_MEAN) {
      if (v2 && hv) st = mean_bwd<2, true>(A, dY, lddy, d, k0, dX, lddx, s);
      else if (v2) st = mean_bwd<2, false>(A, dY, lddy, d, k0, dX, lddx, s);
      else if (hv) st = mean_bwd<1, true>(A, dY, lddy, d, k0, dX, lddx, s);
      else st = mean_bwd<1, false>(A, dY, lddy, d, k0, dX, lddx, s);
    } else {
      if (v2 && hv) st = select_bwd<2, true>(A, dY, lddy, arg, d, k0, dX, lddx, s);
      else if (v2) st = select_bwd<2, false>(A, dY, lddy, arg, d, k0, dX, lddx, s);
      else if (hv) st = select_bwd<1, true>(A, dY, lddy, arg, d, k0, dX, lddx, s);
      else st = select_bwd<1, false>(A, dY, lddy, arg, d, k0, dX, lddx, s);
    }
  }
  return st;
}
