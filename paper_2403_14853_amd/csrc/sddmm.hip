// SDDMM: out[p] = <U[i, :], V[col_p, :]> for every stored entry p of row i, in A's CSR order
// (paper Section 1: one of the two sparse operations GNN training rests on).  With U = dY and
// V = X this is the gradient of Y = A X with respect to A's stored values.
//
// Same work items as SpMM.  The wave keeps U's row in registers, gathers V's rows with the 64
// lanes spread over the feature dimension, and reduces each product across the wave.  Results
// of up to 64 consecutive entries are collected one per lane and stored coalesced.
#include "grouped_ops.h"

namespace {
using namespace isp_dev;

template <int VEC, bool HAS_VAL, bool SCALE, bool ADD>
__global__ void __launch_bounds__(ISP_WG) k_sddmm(isp_view A, const int64_t* __restrict__ indptr,
                                                  const int32_t* __restrict__ indices,
                                                  const float* __restrict__ values, const float* __restrict__ Um,
                                                  int64_t ldu, const float* __restrict__ Vm, int64_t ldv, int d, int k0,
                                                  float* __restrict__ out) {
  constexpr int U = 8;
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * ISP_WAVES_PER_WG + (threadIdx.x >> 6)));
  if (item >= A.n_blocks + A.n_seg) return;
  const item_range it = locate_item(A, indptr, item);
  if (it.skip) return;
  const int col = k0 + lane * VEC;
  const bool on = col < d;

  int row = it.src_row;
  // segment items stay inside one row; block items walk rows [row, row_last)
  const int row_stop = it.is_seg ? row + 1 : it.row_last;
  int64_t p = it.p;
  const int64_t p_end = it.p_end;
  int64_t row_end = it.is_seg ? p_end : indptr[row + 1];
  while (row < row_stop && row_end == p && !it.is_seg) { ++row; row_end = (row < row_stop) ? indptr[row + 1] : INT64_MAX; }

  float u[VEC];
  auto load_u = [&]() {
#pragma unroll
    for (int v = 0; v < VEC; ++v) u[v] = 0.f;
    if (on && row < row_stop) load_vec<VEC>(Um + (int64_t)row * ldu + col, u);
  };
  load_u();

  while (p < p_end) {
    const int64_t left = p_end - p;
    const int cnt = left < ISP_WAVE ? (int)left : ISP_WAVE;
    int c = 0;
    float a = 1.f;
    if (lane < cnt) {
      c = __builtin_nontemporal_load(indices + p + lane);
      if (HAS_VAL && SCALE) a = __builtin_nontemporal_load(values + p + lane);
    }
    float res = 0.f;  // lane t ends up with the dot product of entry p + t
    for (int t = 0; t < cnt; t += U) {
      float x[U][VEC];
      const bool full = t + U <= cnt;
#pragma unroll
      for (int q = 0; q < U; ++q) {
        if (full || t + q < cnt) {
          const int cj = bcast_i(c, t + q);
#pragma unroll
          for (int v = 0; v < VEC; ++v) x[q][v] = 0.f;
          if (on) load_vec<VEC>(Vm + (int64_t)cj * ldv + col, x[q]);
        }
      }
#pragma unroll
      for (int q = 0; q < U; ++q) {
        if (full || t + q < cnt) {
          float part = 0.f;
#pragma unroll
          for (int v = 0; v < VEC; ++v) part = fmaf(u[v], x[q][v], part);
          const float dot = wave_allreduce(part);
          if (lane == t + q) res = dot;
          if (p + t + q + 1 == row_end && !it.is_seg) {
            ++row;
            row_end = (row < row_stop) ? indptr[row + 1] : INT64_MAX;
            while (row < row_stop && row_end == p + t + q + 1) { ++row; row_end = (row < row_stop) ? indptr[row + 1] : INT64_MAX; }
            load_u();
          }
        }
      }
    }
    if (lane < cnt) {
      if (HAS_VAL && SCALE) res *= a;
      if (ADD) res += out[p + lane];
      out[p + lane] = res;
    }
    p += cnt;
  }
}

// ---- grouped fast path (d % 4 == 0, 16-byte aligned operands) ------------------------------------
// ADD: this pass covers a window of the feature columns and adds its partial dot product to out.
// The entry's staged value multiplies the dot product; it is 1 when the kernel is given no values
// (unscaled SDDMM, or a matrix without stored values).
// SPARSE: empty rows own no step (worth it where many rows are empty).
template <bool ADD_ = false, bool SPARSE_ = false>
struct sddmm_policy {
  static constexpr int NSRC = 1, NROW = 1, STEPS = 4;
  static constexpr bool PER_ENTRY = true, ACCUMULATE = false, ADD = ADD_, SPARSE_ROWS = SPARSE_;
  struct args { const float* src[1]; int64_t lds_[1]; const float* rowop[1]; int64_t ldr[1]; float* out_entry; };
  template <int LPG, int W>
  __device__ static inline float entry(float a, const float (&x)[1][W], const float (&r)[1][W], const lane_cols<W / 4>& lc) {
    return a * group_allreduce<LPG>(dotw<W>(r[0], x[0], lc));
  }
};

template <int LPG, int W, bool ADDR32, bool ADD, bool SPARSE>
__global__ void __launch_bounds__(ISP_WG) k_sddmm_grouped(isp_view A, const int64_t* __restrict__ indptr,
                                                          const int32_t* __restrict__ indices,
                                                          const float* __restrict__ values,
                                                          typename sddmm_policy<ADD, SPARSE>::args pa, int d, int k_lo) {
  __shared__ gs_lds lds;
  fused_grouped_item<sddmm_policy<ADD, SPARSE>, LPG, W, ADDR32>(A, indptr, indices, values, pa, d, nullptr, 0, lds, k_lo);
}

// One pass over the feature columns [k_lo, d_hi) (d_hi - k_lo <= W * LPG); add: accumulate into out.
template <int LPG, int W>
isp_status launch_grouped(const isp_csr* A, const float* U, int64_t ldu, const float* V, int64_t ldv, int k_lo,
                          int d_hi, bool add, bool scale, float* out, hipStream_t s) {
  const isp_view& v = A->v;
  const int n_items = v.n_blocks + v.n_seg;
  if (n_items == 0 || v.nnz == 0) return ISP_OK;
  const unsigned grid = (unsigned)((n_items + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG);
  const float* vals = scale ? v.values : nullptr;
  const bool a32 = fused_offsets_fit_32(v.n_cols, ldv, d_hi);
  typename sddmm_policy<false>::args pa{{V}, {ldv}, {U}, {ldu}, out};  // (the same members in every variant)
  // rows without entries: skipped through the list of non-empty rows when they are an eighth of all rows or more
  // (the list costs one LDS read per step, an empty row's step a whole step)
  const bool sparse = A->info.bin_rows[0] * 8 >= A->info.n_rows;
#define ISP_GO(A32, AD, SP)                                                                                  \
  do {                                                                                                       \
    typename sddmm_policy<AD, SP>::args pb{{pa.src[0]}, {pa.lds_[0]}, {pa.rowop[0]}, {pa.ldr[0]}, pa.out_entry}; \
    k_sddmm_grouped<LPG, W, A32, AD, SP><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, vals, pb, d_hi, k_lo); \
  } while (0)
#define ISP_GO2(A32, AD) do { if (sparse) ISP_GO(A32, AD, true); else ISP_GO(A32, AD, false); } while (0)
  if (a32) { if (add) ISP_GO2(true, true); else ISP_GO2(true, false); }
  else { if (add) ISP_GO2(false, true); else ISP_GO2(false, false); }
#undef ISP_GO2
#undef ISP_GO
  ISP_LAUNCH_CHECK();
  return ISP_OK;
}

template <int VEC>
isp_status launch(const isp_csr* A, const float* U, int64_t ldu, const float* V, int64_t ldv, int d, int k0,
                  bool scale, bool add, float* out, hipStream_t s) {
  const isp_view& v = A->v;
  const int n_items = v.n_blocks + v.n_seg;
  if (n_items == 0 || v.nnz == 0) return ISP_OK;
  const unsigned grid = (unsigned)((n_items + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG);
  const bool sc = scale && v.values;
#define ISP_SDDMM_GO(HV, SC, AD) \
  k_sddmm<VEC, HV, SC, AD><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, U, ldu, V, ldv, d, k0, out)
  if (sc) { if (add) ISP_SDDMM_GO(true, true, true); else ISP_SDDMM_GO(true, true, false); }
  else { if (add) ISP_SDDMM_GO(false, false, true); else ISP_SDDMM_GO(false, false, false); }
#undef ISP_SDDMM_GO
  ISP_LAUNCH_CHECK();
  return ISP_OK;
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

}  // namespace

isp_status isp_sddmm_launch(const isp_csr* A, const float* U, int64_t ldu, const float* V, int64_t ldv, int32_t d,
                            bool scale, float* out, hipStream_t s) {
  const isp_view& av = A->v;
  const bool grouped_ok = d % 4 == 0 && ldu % 4 == 0 && ldv % 4 == 0 && aligned(U, 16) &&
                          aligned(V, 16) && A->info.block_cost <= GS_MAX_ROWS &&
                          A->info.block_cost + av.hub_t <= GS_MAX_ENT && av.seg_len <= GS_MAX_ENT &&
                          !A->tune.no_grouped;
  if (grouped_ok) {
    // One pass covers a window of the feature columns; later passes add their partial dot products.
    //  - big graphs with many columns, rows of whole 64-float halves: 64-column passes, so that every L2 holds
    //    half-rows of twice as many hot columns (the same effect, under the same conditions, as the column
    //    slices of SpMM);
    //  - otherwise rows wider than 128 floats go 128 columns at a time on the big graphs, 256 on the others.
    const bool big = av.nnz >= ((int64_t)8 << 20);
    int wp = d;
    if (big && av.n_cols >= (1 << 19) && d > ISP_WAVE && d % ISP_WAVE == 0 && ldu % 32 == 0 && ldv % 32 == 0 &&
        !A->tune.sddmm_one_pass)
      wp = ISP_WAVE;
    else if (big && d > 2 * ISP_WAVE) wp = 2 * ISP_WAVE;
    else if (d > ISP_PARTIAL_TILE) wp = ISP_PARTIAL_TILE;
    isp_status st = ISP_OK;
    for (int k_lo = 0; k_lo < d && st == ISP_OK; k_lo += wp) {
      const int k_hi = k_lo + wp < d ? k_lo + wp : d, w = k_hi - k_lo;
      const bool add = k_lo > 0;
      // one float4 per lane up to 64 columns, two above (half the lanes per dot product: fewer instructions per
      // entry where a step's eight-plus entries are mostly live; measured on the benchmark graphs);
      // ISP_FUSED_W=4 / 8 forces either
      const bool two = A->tune.fused_w ? A->tune.fused_w == 8 : w > 64;
      if (w <= 32) st = launch_grouped<8, 4>(A, U, ldu, V, ldv, k_lo, k_hi, add, scale, out, s);
      else if (!two) {
        if (w <= 64) st = launch_grouped<16, 4>(A, U, ldu, V, ldv, k_lo, k_hi, add, scale, out, s);
        else if (w <= 128) st = launch_grouped<32, 4>(A, U, ldu, V, ldv, k_lo, k_hi, add, scale, out, s);
        else st = launch_grouped<64, 4>(A, U, ldu, V, ldv, k_lo, k_hi, add, scale, out, s);
      }
      else if (w <= 64) st = launch_grouped<8, 8>(A, U, ldu, V, ldv, k_lo, k_hi, add, scale, out, s);
      else if (w <= 128) st = launch_grouped<16, 8>(A, U, ldu, V, ldv, k_lo, k_hi, add, scale, out, s);
      else st = launch_grouped<32, 8>(A, U, ldu, V, ldv, k_lo, k_hi, add, scale, out, s);
    }
    return st;
  }
  int vec = 1;
  if (d > 2 * ISP_WAVE && d % 4 == 0 && ldu % 4 == 0 && ldv % 4 == 0 && aligned(U, 16) && aligned(V, 16)) vec = 4;
  else if (d > ISP_WAVE && d % 2 == 0 && ldu % 2 == 0 && ldv % 2 == 0 && aligned(U, 8) && aligned(V, 8)) vec = 2;
  isp_status st = ISP_OK;
  // feature tiles of 64 * vec columns; the first tile writes out, later tiles add their partial dot products
  for (int k0 = 0; k0 < d && st == ISP_OK; k0 += ISP_WAVE * vec) {
    const bool add = k0 > 0;
    if (vec == 4) st = launch<4>(A, U, ldu, V, ldv, d, k0, scale, add, out, s);
    else if (vec == 2) st = launch<2>(A, U, ldu, V, ldv, d, k0, scale, add, out, s);
    else st = launch<1>(A, U, ldu, V, ldv, d, k0, scale, add, out, s);
  }
  return st;
}
