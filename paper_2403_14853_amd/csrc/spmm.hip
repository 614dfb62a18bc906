// SpMM, sum reduction: Y = A X with A in CSR and X dense row-major (paper: abstract, Sections 1,
// 3.4, 3.5).  The backward dX = A^T dY is this same code run on the cached transpose's handle
// (Section 3.3).  Gather-bound: per nonzero one 4*d-byte row of X is fetched and d FMAs are done,
// so the kernels are built around coalesced row gathers, not around matrix cores.
#include "row_stream.h"

namespace {
using namespace isp_dev;

template <int VEC_, int T_, bool HAS_VAL_>
struct spmm_policy {
  static constexpr int VEC = VEC_, T = T_, NG = 1;
  static constexpr int U = (VEC * T >= 4) ? 4 : 8;
  static constexpr bool HAS_VAL = HAS_VAL_, ACCUMULATE = false;
  struct args { const float* src[1]; int64_t ld[1]; };
  struct row_state {};
  __device__ static inline void row_begin(const args&, row_state&, int, const int (&)[T], const bool (&)[T]) {}
  __device__ static inline void edge(const args&, row_state&, float a, const float (&x)[1][T][VEC],
                                     float (&acc)[T][VEC], const bool (&)[T]) {
#pragma unroll
    for (int tt = 0; tt < T; ++tt)
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[tt][v] = fmaf(a, x[0][tt][v], acc[tt][v]);
  }
};

template <int VEC, int T, bool HAS_VAL>
__global__ void __launch_bounds__(ISP_WG) k_spmm(isp_view A, const int64_t* __restrict__ indptr,
                                                 const int32_t* __restrict__ indices,
                                                 const float* __restrict__ values, const float* __restrict__ X,
                                                 int64_t ldx, int d, int k0, float* __restrict__ Y, int64_t ldy) {
  using P = spmm_policy<VEC, T, HAS_VAL>;
  typename P::args pa;
  pa.src[0] = X;
  pa.ld[0] = ldx;
  stream_item<P>(A, indptr, indices, values, pa, d, k0, Y, ldy);
}

template <int VEC, int T>
__global__ void __launch_bounds__(ISP_WG) k_spmm_fixup(isp_view A, int d, int k0, float* __restrict__ Y, int64_t ldy) {
  hub_fixup<VEC, T, false>(A, d, k0, Y, ldy);
}

template <int VEC, int T>
isp_status launch_tile(const isp_csr* A, const float* X, int64_t ldx, int d, int k0, float* Y, int64_t ldy,
                       hipStream_t s) {
  const isp_view& v = A->v;
  const int n_items = v.n_blocks + v.n_seg;
  if (n_items > 0) {
    const unsigned grid = (unsigned)((n_items + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG);
    if (v.values)
      k_spmm<VEC, T, true><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, X, ldx, d, k0, Y, ldy);
    else
      k_spmm<VEC, T, false><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, X, ldx, d, k0, Y, ldy);
    ISP_LAUNCH_CHECK();
  }
  if (v.n_hub > 0) {
    const unsigned grid = (unsigned)((v.n_hub + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG);
    k_spmm_fixup<VEC, T><<<grid, ISP_WG, 0, s>>>(v, d, k0, Y, ldy);
    ISP_LAUNCH_CHECK();
  }
  return ISP_OK;
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

}  // namespace

isp_status isp_spmm_launch(const isp_csr* A, const float* X, int64_t ldx, int32_t d, float* Y, int64_t ldy,
                           hipStream_t s) {
  // lanes-over-features layout: the widest vector the width and alignment allow
  int vec = 1;
  if (d > 2 * ISP_WAVE && d % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && aligned(X, 16) && aligned(Y, 16)) vec = 4;
  else if (d > ISP_WAVE && d % 2 == 0 && ldx % 2 == 0 && ldy % 2 == 0 && aligned(X, 8) && aligned(Y, 8)) vec = 2;
  isp_status st = ISP_OK;
  int k0 = 0;
  while (k0 < d && st == ISP_OK) {  // column tiles of at most ISP_PARTIAL_TILE floats
    const int w = d - k0;
    int step;
    if (vec == 4) { st = launch_tile<4, 1>(A, X, ldx, d, k0, Y, ldy, s); step = 4 * ISP_WAVE; }
    else if (vec == 2 && w <= 2 * ISP_WAVE) { st = launch_tile<2, 1>(A, X, ldx, d, k0, Y, ldy, s); step = 2 * ISP_WAVE; }
    else if (vec == 2) { st = launch_tile<2, 2>(A, X, ldx, d, k0, Y, ldy, s); step = 4 * ISP_WAVE; }
    else if (w <= ISP_WAVE) { st = launch_tile<1, 1>(A, X, ldx, d, k0, Y, ldy, s); step = ISP_WAVE; }
    else if (w <= 2 * ISP_WAVE) { st = launch_tile<1, 2>(A, X, ldx, d, k0, Y, ldy, s); step = 2 * ISP_WAVE; }
    else { st = launch_tile<1, 4>(A, X, ldx, d, k0, Y, ldy, s); step = 4 * ISP_WAVE; }
    k0 += step;
  }
  return st;
}
