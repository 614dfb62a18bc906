// FusedMM, sigmoid instance (paper Section 1(a): SDDMM and SpMM combined into one operation):
//   forward   s_p = sigmoid(<x_i, x_j>),  y_i = sum_p a_p s_p x_j            (j = column of p)
//   backward  dz_p = a_p <g_i, x_j> s_p (1 - s_p)
//             dX_i = sum_{p in row i} dz_p x_j + sum_{p in column i} (a_p s_p g_r + dz_p x_r)
// The per-edge scores exist only in registers: each gathered row x_j is used for the dot product
// and for the accumulation in the same pass, and the backward recomputes the scores instead of
// reading them back.  The column sum of the backward runs over the rows of the cached transpose.
#include "grouped_ops.h"

namespace {
using namespace isp_dev;

// (hardware exponential and reciprocal, about 1 ulp each; exp overflow gives 1 / inf = 0)
__device__ inline float sigmoidf_fast(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }

// Edge function s = f(z) and its derivative; op is wave-uniform (ISP_OP_SIGMOID / _DOT / _ONE).
// The grouped kernels pass it as a compile-time constant, the generic ones at run time.
__device__ inline void edge_fn(int op, float z, float& s, float& ds) {
  if (op == ISP_OP_SIGMOID) { s = sigmoidf_fast(z); ds = s * (1.f - s); }
  else if (op == ISP_OP_DOT) { s = z; ds = 1.f; }
  else { s = 1.f; ds = 0.f; }
}

template <int VEC, int T>
__device__ inline float dot_lanes(const float (&a)[T][VEC], const float (&b)[T][VEC]) {
  float s = 0.f;
#pragma unroll
  for (int tt = 0; tt < T; ++tt)
#pragma unroll
    for (int v = 0; v < VEC; ++v) s = fmaf(a[tt][v], b[tt][v], s);
  return s;
}

template <int VEC, int T>
__device__ inline void load_row(const float* __restrict__ M, int64_t ld, int row, const int (&col)[T],
                                const bool (&on)[T], float (&o)[T][VEC]) {
#pragma unroll
  for (int tt = 0; tt < T; ++tt) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) o[tt][v] = 0.f;
    if (on[tt]) load_vec<VEC>(M + (int64_t)row * ld + col[tt], o[tt]);
  }
}

constexpr int pick_u(int regs_per_edge) { return regs_per_edge >= 8 ? 2 : (regs_per_edge >= 4 ? 4 : 8); }

// ---- forward ---------------------------------------------------------------------------------
template <int VEC_, int T_, bool HAS_VAL_>
struct fwd_policy {
  static constexpr int VEC = VEC_, T = T_, NG = 1, U = pick_u(VEC_ * T_);
  static constexpr bool HAS_VAL = HAS_VAL_, ACCUMULATE = false, NEEDS_PERM = false, HAS_FINISH = false;
  struct args { const float* src[1]; int64_t ld[1]; int op; };
  struct row_state { float xi[T][VEC]; };
  __device__ static inline void row_begin(const args& pa, row_state& rs, int row, const int (&col)[T],
                                          const bool (&on)[T]) {
    load_row<VEC, T>(pa.src[0], pa.ld[0], row, col, on, rs.xi);
  }
  __device__ static inline void edge(const args& pa, row_state& rs, float a, const float (&x)[1][T][VEC],
                                     float (&acc)[T][VEC], const bool (&)[T], const edge_info&) {
    float sg = 1.f, dsg = 0.f;
    if (pa.op != ISP_OP_ONE) edge_fn(pa.op, wave_allreduce(dot_lanes<VEC, T>(rs.xi, x[0])), sg, dsg);
    const float w = a * sg;
#pragma unroll
    for (int tt = 0; tt < T; ++tt)
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[tt][v] = fmaf(w, x[0][tt][v], acc[tt][v]);
  }
};

// ---- backward, row pass over A: dX_i = sum_p dz_p x_j ----------------------------------------
template <int VEC_, int T_, bool HAS_VAL_>
struct bwd_row_policy {
  static constexpr int VEC = VEC_, T = T_, NG = 1, U = pick_u(VEC_ * T_);
  static constexpr bool HAS_VAL = HAS_VAL_, ACCUMULATE = false, NEEDS_PERM = false, HAS_FINISH = false;
  struct args { const float* src[1]; int64_t ld[1]; const float* G; int64_t ldg; int op; };
  struct row_state { float xi[T][VEC]; float gi[T][VEC]; };
  __device__ static inline void row_begin(const args& pa, row_state& rs, int row, const int (&col)[T],
                                          const bool (&on)[T]) {
    load_row<VEC, T>(pa.src[0], pa.ld[0], row, col, on, rs.xi);
    load_row<VEC, T>(pa.G, pa.ldg, row, col, on, rs.gi);
  }
  __device__ static inline void edge(const args& pa, row_state& rs, float a, const float (&x)[1][T][VEC],
                                     float (&acc)[T][VEC], const bool (&)[T], const edge_info&) {
    if (pa.op == ISP_OP_ONE) return;  // s does not depend on x_i: nothing flows through z
    const float z = wave_allreduce(dot_lanes<VEC, T>(rs.xi, x[0]));
    const float gd = wave_allreduce(dot_lanes<VEC, T>(rs.gi, x[0]));
    float sg, dsg;
    edge_fn(pa.op, z, sg, dsg);
    const float dz = a * gd * dsg;
#pragma unroll
    for (int tt = 0; tt < T; ++tt)
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[tt][v] = fmaf(dz, x[0][tt][v], acc[tt][v]);
  }
};

// ---- backward, row pass over A^T: dX_j += sum_p (a_p s_p g_i + dz_p x_i) ---------------------
// Row j of A^T lists the source rows i of the entries in column j; x_i and g_i are gathered.
template <int VEC_, int T_, bool HAS_VAL_>
struct bwd_col_policy {
  static constexpr int VEC = VEC_, T = T_, NG = 2, U = pick_u(2 * VEC_ * T_);
  static constexpr bool HAS_VAL = HAS_VAL_, ACCUMULATE = true, NEEDS_PERM = false, HAS_FINISH = false;
  struct args { const float* src[2]; int64_t ld[2]; int op; };  // src[0] = X, src[1] = dY
  struct row_state { float xj[T][VEC]; };
  __device__ static inline void row_begin(const args& pa, row_state& rs, int row, const int (&col)[T],
                                          const bool (&on)[T]) {
    load_row<VEC, T>(pa.src[0], pa.ld[0], row, col, on, rs.xj);
  }
  __device__ static inline void edge(const args& pa, row_state& rs, float a, const float (&x)[2][T][VEC],
                                     float (&acc)[T][VEC], const bool (&)[T], const edge_info&) {
    float sg = 1.f, dsg = 0.f, gd = 0.f;
    if (pa.op != ISP_OP_ONE) {
      edge_fn(pa.op, wave_allreduce(dot_lanes<VEC, T>(rs.xj, x[0])), sg, dsg);
      gd = wave_allreduce(dot_lanes<VEC, T>(rs.xj, x[1]));
    }
    const float w = a * sg;
    const float dz = a * gd * dsg;
#pragma unroll
    for (int tt = 0; tt < T; ++tt)
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[tt][v] = fmaf(w, x[1][tt][v], fmaf(dz, x[0][tt][v], acc[tt][v]));
  }
};

template <class P>
__global__ void __launch_bounds__(ISP_WG) k_fused(isp_view A, const int64_t* __restrict__ indptr,
                                                  const int32_t* __restrict__ indices,
                                                  const float* __restrict__ values, typename P::args pa, int d,
                                                  float* __restrict__ Y, int64_t ldy, int store_group, int group_cnt) {
  stream_item<P>(A, indptr, indices, values, pa, d, 0, Y, ldy, store_group, group_cnt);
}

template <int VEC, int T, bool ACC>
__global__ void __launch_bounds__(ISP_WG) k_fused_fixup(isp_view A, int d, float* __restrict__ Y, int64_t ldy) {
  hub_fixup<VEC, T, ACC>(A, d, 0, Y, ldy);
}

template <int VEC, bool ACC>
__global__ void __launch_bounds__(ISP_WG) k_fused_fixup_group(isp_view A, int d, int k0, float* __restrict__ Y,
                                                              int64_t ldy, int stride, int slot) {
  hub_fixup<VEC, 1, ACC>(A, d, k0, Y, ldy, stride, slot);
}

// store_group < 0: one launch covers all d <= 256 columns.  Otherwise (wider rows) hub segments compute with
// whole rows and store column groups [store_group, store_group + group_cnt), one partial row per group, and
// one fix-up per group adds them; the row blocks do all their work in the launch that starts at group 0.
template <class P>
isp_status run_pass(const isp_csr* A, const typename P::args& pa, int d, float* Y, int64_t ldy, hipStream_t s,
                    int store_group = -1, int group_cnt = 1) {
  const isp_view& v = A->v;
  const int n_items = v.n_blocks + v.n_seg;
  if (n_items > 0) {
    const unsigned grid = (unsigned)((n_items + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG);
    k_fused<P><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, pa, d, Y, ldy, store_group, group_cnt);
    ISP_LAUNCH_CHECK();
  }
  if (v.n_hub > 0) {
    const unsigned grid = (unsigned)((v.n_hub + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG);
    if (store_group < 0) {
      k_fused_fixup<P::VEC, P::T, P::ACCUMULATE><<<grid, ISP_WG, 0, s>>>(v, d, Y, ldy);
      ISP_LAUNCH_CHECK();
    } else {
      for (int g = 0; g < group_cnt; ++g) {
        k_fused_fixup_group<P::VEC, P::ACCUMULATE><<<grid, ISP_WG, 0, s>>>(v, d, (store_group + g) * ISP_WAVE * P::VEC, Y,
                                                                          ldy, group_cnt, g);
        ISP_LAUNCH_CHECK();
      }
    }
  }
  return ISP_OK;
}

// ---- grouped fast path (d % 4 == 0, 16-byte aligned operands) -----------------------------------
struct g_args1 { const float* src[1]; int64_t lds_[1]; const float* rowop[1]; int64_t ldr[1]; float* out_entry; int op; };
struct g_args12 { const float* src[1]; int64_t lds_[1]; const float* rowop[2]; int64_t ldr[2]; float* out_entry; int op; };
struct g_args21 { const float* src[2]; int64_t lds_[2]; const float* rowop[1]; int64_t ldr[1]; float* out_entry; int op; };

template <int OP>
struct g_fwd {  // gathered x_j, row operand x_i
  static constexpr int NSRC = 1, NROW = 1, STEPS = 4;
  static constexpr bool PER_ENTRY = false, ACCUMULATE = false;
  using args = g_args1;
  template <int LPG, int W>
  __device__ static inline void edge(const args&, float a, const float (&x)[1][W], const float (&r)[1][W],
                                     float (&acc)[W], const lane_cols<W / 4>& lc, bool live) {
    float sg = 1.f, dsg = 0.f;
    if (OP != ISP_OP_ONE) edge_fn(OP, group_allreduce<LPG>(dotw<W>(r[0], x[0], lc)), sg, dsg);
    const float w = a * sg;
    if (live) {
#pragma unroll
      for (int v = 0; v < W; ++v) acc[v] = fmaf(w, x[0][v], acc[v]);
    }
  }
};

template <int OP>
struct g_bwd_row {  // gathered x_j, row operands x_i and g_i:  dX_i += dz x_j
  static constexpr int NSRC = 1, NROW = 2, STEPS = 3;  // (three operand rows per step: three steps per buffer keep four waves resident)
  static constexpr bool PER_ENTRY = false, ACCUMULATE = false;
  using args = g_args12;
  template <int LPG, int W>
  __device__ static inline void edge(const args&, float a, const float (&x)[1][W], const float (&r)[2][W],
                                     float (&acc)[W], const lane_cols<W / 4>& lc, bool live) {
    if (OP == ISP_OP_ONE) return;  // s does not depend on x_i: nothing flows through z
    const float z = group_allreduce<LPG>(dotw<W>(r[0], x[0], lc));
    const float gd = group_allreduce<LPG>(dotw<W>(r[1], x[0], lc));
    float sg, dsg;
    edge_fn(OP, z, sg, dsg);
    const float dz = a * gd * dsg;
    if (live) {
#pragma unroll
      for (int v = 0; v < W; ++v) acc[v] = fmaf(dz, x[0][v], acc[v]);
    }
  }
};

template <int OP>
struct g_bwd_col {  // over A^T: gathered x_i and g_i, row operand x_j:  dX_j += a s g_i + dz x_i
  static constexpr int NSRC = 2, NROW = 1, STEPS = 3;
  static constexpr bool PER_ENTRY = false, ACCUMULATE = true;
  using args = g_args21;
  template <int LPG, int W>
  __device__ static inline void edge(const args&, float a, const float (&x)[2][W], const float (&r)[1][W],
                                     float (&acc)[W], const lane_cols<W / 4>& lc, bool live) {
    float sg = 1.f, dsg = 0.f, gd = 0.f;
    if (OP != ISP_OP_ONE) {
      edge_fn(OP, group_allreduce<LPG>(dotw<W>(r[0], x[0], lc)), sg, dsg);
      gd = group_allreduce<LPG>(dotw<W>(r[0], x[1], lc));
    }
    const float w = a * sg;
    const float dz = a * gd * dsg;
    if (live) {
#pragma unroll
      for (int v = 0; v < W; ++v) acc[v] = fmaf(w, x[1][v], fmaf(dz, x[0][v], acc[v]));
    }
  }
};

// Backward in ONE pass over A when A^T's structure equals A's (symmetric pattern, ascending rows): entry p of
// row i names neighbour j, and position p of A^T holds the mirrored entry (j, i) with value a_ji.  Both sums of
// the backward then run over the same neighbours, and x_j and g_j are gathered once for both:
//   dX_i = sum_j (dz_ij + dz_ji) x_j + a_ji s g_j,   dz_ij = a_ij <g_i, x_j> f'(z),  dz_ji = a_ji <g_j, x_i> f'(z),
// z = <x_i, x_j> being the same for (i, j) and (j, i).  Two gathered rows per entry instead of three, one sweep
// over the index arrays instead of two.
struct g_args22 { const float* src[2]; int64_t lds_[2]; const float* rowop[2]; int64_t ldr[2]; float* out_entry; int op; const float* val2; };

template <int OP>
struct g_bwd_mirror {  // gathered x_j and g_j, row operands x_i and g_i
  static constexpr int NSRC = 2, NROW = 2, STEPS = 2;
  static constexpr bool PER_ENTRY = false, ACCUMULATE = false, HAS_VAL2 = true;
  using args = g_args22;
  template <int LPG, int W>
  __device__ static inline void edge(const args&, float a, float at, const float (&x)[2][W], const float (&r)[2][W],
                                     float (&acc)[W], const lane_cols<W / 4>& lc, bool live) {
    float sg = 1.f, dsg = 0.f, gd_ij = 0.f, gd_ji = 0.f;
    if (OP != ISP_OP_ONE) {
      edge_fn(OP, group_allreduce<LPG>(dotw<W>(r[0], x[0], lc)), sg, dsg);
      gd_ij = group_allreduce<LPG>(dotw<W>(r[1], x[0], lc));  // <g_i, x_j>
      gd_ji = group_allreduce<LPG>(dotw<W>(x[1], r[0], lc));  // <g_j, x_i>
    }
    const float w = at * sg;
    const float dz = (a * gd_ij + at * gd_ji) * dsg;
    if (live) {
#pragma unroll
      for (int v = 0; v < W; ++v) acc[v] = fmaf(w, x[1][v], fmaf(dz, x[0][v], acc[v]));
    }
  }
};

template <class P, int LPG, int W, bool ADDR32>
__global__ void __launch_bounds__(ISP_WG) k_fused_grouped(isp_view A, const int64_t* __restrict__ indptr,
                                                          const int32_t* __restrict__ indices,
                                                          const float* __restrict__ values, typename P::args pa, int d,
                                                          float* __restrict__ Y, int64_t ldy) {
  __shared__ gs_lds lds;
  fused_grouped_item<P, LPG, W, ADDR32>(A, indptr, indices, values, pa, d, Y, ldy, lds);
}

// LPG lanes with W floats each span the feature width: W * LPG >= d.
template <class P, int LPG, int W>
isp_status run_grouped(const isp_csr* A, const typename P::args& pa, int d, float* Y, int64_t ldy, hipStream_t s) {
  const isp_view& v = A->v;
  const int n_items = v.n_blocks + v.n_seg;
  if (n_items > 0) {
    const unsigned grid = (unsigned)((n_items + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG);
    bool a32 = true;
    for (int k = 0; k < P::NSRC; ++k) a32 = a32 && fused_offsets_fit_32(v.n_cols, pa.lds_[k], d);
    if (a32) k_fused_grouped<P, LPG, W, true><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, pa, d, Y, ldy);
    else k_fused_grouped<P, LPG, W, false><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, v.values, pa, d, Y, ldy);
    ISP_LAUNCH_CHECK();
  }
  if (v.n_hub > 0) {
    const unsigned grid = (unsigned)((v.n_hub + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG);
    k_fused_fixup<4, 1, P::ACCUMULATE><<<grid, ISP_WG, 0, s>>>(v, d, Y, ldy);
    ISP_LAUNCH_CHECK();
  }
  return ISP_OK;
}

// One or two float4 per lane.  Two halve the lanes per dot product, so a step covers twice the entries with one
// lane-reduction stage and one evaluation of the edge function less per entry, and a step costs more
// instructions: it pays where steps are full.  Measured on the benchmark graphs at widths 48 .. 256: two above
// 64 columns; up to 64 columns one, except in the forward pass (one gathered row, the fewest instructions per
// step) on graphs whose non-empty rows average 24 entries or more.  ISP_FUSED_W=4 / 8 forces either (d > 32).
template <class P>
isp_status run_grouped_d(const isp_csr* A, const typename P::args& pa, int d, float* Y, int64_t ldy, hipStream_t s) {
  if (d <= 32) return run_grouped<P, 8, 4>(A, pa, d, Y, ldy, s);
  const int64_t live_rows = A->info.n_rows - A->info.bin_rows[0];
  const bool long_rows = live_rows > 0 && A->info.nnz >= 24 * live_rows;
  const bool fwd = P::NSRC + P::NROW == 2;
  const bool two = A->tune.fused_w ? A->tune.fused_w == 8 : (d > 64 || (fwd && long_rows));
  if (!two) {
    if (d <= 64) return run_grouped<P, 16, 4>(A, pa, d, Y, ldy, s);
    if (d <= 128) return run_grouped<P, 32, 4>(A, pa, d, Y, ldy, s);
    return run_grouped<P, 64, 4>(A, pa, d, Y, ldy, s);
  }
  if (d <= 64) return run_grouped<P, 8, 8>(A, pa, d, Y, ldy, s);
  if (d <= 128) return run_grouped<P, 16, 8>(A, pa, d, Y, ldy, s);
  return run_grouped<P, 32, 8>(A, pa, d, Y, ldy, s);
}

// Column groups (of 256) a hub segment may store per launch of a wide pass: as many as the partial-row scratch
// holds for all segments at once (the scratch is sized for the worst-case segment count, usually several times
// the actual one), at least one.  ISP_WIDE_GROUPS (read at build) caps it, for tests.
int groups_per_launch(const isp_csr* A, int n_groups) {
  int64_t gc = A->v.n_seg > 0 ? A->partial_rows / A->v.n_seg : n_groups;
  if (A->tune.wide_groups > 0 && gc > A->tune.wide_groups) gc = A->tune.wide_groups;
  return gc < 1 ? 1 : (gc > n_groups ? n_groups : (int)gc);
}

bool grouped_partition_ok(const isp_csr* A) {
  return A->info.block_cost <= GS_MAX_ROWS && A->info.block_cost + A->v.hub_t <= GS_MAX_ENT &&
         A->v.seg_len <= GS_MAX_ENT && !A->tune.no_grouped;
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// 0: float4 lanes, 1: float2 lanes, 2..4: scalar lanes with 1, 2, 4 column groups
int pick_shape(int d, bool ok4, bool ok2) {
  if (d > 2 * ISP_WAVE && d % 4 == 0 && ok4) return 0;
  if (d > ISP_WAVE && d <= 2 * ISP_WAVE && d % 2 == 0 && ok2) return 1;
  if (d <= ISP_WAVE) return 2;
  if (d <= 2 * ISP_WAVE) return 3;
  return 4;
}

#define ISP_SHAPE_SWITCH(shape, has_val, CALL)                                   \
  switch (shape) {                                                              \
    case 0: if (has_val) { CALL(4, 1, true); } else { CALL(4, 1, false); } break; \
    case 1: if (has_val) { CALL(2, 1, true); } else { CALL(2, 1, false); } break; \
    case 2: if (has_val) { CALL(1, 1, true); } else { CALL(1, 1, false); } break; \
    case 3: if (has_val) { CALL(1, 2, true); } else { CALL(1, 2, false); } break; \
    default: if (has_val) { CALL(1, 4, true); } else { CALL(1, 4, false); } break; \
  }

}  // namespace

isp_status isp_fusedmm_launch(const isp_csr* A, const float* X, int64_t ldx, int32_t d, int op, float* Y,
                              int64_t ldy, hipStream_t s) {
  const bool ok4 = ldx % 4 == 0 && ldy % 4 == 0 && aligned(X, 16) && aligned(Y, 16);
  const bool ok2 = ldx % 2 == 0 && ldy % 2 == 0 && aligned(X, 8) && aligned(Y, 8);
  if (ok4 && d % 4 == 0 && d <= ISP_PARTIAL_TILE && grouped_partition_ok(A)) {
    g_args1 pa{{X}, {ldx}, {X}, {ldx}, nullptr, op};
    if (op == ISP_OP_SIGMOID) return run_grouped_d<g_fwd<ISP_OP_SIGMOID>>(A, pa, d, Y, ldy, s);
    if (op == ISP_OP_DOT) return run_grouped_d<g_fwd<ISP_OP_DOT>>(A, pa, d, Y, ldy, s);
    return run_grouped_d<g_fwd<ISP_OP_ONE>>(A, pa, d, Y, ldy, s);
  }
  const bool hv = A->v.values != nullptr;
  isp_status st = ISP_OK;
  if (d > ISP_PARTIAL_TILE) {
    // wider than a hub partial row: whole rows in the arithmetic (the score needs them), 256 columns stored
    // per launch (the caller has checked d <= 1024)
    if (!(ok4 && d % 4 == 0))
      return isp_fail(ISP_EUNSUPPORTED, "FusedMM with d > %d needs d %% 4 == 0 and 16-byte aligned rows", ISP_PARTIAL_TILE);
    const int n_groups = (d + ISP_PARTIAL_TILE - 1) / ISP_PARTIAL_TILE;
    const int gc = groups_per_launch(A, n_groups);
    for (int w = 0; w < n_groups && st == ISP_OK; w += gc) {
      const int cnt = n_groups - w < gc ? n_groups - w : gc;
#define ISP_WIDE(T, HV)                             \
  {                                                 \
    using P = fwd_policy<4, T, HV>;                 \
    P::args pa;                                     \
    pa.src[0] = X;                                  \
    pa.ld[0] = ldx;                                 \
    pa.op = op;                                     \
    st = run_pass<P>(A, pa, d, Y, ldy, s, w, cnt);  \
  }
      if (n_groups <= 2) { if (hv) ISP_WIDE(2, true) else ISP_WIDE(2, false) }
      else { if (hv) ISP_WIDE(4, true) else ISP_WIDE(4, false) }
#undef ISP_WIDE
    }
    return st;
  }
  const int shape = pick_shape(d, ok4, ok2);
#define ISP_FWD(V, T, HV)                         \
  {                                               \
    using P = fwd_policy<V, T, HV>;               \
    P::args pa;                                   \
    pa.src[0] = X;                                \
    pa.ld[0] = ldx;                               \
    pa.op = op;                                   \
    st = run_pass<P>(A, pa, d, Y, ldy, s);        \
  }
  ISP_SHAPE_SWITCH(shape, hv, ISP_FWD)
#undef ISP_FWD
  return st;
}

isp_status isp_fusedmm_bwd_launch(const isp_csr* A, const float* X, int64_t ldx, const float* G, int64_t ldg,
                                  int32_t d, int op, float* dX, int64_t lddx, hipStream_t s) {
  const bool ok4 = ldx % 4 == 0 && ldg % 4 == 0 && lddx % 4 == 0 && aligned(X, 16) && aligned(G, 16) && aligned(dX, 16);
  const bool ok2 = ldx % 2 == 0 && ldg % 2 == 0 && lddx % 2 == 0 && aligned(X, 8) && aligned(G, 8) && aligned(dX, 8);
  if (ok4 && d % 4 == 0 && d <= ISP_PARTIAL_TILE && grouped_partition_ok(A) && A->mirror_aligned && !A->tune.no_mirror) {
    // symmetric pattern: one pass over A serves both sums (the mirrored entries' values are A^T's)
    g_args22 pm{{X, G}, {ldx, ldg}, {X, G}, {ldx, ldg}, nullptr, op, A->At->v.values};
    if (op == ISP_OP_SIGMOID) return run_grouped_d<g_bwd_mirror<ISP_OP_SIGMOID>>(A, pm, d, dX, lddx, s);
    if (op == ISP_OP_DOT) return run_grouped_d<g_bwd_mirror<ISP_OP_DOT>>(A, pm, d, dX, lddx, s);
    return run_grouped_d<g_bwd_mirror<ISP_OP_ONE>>(A, pm, d, dX, lddx, s);
  }
  if (ok4 && d % 4 == 0 && d <= ISP_PARTIAL_TILE && grouped_partition_ok(A) && grouped_partition_ok(A->At)) {
    g_args12 p1{{X}, {ldx}, {X, G}, {ldx, ldg}, nullptr, op};
    g_args21 p2{{X, G}, {ldx, ldg}, {X}, {ldx}, nullptr, op};
    isp_status st1;
    if (op == ISP_OP_SIGMOID) {
      st1 = run_grouped_d<g_bwd_row<ISP_OP_SIGMOID>>(A, p1, d, dX, lddx, s);
      return st1 != ISP_OK ? st1 : run_grouped_d<g_bwd_col<ISP_OP_SIGMOID>>(A->At, p2, d, dX, lddx, s);
    }
    if (op == ISP_OP_DOT) {
      st1 = run_grouped_d<g_bwd_row<ISP_OP_DOT>>(A, p1, d, dX, lddx, s);
      return st1 != ISP_OK ? st1 : run_grouped_d<g_bwd_col<ISP_OP_DOT>>(A->At, p2, d, dX, lddx, s);
    }
    st1 = run_grouped_d<g_bwd_row<ISP_OP_ONE>>(A, p1, d, dX, lddx, s);
    return st1 != ISP_OK ? st1 : run_grouped_d<g_bwd_col<ISP_OP_ONE>>(A->At, p2, d, dX, lddx, s);
  }
  const bool hv = A->v.values != nullptr;
  isp_status st = ISP_OK;
  if (d > ISP_PARTIAL_TILE) {  // as in the forward: whole rows in the arithmetic, one column group stored per launch
    if (!(ok4 && d % 4 == 0))
      return isp_fail(ISP_EUNSUPPORTED, "FusedMM with d > %d needs d %% 4 == 0 and 16-byte aligned rows", ISP_PARTIAL_TILE);
    const int n_groups = (d + ISP_PARTIAL_TILE - 1) / ISP_PARTIAL_TILE;
    // every row pass before the first column pass: the column pass of group 0 already adds to all columns of
    // the rows that are not hubs of A^T, which a later row pass's fix-up must not overwrite
#define ISP_WIDE_ROW(T, HV)                                              \
  {                                                                      \
    using P1 = bwd_row_policy<4, T, HV>;                                 \
    P1::args p1;                                                         \
    p1.src[0] = X; p1.ld[0] = ldx; p1.G = G; p1.ldg = ldg; p1.op = op;   \
    st = run_pass<P1>(A, p1, d, dX, lddx, s, w, cnt);                    \
  }
#define ISP_WIDE_COL(T, HV)                                              \
  {                                                                      \
    using P2 = bwd_col_policy<4, T, HV>;                                 \
    P2::args p2;                                                         \
    p2.src[0] = X; p2.ld[0] = ldx; p2.src[1] = G; p2.ld[1] = ldg; p2.op = op; \
    st = run_pass<P2>(A->At, p2, d, dX, lddx, s, w, cnt);                \
  }
    const int gc1 = groups_per_launch(A, n_groups), gc2 = groups_per_launch(A->At, n_groups);
    for (int w = 0; w < n_groups && st == ISP_OK; w += gc1) {
      const int cnt = n_groups - w < gc1 ? n_groups - w : gc1;
      if (n_groups <= 2) { if (hv) ISP_WIDE_ROW(2, true) else ISP_WIDE_ROW(2, false) }
      else { if (hv) ISP_WIDE_ROW(4, true) else ISP_WIDE_ROW(4, false) }
    }
    for (int w = 0; w < n_groups && st == ISP_OK; w += gc2) {
      const int cnt = n_groups - w < gc2 ? n_groups - w : gc2;
      if (n_groups <= 2) { if (hv) ISP_WIDE_COL(2, true) else ISP_WIDE_COL(2, false) }
      else { if (hv) ISP_WIDE_COL(4, true) else ISP_WIDE_COL(4, false) }
    }
#undef ISP_WIDE_ROW
#undef ISP_WIDE_COL
    return st;
  }
  const int shape = pick_shape(d, ok4, ok2);
#define ISP_BWD(V, T, HV)                                  \
  {                                                        \
    using P1 = bwd_row_policy<V, T, HV>;                   \
    P1::args p1;                                           \
    p1.src[0] = X; p1.ld[0] = ldx; p1.G = G; p1.ldg = ldg; p1.op = op; \
    st = run_pass<P1>(A, p1, d, dX, lddx, s);              \
    if (st == ISP_OK) {                                    \
      using P2 = bwd_col_policy<V, T, HV>;                 \
      P2::args p2;                                         \
      p2.src[0] = X; p2.ld[0] = ldx; p2.src[1] = G; p2.ld[1] = ldg; p2.op = op; \
      st = run_pass<P2>(A->At, p2, d, dX, lddx, s);        \
    }                                                      \
  }
  ISP_SHAPE_SWITCH(shape, hv, ISP_BWD)
#undef ISP_BWD
  return st;
}
