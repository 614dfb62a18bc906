// SpMM, sum reduction: Y = A X with A in CSR and X dense row-major (paper: abstract, Sections 1,
// 3.4, 3.5).  The backward dX = A^T dY is this same code run on the cached transpose's handle
// (Section 3.3).  Gather-bound: per nonzero one 4*d-byte row of X is fetched and d FMAs are done,
// so the kernels are built around coalesced row gathers, not around matrix cores.
#include "group_stream.h"

namespace {
using namespace isp_dev;

template <int VEC_, int T_, bool HAS_VAL_>
struct spmm_policy {
  static constexpr int VEC = VEC_, T = T_, NG = 1;
  static constexpr int U = (VEC * T >= 4) ? 4 : 8;
  static constexpr bool HAS_VAL = HAS_VAL_, ACCUMULATE = false, NEEDS_PERM = false, HAS_FINISH = false;
  struct args { const float* src[1]; int64_t ld[1]; };
  struct row_state {};
  __device__ static inline void row_begin(const args&, row_state&, int, const int (&)[T], const bool (&)[T]) {}
  __device__ static inline void edge(const args&, row_state&, float a, const float (&x)[1][T][VEC],
                                     float (&acc)[T][VEC], const bool (&)[T], const edge_info&) {
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

// One workgroup per hub row.
template <int VEC, int T>
__global__ void __launch_bounds__(ISP_WG) k_spmm_fixup(isp_view A, int d, int k0, float* __restrict__ Y, int64_t ldy) {
  hub_fixup_wg<VEC, T, false>(A, d, k0, Y, ldy);
}

// Mean reduction: the fixed-order sum of a hub row's segments, divided by the row's length.
__global__ void __launch_bounds__(ISP_WG) k_spmm_fixup_mean(isp_view A, int d, int k0, float* __restrict__ Y,
                                                            int64_t ldy) {
  hub_fixup_wg<4, 1, true>(A, d, k0, Y, ldy);
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
    k_spmm_fixup<VEC, T><<<(unsigned)v.n_hub, ISP_WG, 0, s>>>(v, d, k0, Y, ldy);
    ISP_LAUNCH_CHECK();
  }
  return ISP_OK;
}


// ---- grouped fast path -------------------------------------------------------------------------
// LPG lanes x float4 cover one slice of 4 * LPG feature columns; G = 64 / LPG nonzeros per gather
// instruction.  Slice s of tile k_base covers columns [k_base + s * 4 * LPG, +4 * LPG).
// ADDR32: every byte offset into X fits 32 bits and both factors of column * row-pitch fit 24 bits, so
// the gather address is one full-rate 24-bit multiply-add on top of a scalar base pointer.
// SPARSE_ROWS: empty rows own no step (their output is zeroed up front and a list of the item's non-empty
// rows says where each row end belongs); chosen for matrices in which many rows are empty.
template <int LPG, bool HAS_VAL, bool ADDR32, int VEC = 4, bool SPARSE_ROWS = false>
__global__ void __launch_bounds__(ISP_WG) __attribute__((amdgpu_waves_per_eu(4, 4))) k_spmm_grouped(isp_view A, const int64_t* __restrict__ indptr,
                                                         const int32_t* __restrict__ indices,
                                                         const float* __restrict__ values,
                                                         const float* __restrict__ X, int64_t ldx, int d, int k_base,
                                                         int n_slices, float* __restrict__ Y, int64_t ldy, int mean_mode) {
  // mean_mode 1: divide every finished row by its length (mean reduction, forward)
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
  const int col = k_base + (slice * LPG + q) * VEC;
  const bool lane_on = col < d;
  // lanes without a live entry (row tails, null steps, columns past d) still issue their gather -
  // from row 0 of X - so that every step is exactly one load per lane (exact wait counts, no
  // branches around loads); what they fetch is never used
  const float* __restrict__ xcol = lane_on ? X + col : X;
  const unsigned lane_byte = lane_on ? (unsigned)col * 4u : 0u;
  const unsigned pitch_byte = (unsigned)ldx * 4u;
  // Rows of a derived matrix (packed layout) beyond the real ones are pieces of long rows: like a hub segment
  // each adds into a partial row, named by piece_slot.  A block never mixes real rows and pieces.
  const bool pieces = !it.is_seg && (int64_t)it.row >= A.n_real_rows;
  const bool to_partial = it.is_seg || pieces;
  const int32_t* __restrict__ slot_of = A.piece_slot - (pieces ? A.n_real_rows : 0);  // indexed by the piece's row
  // The block's partial-row numbers are fetched up front, one per lane (a block holds at most 129 pieces: each
  // costs at least 2 of the 256 units), so that a row end does not wait for a load of its own.
  int slot_lo = 0, slot_hi = 0;
  if (pieces) {
    const int n_pc = it.row_last - it.row;
    if (lane < n_pc) slot_lo = slot_of[it.row + lane];
    if (lane + ISP_WAVE < n_pc) slot_hi = slot_of[it.row + lane + ISP_WAVE];
  }
  float* __restrict__ out = to_partial ? A.partials + (col - k_base) : Y + col;
  const int64_t ldo = to_partial ? (int64_t)ISP_PARTIAL_TILE : ldy;
  float acc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
  const bool listed = SPARSE_ROWS && !it.is_seg;  // else every row owns a step and the k-th row end is row k's
  if (listed && lane_on && !pieces) {  // the empty rows' outputs (also their mean); a piece is never empty
    const int n_empty = it.row_last - it.row - n_live;  // they are listed behind the non-empty rows
    for (int i = g; i < n_empty; i += G) store_vec<VEC>(out + (int64_t)(it.row + (int)L.ss[n_live + 1 + i]) * ldo, acc);
  }
  // local index of the row the next row end belongs to; with the list it is read one row ahead so that a
  // row's store does not wait for it (the list ends with a spare entry)
  int k_done = 0;
  int r_next = listed ? (int)L.ss[0] : 0;

  auto finish_row = [&]() {
    const int r_local = __builtin_amdgcn_readfirstlane(r_next);  // (wave-uniform: scalar address math)
    int row = it.row + r_local;
    if (pieces) {  // the piece's partial row: from the lanes that fetched it, beyond 128 pieces by a load
      if (r_local < ISP_WAVE) row = __builtin_amdgcn_readlane(slot_lo, r_local);
      else if (r_local < 2 * ISP_WAVE) row = __builtin_amdgcn_readlane(slot_hi, r_local - ISP_WAVE);
      else row = __builtin_amdgcn_readfirstlane(slot_of[row]);
    }
    ++k_done;
    r_next = listed ? (int)L.ss[k_done] : k_done;
    // the groups' sums, spread over the groups: this lane ends up with R finished columns starting at its idx0-th
    constexpr int R = VEC / G > 0 ? VEC / G : 1;
    const int idx0 = group_reduce_scatter<LPG, VEC>(acc, lane);
    if (group_owner<LPG, VEC>(lane) && lane_on) {
      float t[R];
#pragma unroll
      for (int c = 0; c < R; ++c) t[c] = acc[c];
      if (mean_mode == 1 && !to_partial) {  // segments and pieces keep plain partial sums; their fix-up divides
        const int len = (int)L.rp[r_local + 1] - (int)L.rp[r_local];
        const float inv = len > 0 ? 1.f / (float)len : 0.f;
#pragma unroll
        for (int c = 0; c < R; ++c) t[c] *= inv;
      }
      store_vec<R>(out + (int64_t)row * ldo + idx0, t);
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
  };
  // descriptors of U consecutive steps = one 16-byte LDS read
  auto issue = [&](int s0, unsigned (&dsc)[U], float (&x)[U][VEC], float (&a)[U]) {
    const uint4 pk = *reinterpret_cast<const uint4*>(L.step + s0);
    // the table is the same in every lane: held in scalar registers, a step's offset, count and row-end flag
    // cost no vector instructions
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
      const int cj = act ? e[u].x : 0;
      if constexpr (ADDR32) {
        const unsigned off = __umul24((unsigned)cj, pitch_byte) + lane_byte;
        load_vec<VEC>(reinterpret_cast<const float*>(reinterpret_cast<const char*>(X) + off), x[u]);
      } else {
        load_vec<VEC>(xcol + (int64_t)cj * ldx, x[u]);
      }
    }
  };
  auto consume = [&](const unsigned (&dsc)[U], const float (&x)[U][VEC], const float (&a)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (g < gs_cnt(dsc[u]) && lane_on) {  // divergent on purpose: dead lanes skip the FMAs, nothing to zero
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = fmaf(a[u], x[u][v], acc[v]);
      }
      if (dsc[u] & GS_LAST) finish_row();
    }
  };

  const int n_groups = n_steps / U;
  if (n_groups == 0) return;
  unsigned dA[U], dB[U];
  float xA[U][VEC], xB[U][VEC], aA[U], aB[U];
  issue(0, dA, xA, aA);
  int gi = 0;
  while (gi + 2 < n_groups) {  // steady state: the next group's gathers are in flight while one is consumed
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

template <int LPG, int VEC = 4>
isp_status launch_grouped(const isp_csr* A, const float* X, int64_t ldx, int d, int k_base, int n_slices, float* Y,
                          int64_t ldy, int mean_mode, const float* values_override, hipStream_t s,
                          const float* values_override_packed = nullptr) {
  // The packed layout (a derived matrix in which the pieces of long rows share work items) when the handle has
  // one; an override of the values is in the order of A's own entries and therefore runs on A's own partition.
  const bool packed = A->has_packed && (!values_override || values_override_packed) &&
                      A->packed_block_cost + A->vp.hub_t <= GS_MAX_ENT &&
                      A->packed_block_cost / A->packed_row_cost <= GS_MAX_ROWS;
  const isp_view& v = packed ? A->vp : A->v;
  // (one value per stored entry, in the order of the view's entries)
  const float* vals = values_override ? (packed ? values_override_packed : values_override) : v.values;
  const int n_items = v.n_blocks + v.n_seg;
  if (n_items > 0) {
    const unsigned grid = (unsigned)((n_items + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG) * (unsigned)n_slices;
    const bool a32 = v.n_cols < (1 << 24) && ldx * 4 < (1 << 24) &&
                     ((uint64_t)v.n_cols * (uint64_t)ldx + (uint64_t)d) * 4u < ((uint64_t)1 << 32);
    // the list of non-empty rows pays once a fair share of the rows is empty (directed graphs)
    const bool sparse_rows = A->info.bin_rows[0] * 16 > A->info.n_rows;
#define ISP_GO(HV, A32)                                                                                           \
  do {                                                                                                            \
    if (sparse_rows)                                                                                              \
      k_spmm_grouped<LPG, HV, A32, VEC, true><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, vals, X, ldx, d,     \
                                                                    k_base, n_slices, Y, ldy, mean_mode);          \
    else                                                                                                          \
      k_spmm_grouped<LPG, HV, A32, VEC, false><<<grid, ISP_WG, 0, s>>>(v, v.indptr, v.indices, vals, X, ldx, d,    \
                                                                     k_base, n_slices, Y, ldy, mean_mode);         \
  } while (0)
    if constexpr (VEC < 4) {  // narrow lanes are only dispatched with 32-bit addressing
      if (vals) ISP_GO(true, true); else ISP_GO(false, true);
    } else {
      if (vals) { if (a32) ISP_GO(true, true); else ISP_GO(true, false); }
      else { if (a32) ISP_GO(false, true); else ISP_GO(false, false); }
    }
#undef ISP_GO
    ISP_LAUNCH_CHECK();
  }
  if (v.n_hub > 0) {
    // the columns this launch covered: [k_base, min(d, k_base + n_slices * LPG * VEC))
    const int d_hi = (k_base + n_slices * LPG * VEC < d) ? k_base + n_slices * LPG * VEC : d;
    if (mean_mode == 1) k_spmm_fixup_mean<<<(unsigned)v.n_hub, ISP_WG, 0, s>>>(v, d_hi, k_base, Y, ldy);  // VEC = 4 only
    else k_spmm_fixup<VEC, 4 / VEC><<<(unsigned)v.n_hub, ISP_WG, 0, s>>>(v, d_hi, k_base, Y, ldy);
    ISP_LAUNCH_CHECK();
  }
  return ISP_OK;
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

}  // namespace

// The grouped fast path; *done = false (and nothing launched) when the operands do not qualify.
// mean_mode: see k_spmm_grouped.  values_override (optional): nnz values, in A's entry order, used in place of
// A's own (the backward of the mean reduction passes the transpose's values divided by the source rows' lengths).
isp_status isp_spmm_grouped_launch(const isp_csr* A, const float* X, int64_t ldx, int32_t d, float* Y, int64_t ldy,
                                   int mean_mode, const float* values_override, hipStream_t s, bool* done,
                                   const float* values_override_packed) {
  const isp_view& av = A->v;
  // Lane width: float4 when width, pitch and pointers allow; float2 / float lanes otherwise (any d),
  // those two only with 32-bit addressing and for the plain sum.
  int vec = 1;
  if (d % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && aligned(X, 16) && aligned(Y, 16)) vec = 4;
  else if (d % 2 == 0 && ldx % 2 == 0 && ldy % 2 == 0 && aligned(X, 8) && aligned(Y, 8)) vec = 2;
  const bool a32 = av.n_cols < (1 << 24) && ldx * 4 < (1 << 24) &&
                   ((uint64_t)av.n_cols * (uint64_t)ldx + (uint64_t)d) * 4u < ((uint64_t)1 << 32);
  // (a matrix without entries never reads X, which may then be absent: the generic path handles it)
  const bool grouped_ok = av.nnz > 0 && (vec == 4 || (a32 && mean_mode == 0)) && A->info.block_cost <= GS_MAX_ROWS &&
                          A->info.block_cost + av.hub_t <= GS_MAX_ENT && av.seg_len <= GS_MAX_ENT &&
                          !A->tune.no_grouped;
  *done = grouped_ok;
  if (!grouped_ok) return ISP_OK;
  if (vec < 4) {
    // narrow lanes: the smallest group that covers the row, at most 64 * vec columns per slice
    isp_status st = ISP_OK;
    for (int k_base = 0; k_base < d && st == ISP_OK; k_base += ISP_PARTIAL_TILE) {
      const int w = (d - k_base < ISP_PARTIAL_TILE) ? d - k_base : ISP_PARTIAL_TILE;
      const int lpg = w <= 16 * vec ? 16 : (w <= 32 * vec ? 32 : 64);
      const int ns = (w + lpg * vec - 1) / (lpg * vec);
      if (vec == 2) {
        if (lpg == 16) st = launch_grouped<16, 2>(A, X, ldx, d, k_base, ns, Y, ldy, 0, values_override, s, values_override_packed);
        else if (lpg == 32) st = launch_grouped<32, 2>(A, X, ldx, d, k_base, ns, Y, ldy, 0, values_override, s, values_override_packed);
        else st = launch_grouped<64, 2>(A, X, ldx, d, k_base, ns, Y, ldy, 0, values_override, s, values_override_packed);
      } else {
        if (lpg == 16) st = launch_grouped<16, 1>(A, X, ldx, d, k_base, ns, Y, ldy, 0, values_override, s, values_override_packed);
        else if (lpg == 32) st = launch_grouped<32, 1>(A, X, ldx, d, k_base, ns, Y, ldy, 0, values_override, s, values_override_packed);
        else st = launch_grouped<64, 1>(A, X, ldx, d, k_base, ns, Y, ldy, 0, values_override, s, values_override_packed);
      }
    }
    return st;
  }
  // float4 lanes: 4 / 8 / 16 / 32 / 64 lanes per group <-> column slices of 16 / 32 / 64 / 128 / 256 floats.
  // Measured on R-MAT graphs (2.4 M and 124 M nonzeros, d = 8..256): the slice that just covers
  // the row wins up to d = 128; on large graphs with many columns two 64-float slices per 128-float
  // row win (dealt to alternating XCDs, each L2 then keeps half-rows of twice as many hot columns,
  // which outweighs staging the CSR arrays twice) provided both halves are whole 128-byte lines.  With
  // few columns (233 k measured) a column band's hot rows fit an L2 whole and one slice is faster.
  // ISP_SPMM_LPG / ISP_SPMM_TILE (read when the handle was built) override the choices for tuning.
  const bool big = av.nnz >= (int64_t)8 << 20;
  const bool large = big && av.n_cols >= (1 << 19);
  int lpg = d <= 32 ? 8 : (d <= 64 ? 16 : 32);
  // columns per launch: rows wider than 128 floats are covered 128 columns at a time on the big graphs
  // (233 k columns, d = 256: 5.7 vs 6.0 ms; 2.4 M columns: 10.8 vs 12.1 ms)
  const int tile_dflt = big ? 128 : ISP_PARTIAL_TILE;
  int tile = tile_dflt;
  if (large && d > 64 && d % 64 == 0 && ldx % 32 == 0) lpg = 16;  // (rows start on 128-byte lines)
  if (A->tune.spmm_lpg) lpg = A->tune.spmm_lpg;
  isp_status st = ISP_OK;
  if (A->tune.spmm_tile) tile = A->tune.spmm_tile;
  for (int k_base = 0; k_base < d && st == ISP_OK; k_base += tile) {
    const int w = (d - k_base < tile) ? d - k_base : tile;
    const int ns = (w + 4 * lpg - 1) / (4 * lpg);
    switch (lpg) {
      case 4: st = launch_grouped<4>(A, X, ldx, d, k_base, ns, Y, ldy, mean_mode, values_override, s, values_override_packed); break;
      case 8: st = launch_grouped<8>(A, X, ldx, d, k_base, ns, Y, ldy, mean_mode, values_override, s, values_override_packed); break;
      case 16: st = launch_grouped<16>(A, X, ldx, d, k_base, ns, Y, ldy, mean_mode, values_override, s, values_override_packed); break;
      case 32: st = launch_grouped<32>(A, X, ldx, d, k_base, ns, Y, ldy, mean_mode, values_override, s, values_override_packed); break;
      default: st = launch_grouped<64>(A, X, ldx, d, k_base, ns, Y, ldy, mean_mode, values_override, s, values_override_packed); break;
    }
  }
  return st;
}

isp_status isp_spmm_launch(const isp_csr* A, const float* X, int64_t ldx, int32_t d, float* Y, int64_t ldy,
                           hipStream_t s) {
  bool done = false;
  isp_status st0 = isp_spmm_grouped_launch(A, X, ldx, d, Y, ldy, 0, nullptr, s, &done);
  if (done || st0 != ISP_OK) return st0;
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
