// Grouped kernels for the operations that need a whole dot product per nonzero (SDDMM and the
// FusedMM passes).  Same work items, LDS staging and step tables as the grouped SpMM; here a
// group of LPG lanes spans the full feature width (W * LPG >= d with W = 4 or 8 floats per lane, as one
// or two float4), so G = 64 / LPG dot products are reduced side by side with the same DPP
// instructions.  Two float4 per lane halve the lanes per dot product: a step covers twice the entries,
// with one lane-reduction stage and one evaluation of the edge function less per entry - these kernels
// keep the vector ALU busy 55 - 70 % of the time, so instructions per entry count.  In row blocks the row operand (U's row
// for SDDMM, x_i / g_i for FusedMM) is re-read with every step instead of being kept across steps: it
// is an L1 hit after a row's first step and keeps the main loop free of row-change stalls; a hub
// segment, which is one row throughout, loads it once.
#pragma once
#include <type_traits>
#include "group_stream.h"

namespace isp_dev {

// Policy P:  NSRC gathered operands (rows picked by column index), NROW row operands (rows picked
// by the step's matrix row); STEPS steps issued back to back per buffer (two buffers in flight);
// args { src[NSRC], lds_[NSRC], rowop[NROW], ldr[NROW], out_entry };
// either edge<LPG>(args, a, src, rowop, acc, lane_on, live) accumulating into the row's result in live
// lanes, or (PER_ENTRY) entry<LPG>(a, src, rowop, lane_on) returning the value stored for the entry.
// A policy with HAS_VAL2 = true also gets a second value per stored entry, args::val2[p] (a parallel array in
// the order of the matrix's entries; null = all ones), as an extra argument of edge().
// ADDR32: every byte offset into the gathered operands fits 32 bits and both factors of column * row pitch
// fit 24 bits (fused_offsets_fit_32 below), so a gather address is one full-rate 24-bit multiply-add on a
// scalar base pointer instead of a 64-bit multiply (three quarter-rate instructions).
// values may be null (every stored value is 1).
// A lane's float4 vectors: whether each lies inside the feature width, and its first column (0 when it does not,
// so that the lane still reads valid memory).
template <int NV>
struct lane_cols {
  bool on[NV];
  int off[NV];
};

template <class P, class = void>
struct policy_has_val2 : std::false_type {};
template <class P>
struct policy_has_val2<P, std::void_t<decltype(P::HAS_VAL2)>> : std::bool_constant<P::HAS_VAL2> {};

template <class P, class = void>
struct policy_sparse_rows : std::bool_constant<!P::PER_ENTRY> {};
template <class P>
struct policy_sparse_rows<P, std::void_t<decltype(P::SPARSE_ROWS)>> : std::bool_constant<P::SPARSE_ROWS> {};

template <class P, int LPG, int W, bool ADDR32>
__device__ inline void fused_grouped_item(const isp_view& A, const int64_t* __restrict__ indptr,
                                          const int32_t* __restrict__ indices, const float* __restrict__ values,
                                          const typename P::args& pa, int d, float* __restrict__ Y, int64_t ldy,
                                          gs_lds& lds, int k_lo = 0) {
  // k_lo: first feature column of this pass (only the per-entry policies run in column windows;
  // their partial dot products are then added up across passes)
  static_assert(W == 4 || W == 8, "one or two float4 per lane");
  constexpr int G = ISP_WAVE / LPG;
  constexpr int NV = W / 4;  // float4 vectors per lane: vector v covers columns [v * 4 * LPG, (v + 1) * 4 * LPG)
  constexpr int NSRC = P::NSRC, NROW = P::NROW;
  // Steps in flight: two buffers of P::STEPS steps with one float4 per lane; with two, a step carries twice the
  // entries and twice the registers, and P::STEPS buffers of one step each keep as many entries in flight.
  constexpr int U = W == 4 ? P::STEPS : 1;
  constexpr int NB = W == 4 ? 2 : P::STEPS;
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  const int w = threadIdx.x >> 6;
  const int item = __builtin_amdgcn_readfirstlane((int)blockIdx.x * ISP_WAVES_PER_WG + w);
  if (item >= A.n_blocks + A.n_seg) return;
  const item_range it = locate_item(A, indptr, item);
  if (it.skip) return;
  gs_wave_lds& L = lds.w[w];
  // The policies with row results skip empty rows altogether (no step; the list of non-empty rows in L.ss
  // says which row the steps between two row ends belong to): directed graphs leave many rows empty (half of
  // them in the FusedMM benchmark graph).  The per-entry policy says which table it wants (SPARSE_ROWS): the
  // list costs one LDS read per step, an empty row's step a whole step.
  constexpr bool sparse_rows = policy_sparse_rows<P>::value;
  constexpr int PAD = W == 4 ? U : NB;  // (the ring of one-step buffers runs whole rounds only)
  int n_live = 0;  // non-empty rows of a row block
  const int n_steps = values ? gs_prepare<G, true, sparse_rows, PAD>(it, indptr, indices, values, L, lane, &n_live)
                             : gs_prepare<G, false, sparse_rows, PAD>(it, indptr, indices, values, L, lane, &n_live);

  const int g = lane / LPG, q = lane % LPG;
  lane_cols<NV> lc;  // this lane's columns: in range?  offset of the first (0 when out of range)
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int col = k_lo + v * 4 * LPG + q * 4;
    lc.on[v] = col < d;
    lc.off[v] = lc.on[v] ? col : 0;
  }
  unsigned src_pitch[NSRC];  // row pitches of the gathered operands in bytes (ADDR32)
#pragma unroll
  for (int k = 0; k < NSRC; ++k) src_pitch[k] = (unsigned)pa.lds_[k] * 4u;
  float* __restrict__ out = it.is_seg ? A.partials : Y;
  const int64_t ldo = it.is_seg ? (int64_t)ISP_PARTIAL_TILE : ldy;
  // An empty row owns no step.  The k-th row end of the step table belongs to the k-th non-empty row of the
  // item, whose local index is L.ss[k] (a hub segment is its one row).
  int k_done = 0;            // row ends consumed
  const bool listed = sparse_rows && !it.is_seg;  // else the k-th row end belongs to row k
  int r_next = listed ? (int)L.ss[0] : 0;      // read one row ahead (the list ends with a spare entry)
  int k_issued = 0;          // row ends passed by the steps issued so far
  float acc[W];
#pragma unroll
  for (int v = 0; v < W; ++v) acc[v] = 0.f;
  auto store_row = [&](int64_t row) {  // this lane's columns of acc to row `row` of the output
    float* o = out + row * ldo;
#pragma unroll
    for (int v = 0; v < NV; ++v)
      if (lc.on[v]) {
        float t[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) t[c] = acc[4 * v + c];
        store_vec<4>(o + lc.off[v], t);
      }
  };
  if (!P::PER_ENTRY && !P::ACCUMULATE && listed) {  // outputs of the empty rows, listed behind the non-empty ones
    const int n_empty = it.row_last - it.row - n_live;
    for (int i = g; i < n_empty; i += G) store_row(it.row + (int)L.ss[n_live + 1 + i]);
  }

  auto finish_row = [&]() {
    const int row = it.row + __builtin_amdgcn_readfirstlane(r_next);  // (wave-uniform: scalar address math)
    ++k_done;
    r_next = listed ? (int)L.ss[k_done] : k_done;
    // the groups' sums, spread over the groups: this lane ends up with R finished columns starting at its idx0-th
    constexpr int R = W / G > 0 ? W / G : 1;
    const int idx0 = group_reduce_scatter<LPG, W>(acc, lane);
    const bool on = NV == 1 ? lc.on[0] : (idx0 >= 4 ? lc.on[NV - 1] : lc.on[0]);
    if (group_owner<LPG, W>(lane) && on) {
      float* o = out + (int64_t)row * ldo + (idx0 >= 4 ? lc.off[NV - 1] + idx0 - 4 : lc.off[0] + idx0);
      float t[R];
#pragma unroll
      for (int c = 0; c < R; ++c) t[c] = acc[c];
      if (P::ACCUMULATE && !it.is_seg) {
        float old[R];
        load_vec<R>(o, old);
#pragma unroll
        for (int c = 0; c < R; ++c) t[c] += old[c];
      }
      store_vec<R>(o, t);
    }
#pragma unroll
    for (int v = 0; v < W; ++v) acc[v] = 0.f;
  };
  auto load_w = [&](const float* p, float (&dst)[W]) {  // this lane's columns of the row that starts at p
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      float t[4];
      load_vec<4>(p + lc.off[v], t);
#pragma unroll
      for (int c = 0; c < 4; ++c) dst[4 * v + c] = t[c];
    }
  };
  // SEG (a hub segment: one matrix row for the whole item): the row operand is loaded once and stays in
  // registers.  Row blocks re-read it with every step, which keeps their loop free of row-change stalls.
  auto run = [&](auto seg_tag) {
    constexpr bool SEG = decltype(seg_tag)::value;
    constexpr int NR = SEG ? 0 : NROW;  // per-step row-operand registers
    float rS[NROW][W];
    if constexpr (SEG) {
#pragma unroll
      for (int k = 0; k < NROW; ++k) load_w(pa.rowop[k] + (int64_t)it.src_row * pa.ldr[k], rS[k]);
    }
    auto issue = [&](int s0, unsigned (&dsc)[U], float (&x)[U][NSRC][W], float (&r)[U][NR + 1][W], float (&a)[U],
                     float (&a2)[U]) {
      int2 e[U];
      int srow[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        dsc[u] = __builtin_amdgcn_readfirstlane((unsigned)L.step[s0 + u]);  // the same in every lane
        e[u] = L.ent[gs_off(dsc[u]) + g];
        // (null steps past the end read the spare 0 after the list, or name the row after the item's last)
        if constexpr (!SEG)
          srow[u] = it.src_row + (sparse_rows ? __builtin_amdgcn_readfirstlane((int)L.ss[k_issued]) : k_issued);
        k_issued += (int)((dsc[u] >> 15) & 1u);  // a row end moves the following steps to the next non-empty row
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool act = g < gs_cnt(dsc[u]);
        a[u] = __int_as_float(e[u].y);
        const int cj = act ? e[u].x : 0;  // dead groups gather row 0; what they fetch is never used
        if constexpr (policy_has_val2<P>::value) {
          // (a dead lane reads the step's first entry, or the item's first one in a null step: valid positions)
          a2[u] = 1.f;
          if (pa.val2) a2[u] = pa.val2[it.p + gs_off(dsc[u]) + (act ? g : 0)];
        }
#pragma unroll
        for (int k = 0; k < NSRC; ++k) {
          if constexpr (ADDR32) {
            const unsigned base = __umul24((unsigned)cj, src_pitch[k]);
#pragma unroll
            for (int v = 0; v < NV; ++v) {
              float t[4];
              load_vec<4>(reinterpret_cast<const float*>(reinterpret_cast<const char*>(pa.src[k]) + (base + (unsigned)lc.off[v] * 4u)), t);
#pragma unroll
              for (int c = 0; c < 4; ++c) x[u][k][4 * v + c] = t[c];
            }
          } else {
            load_w(pa.src[k] + (int64_t)cj * pa.lds_[k], x[u][k]);
          }
        }
        if constexpr (!SEG) {
          const int64_t ri = srow[u] < (int)A.n_rows ? srow[u] : 0;  // null steps after the matrix's last row
#pragma unroll
          for (int k = 0; k < NROW; ++k) load_w(pa.rowop[k] + ri * pa.ldr[k], r[u][k]);
        }
      }
    };
    auto consume = [&](const unsigned (&dsc)[U], const float (&x)[U][NSRC][W], const float (&r)[U][NR + 1][W],
                       const float (&a)[U], const float (&a2)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        // The policies mask the per-lane partial dot products of columns past d and accumulate only in live
        // groups; a lane's columns past d collect sums that are never stored.
        const bool live = g < gs_cnt(dsc[u]);
        float rr[NROW][W];
#pragma unroll
        for (int k = 0; k < NROW; ++k)
#pragma unroll
          for (int v = 0; v < W; ++v) rr[k][v] = SEG ? rS[k][v] : r[u][k < NR ? k : 0][v];
        if constexpr (P::PER_ENTRY) {
          // one output per stored entry, parked in the entry's LDS slot (its value has been read by
          // the step's issue) and written out in one coalesced sweep when the item is done
          const float val = P::template entry<LPG, W>(a[u], x[u], rr, lc);
          if (live && q == 0) L.ent[gs_off(dsc[u]) + g].y = __float_as_int(val);
        } else {
          if constexpr (policy_has_val2<P>::value) P::template edge<LPG, W>(pa, a[u], a2[u], x[u], rr, acc, lc, live);
          else P::template edge<LPG, W>(pa, a[u], x[u], rr, acc, lc, live);
          if (dsc[u] & GS_LAST) finish_row();
        }
      }
    };

    if constexpr (W == 4) {
      const int n_groups = n_steps / U;
      unsigned dA[U], dB[U];
      float xA[U][NSRC][W], xB[U][NSRC][W], rA[U][NR + 1][W], rB[U][NR + 1][W], aA[U], aB[U];
      float a2A[U], a2B[U];  // (unused, and optimised away, unless the policy takes a second value)
      issue(0, dA, xA, rA, aA, a2A);
      int gi = 0;
      while (gi + 2 < n_groups) {
        issue((gi + 1) * U, dB, xB, rB, aB, a2B);
        consume(dA, xA, rA, aA, a2A);
        issue((gi + 2) * U, dA, xA, rA, aA, a2A);
        consume(dB, xB, rB, aB, a2B);
        gi += 2;
      }
      if (gi + 1 < n_groups) {
        issue((gi + 1) * U, dB, xB, rB, aB, a2B);
        consume(dA, xA, rA, aA, a2A);
        consume(dB, xB, rB, aB, a2B);
      } else {
        consume(dA, xA, rA, aA, a2A);
      }
    } else {
      // a ring of NB one-step buffers; n_steps is a multiple of NB, so every round is whole and no issue sits
      // behind a condition
      unsigned dR[NB][U];
      float xR[NB][U][NSRC][W], rR[NB][U][NR + 1][W], aR[NB][U], a2R[NB][U];
#pragma unroll
      for (int b = 0; b < NB; ++b) issue(b, dR[b], xR[b], rR[b], aR[b], a2R[b]);
      for (int s0 = NB; s0 < n_steps; s0 += NB) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          consume(dR[b], xR[b], rR[b], aR[b], a2R[b]);
          issue(s0 + b, dR[b], xR[b], rR[b], aR[b], a2R[b]);
        }
      }
#pragma unroll
      for (int b = 0; b < NB; ++b) consume(dR[b], xR[b], rR[b], aR[b], a2R[b]);
    }
  };
  if (n_steps == 0) return;
  if (it.is_seg) run(std::true_type{}); else run(std::false_type{});
  if constexpr (P::PER_ENTRY) {
    wave_lds_sync();
    const int n_ent = (int)(it.p_end - it.p);
    for (int i = lane; i < n_ent; i += ISP_WAVE) {
      float* o = pa.out_entry + it.p + i;
      const float val = __int_as_float(L.ent[i].y);
      *o = P::ADD ? *o + val : val;
    }
  }
}

// Host side: true when a kernel over matrix columns [0, n_cols) may gather from rows of pitch ld floats
// (d columns used) with 32-bit byte offsets formed by a 24-bit multiply.
inline bool fused_offsets_fit_32(int64_t n_cols, int64_t ld, int d) {
  return n_cols < (1 << 24) && ld * 4 < (1 << 24) &&
         ((uint64_t)n_cols * (uint64_t)ld + (uint64_t)d) * 4u < ((uint64_t)1 << 32);
}

// Partial dot product of a lane's columns; vectors whose columns lie past d contribute zero.
template <int W>
__device__ inline float dotw(const float (&a)[W], const float (&b)[W], const lane_cols<W / 4>& lc) {
  float s = 0.f;
#pragma unroll
  for (int v = 0; v < W / 4; ++v) {
    const float p = fmaf(a[4 * v + 3], b[4 * v + 3], fmaf(a[4 * v + 2], b[4 * v + 2], fmaf(a[4 * v + 1], b[4 * v + 1], a[4 * v] * b[4 * v])));
    s += lc.on[v] ? p : 0.f;
  }
  return s;
}

}  // namespace isp_dev
