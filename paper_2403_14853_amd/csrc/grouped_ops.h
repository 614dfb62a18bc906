// Grouped kernels for the operations that need a whole dot product per nonzero (SDDMM and the
// FusedMM passes).  Same work items, LDS staging and step tables as the grouped SpMM; here a
// group of LPG lanes spans the full feature width (4 * LPG >= d), so G = 64 / LPG dot products
// are reduced side by side with the same DPP instructions.  In row blocks the row operand (U's row
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
template <class P, class = void>
struct policy_has_val2 : std::false_type {};
template <class P>
struct policy_has_val2<P, std::void_t<decltype(P::HAS_VAL2)>> : std::bool_constant<P::HAS_VAL2> {};

template <class P, int LPG, bool ADDR32>
__device__ inline void fused_grouped_item(const isp_view& A, const int64_t* __restrict__ indptr,
                                          const int32_t* __restrict__ indices, const float* __restrict__ values,
                                          const typename P::args& pa, int d, float* __restrict__ Y, int64_t ldy,
                                          gs_lds& lds, int k_lo = 0) {
  // k_lo: first feature column of this pass (only the per-entry policies run in column windows;
  // their partial dot products are then added up across passes)
  constexpr int G = ISP_WAVE / LPG;
  constexpr int NSRC = P::NSRC, NROW = P::NROW;
  constexpr int U = P::STEPS;  // steps in flight per buffer; two buffers
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  const int w = threadIdx.x >> 6;
  const int item = __builtin_amdgcn_readfirstlane((int)blockIdx.x * ISP_WAVES_PER_WG + w);
  if (item >= A.n_blocks + A.n_seg) return;
  const item_range it = locate_item(A, indptr, item);
  if (it.skip) return;
  gs_wave_lds& L = lds.w[w];
  // The policies with row results skip empty rows altogether (no step; the list of non-empty rows in L.ss
  // says where each row end belongs): directed graphs leave many rows empty (half of them in the FusedMM
  // benchmark graph).  The per-entry policy has no row results and keeps the plain table.
  constexpr bool sparse_rows = !P::PER_ENTRY;
  const int n_steps = values ? gs_prepare<G, true, sparse_rows, U>(it, indptr, indices, values, L, lane)
                             : gs_prepare<G, false, sparse_rows, U>(it, indptr, indices, values, L, lane);

  const int g = lane / LPG, q = lane % LPG;
  const int col = k_lo + q * 4;
  const bool lane_on = col < d;
  const int coff = lane_on ? col : 0;
  const unsigned lane_byte = (unsigned)coff * 4u;
  unsigned src_pitch[NSRC];  // row pitches of the gathered operands in bytes (ADDR32)
#pragma unroll
  for (int k = 0; k < NSRC; ++k) src_pitch[k] = (unsigned)pa.lds_[k] * 4u;
  float* __restrict__ out = it.is_seg ? A.partials + col : Y + col;
  const int64_t ldo = it.is_seg ? (int64_t)ISP_PARTIAL_TILE : ldy;
  // An empty row owns no step.  The k-th row end of the step table belongs to the k-th non-empty row of the
  // item, whose local index is L.ss[k] (a hub segment is its one row).
  int k_done = 0;            // row ends consumed
  const bool listed = sparse_rows && !it.is_seg;  // else the k-th row end belongs to row k
  int r_next = listed ? (int)L.ss[0] : 0;      // read one row ahead (the list ends with a spare entry)
  int k_issued = 0;          // row ends passed by the steps issued so far
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (!P::PER_ENTRY && !P::ACCUMULATE && listed && lane_on) {  // outputs of the empty rows
    const int n_rows = it.row_last - it.row;
    for (int r = g; r < n_rows; r += G)
      if (L.rp[r + 1] == L.rp[r]) store_vec<4>(out + (int64_t)(it.row + r) * ldo, acc);
  }

  auto finish_row = [&]() {
    const int row = it.row + __builtin_amdgcn_readfirstlane(r_next);  // (wave-uniform: scalar address math)
    ++k_done;
    r_next = listed ? (int)L.ss[k_done] : k_done;
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[v] = group_sum<LPG>(acc[v]);
    if (g == 0 && lane_on) {
      float* o = out + (int64_t)row * ldo;
      if (P::ACCUMULATE && !it.is_seg) {
        float old[4];
        load_vec<4>(o, old);
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[v] += old[v];
      }
      store_vec<4>(o, acc);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[v] = 0.f;
  };
  // SEG (a hub segment: one matrix row for the whole item): the row operand is loaded once and stays in
  // registers.  Row blocks re-read it with every step, which keeps their loop free of row-change stalls.
  auto run = [&](auto seg_tag) {
    constexpr bool SEG = decltype(seg_tag)::value;
    constexpr int NR = SEG ? 0 : NROW;  // per-step row-operand registers
    float rS[NROW][4];
    if constexpr (SEG) {
#pragma unroll
      for (int k = 0; k < NROW; ++k) load_vec<4>(pa.rowop[k] + (int64_t)it.src_row * pa.ldr[k] + coff, rS[k]);
    }
    auto issue = [&](int s0, unsigned (&dsc)[U], float (&x)[U][NSRC][4], float (&r)[U][NR + 1][4], float (&a)[U],
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
        const bool act = g < gs_cnt(dsc[u]) && lane_on;
        a[u] = __int_as_float(e[u].y);
        const int cj = act ? e[u].x : 0;  // dead lanes gather row 0; what they fetch is never used
        if constexpr (policy_has_val2<P>::value) {
          // (a dead lane reads the step's first entry, or the item's first one in a null step: valid positions)
          a2[u] = 1.f;
          if (pa.val2) a2[u] = pa.val2[it.p + gs_off(dsc[u]) + (g < gs_cnt(dsc[u]) ? g : 0)];
        }
#pragma unroll
        for (int k = 0; k < NSRC; ++k) {
          if constexpr (ADDR32) {
            const unsigned off = __umul24((unsigned)cj, src_pitch[k]) + lane_byte;
            load_vec<4>(reinterpret_cast<const float*>(reinterpret_cast<const char*>(pa.src[k]) + off), x[u][k]);
          } else {
            load_vec<4>(pa.src[k] + (int64_t)cj * pa.lds_[k] + coff, x[u][k]);
          }
        }
        if constexpr (!SEG) {
          const int64_t ri = srow[u] < (int)A.n_rows ? srow[u] : 0;  // null steps after the matrix's last row
#pragma unroll
          for (int k = 0; k < NROW; ++k) load_vec<4>(pa.rowop[k] + ri * pa.ldr[k] + coff, r[u][k]);
        }
      }
    };
    auto consume = [&](const unsigned (&dsc)[U], const float (&x)[U][NSRC][4], const float (&r)[U][NR + 1][4],
                       const float (&a)[U], const float (&a2)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        // The policies mask the per-lane partial dot products with lane_on (columns past d) and
        // accumulate only in live lanes, so nothing fetched by a dead lane reaches a result.
        const bool live = g < gs_cnt(dsc[u]);
        float rr[NROW][4];
#pragma unroll
        for (int k = 0; k < NROW; ++k)
#pragma unroll
          for (int v = 0; v < 4; ++v) rr[k][v] = SEG ? rS[k][v] : r[u][k < NR ? k : 0][v];
        if constexpr (P::PER_ENTRY) {
          // one output per stored entry, parked in the entry's LDS slot (its value has been read by
          // the step's issue) and written out in one coalesced sweep when the item is done
          const float val = P::template entry<LPG>(a[u], x[u], rr, lane_on);
          if (live && q == 0) L.ent[gs_off(dsc[u]) + g].y = __float_as_int(val);
        } else {
          if constexpr (policy_has_val2<P>::value) P::template edge<LPG>(pa, a[u], a2[u], x[u], rr, acc, lane_on, live && lane_on);
          else P::template edge<LPG>(pa, a[u], x[u], rr, acc, lane_on, live && lane_on);
          if (dsc[u] & GS_LAST) finish_row();
        }
      }
    };

    const int n_groups = n_steps / U;
    unsigned dA[U], dB[U];
    float xA[U][NSRC][4], xB[U][NSRC][4], rA[U][NR + 1][4], rB[U][NR + 1][4], aA[U], aB[U];
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

// Partial dot product of a lane's four columns; lanes whose columns lie past d contribute zero.
__device__ inline float dot4(const float (&a)[4], const float (&b)[4], bool lane_on) {
  const float p = fmaf(a[3], b[3], fmaf(a[2], b[2], fmaf(a[1], b[1], a[0] * b[0])));
  return lane_on ? p : 0.f;
}

}  // namespace isp_dev
