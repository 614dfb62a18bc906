// Grouped row-streaming skeleton (gfx950, wave64): the fast path when the feature width and the
// operands' alignment allow 16-byte lanes.
//
// A wavefront owns one work item (a block of whole short rows or one hub-row segment) whose
// nonzeros are contiguous in the CSR arrays.  The 64 lanes form G = 64 / LPG groups of LPG
// lanes; a group gathers one dense row slice of 4 * LPG floats with one float4 per lane, so a
// single load instruction serves G nonzeros.  The item's (column, value) pairs are staged once
// in LDS; a per-item step table, also in LDS, says for every step which G consecutive entries
// it covers and whether it ends a row (a step never crosses a row boundary; an empty row owns one
// step without entries or, in the kernels that ask for it, none: they zero its output beforehand,
// and a list of the non-empty rows says which row each row end of the table belongs to).  The main
// loop is therefore flat: U steps are issued back to back (LDS read -> address -> gather) before
// the first is consumed, independent of where rows begin and end, which keeps short rows from
// serialising on memory latency.  When
// a step ends a row the G group accumulators are summed with lane shuffles that leave each group
// with a share of the finished columns (group_reduce_scatter), and every group writes its share.  Feature columns beyond one slice are covered by further workgroups
// (blockIdx % n_slices), dealt round-robin to the XCDs.
#pragma once
#include "row_stream.h"

namespace isp_dev {

// Partition limits this skeleton is sized for (csr_build clamps its parameters to them).
constexpr int GS_MAX_ENT = 768;    // nonzeros per item:  block_cost - 1 + hub_t  or  seg_len
constexpr int GS_MAX_ROWS = 256;   // rows per item: block_cost
constexpr int GS_MAX_STEPS = GS_MAX_ENT + GS_MAX_ROWS;  // G = 1 worst case

constexpr int GS_U = 8;            // steps issued back to back; step tables are padded to a multiple

typedef unsigned short gs_u16;
struct __attribute__((aligned(16))) gs_wave_lds {
  int2 ent[GS_MAX_ENT + 8];               // (column, value bits) of the item's nonzeros
  gs_u16 step[GS_MAX_STEPS + GS_U];       // step descriptors, padded with null steps
  gs_u16 rp[GS_MAX_ROWS + 8];             // row start offsets relative to the item
  gs_u16 ss[GS_MAX_ROWS + 8];             // first step of each row; afterwards the list of non-empty rows
};
struct gs_lds { gs_wave_lds w[ISP_WAVES_PER_WG]; };

// step descriptor (16 bits): bits 0..9 entry offset, 10..14 live entries (0..16), bit 15 ends a row
constexpr unsigned GS_LAST = 0x8000u;
__device__ inline gs_u16 gs_pack(int off, int cnt, bool last) {
  return (gs_u16)((unsigned)off | ((unsigned)cnt << 10) | (last ? GS_LAST : 0u));
}
__device__ inline int gs_off(unsigned dsc) { return (int)(dsc & 0x3ffu); }
__device__ inline int gs_cnt(unsigned dsc) { return (int)((dsc >> 10) & 31u); }

// Orders this wave's earlier LDS writes before its later LDS reads (other lanes' data).  The LDS
// unit executes one wave's operations in order, so only the compiler has to be held back.
__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

__device__ inline int wave_exclusive_scan_i(int v, int lane, int* total) {
  int inc = v;
#pragma unroll
  for (int o = 1; o < ISP_WAVE; o <<= 1) {
    const int t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  *total = __shfl(inc, ISP_WAVE - 1);
  return inc - v;
}

// Stage the item's entries and build its step table.  Returns the number of steps, rounded up to
// a multiple of PAD (the caller's steps per issue, at most GS_U) with null steps (no live entry, not a
// row end); 0 when the item has no entries.
// SPARSE_ROWS: empty rows own no step, and ss ends up holding the local indices of the non-empty rows, in
// order, then one spare 0, then the local indices of the empty rows (the kernel writes their outputs itself:
// gs_empty_rows below); otherwise an empty row owns one step without entries.  rp holds the rows' start offsets.
// *n_live (optional): the number of non-empty rows of a row block (SPARSE_ROWS only).
template <int G, bool HAS_VAL, bool SPARSE_ROWS = false, int PAD = GS_U>
__device__ inline int gs_prepare(const item_range& it, const int64_t* __restrict__ indptr,
                                 const int32_t* __restrict__ indices, const float* __restrict__ values,
                                 gs_wave_lds& L, int lane, int* n_live_out = nullptr) {
  constexpr bool sparse_rows = SPARSE_ROWS;
  static_assert(PAD >= 1 && PAD <= GS_U, "the step table has room for GS_U null steps");
  int2* __restrict__ ent = L.ent;
  gs_u16* __restrict__ step = L.step;
  gs_u16* __restrict__ rp = L.rp;
  gs_u16* __restrict__ ss = L.ss;
  const int n_ent = (int)(it.p_end - it.p);
  // Eight loads per lane are issued before the first is stored: the item's entries arrive in one or two round
  // trips to memory instead of one per 64 entries (nothing else of the item can start before they are here).
  constexpr int SB = 8;
  for (int base = 0; base < n_ent; base += SB * ISP_WAVE) {
    int c[SB];
    float v[SB];
#pragma unroll
    for (int u = 0; u < SB; ++u) {
      const int i = base + u * ISP_WAVE + lane;
      c[u] = 0;
      v[u] = 1.f;
      if (i < n_ent) {
        c[u] = __builtin_nontemporal_load(indices + it.p + i);
        if (HAS_VAL) v[u] = __builtin_nontemporal_load(values + it.p + i);
      }
    }
#pragma unroll
    for (int u = 0; u < SB; ++u) {
      const int i = base + u * ISP_WAVE + lane;
      if (i < n_ent) ent[i] = make_int2(c[u], __float_as_int(v[u]));
    }
  }
  const int n_rows = it.row_last - it.row;
  if (it.is_seg) {
    // one row, no table to search: step s covers entries [s * G, s * G + G), the last one ends the row
    const int n_steps = (n_ent + G - 1) / G;
    const int n_padded = (n_steps + PAD - 1) / PAD * PAD;
    for (int s = lane; s < n_padded; s += ISP_WAVE) {
      const int left = n_ent - s * G;
      step[s] = s < n_steps ? gs_pack(s * G, left >= G ? G : left, s + 1 == n_steps) : (gs_u16)0;
    }
    wave_lds_sync();
    if (n_live_out) *n_live_out = 1;
    return n_padded;
  }
  for (int r = lane; r <= n_rows; r += ISP_WAVE) rp[r] = (gs_u16)(indptr[it.row + r] - it.p);
  wave_lds_sync();
  // steps per row (an empty row owns none) and the row's rank among the non-empty rows, scanned together:
  // low half = steps, high half = non-empty rows
  constexpr int CHUNKS = GS_MAX_ROWS / ISP_WAVE;
  int carry = 0, rank[CHUNKS];
#pragma unroll
  for (int ci = 0; ci < CHUNKS; ++ci) rank[ci] = -1 - GS_MAX_ROWS - 1;  // (no row)
#pragma unroll
  for (int ci = 0; ci < CHUNKS; ++ci) {
    if (ci * ISP_WAVE >= n_rows) break;  // (most items hold fewer than 64 rows: one scan)
    const int r = ci * ISP_WAVE + lane;
    int v = 0;
    if (r < n_rows) {
      const int len = (int)rp[r + 1] - (int)rp[r];
      // (without the list an empty row owns one step that ends it and has no entry)
      v = len > 0 ? ((len + G - 1) / G) | (1 << 16) : (sparse_rows ? 0 : 1 | (1 << 16));
    }
    int tot;
    const int ex = wave_exclusive_scan_i(v, lane, &tot);
    if (r < n_rows) ss[r] = (gs_u16)((carry + ex) & 0xffff);
    // non-empty rows before this one; an empty row keeps it as -1 - (that number)
    rank[ci] = v ? (carry + ex) >> 16 : (r < n_rows ? -1 - ((carry + ex) >> 16) : -1 - GS_MAX_ROWS - 1);
    carry += tot;
  }
  const int n_steps = carry & 0xffff;
  const int n_live = carry >> 16;
  if (lane == 0) ss[n_rows] = (gs_u16)n_steps;
  wave_lds_sync();
  const int n_padded = (n_steps + PAD - 1) / PAD * PAD;
  for (int s = lane; s < n_padded; s += ISP_WAVE) {
    gs_u16 dsc = 0;  // null step
    if (s < n_steps) {
      int lo = 0, hi = n_rows;  // last row r with ss[r] <= s: the non-empty row that owns step s
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int)ss[mid] <= s) lo = mid; else hi = mid;
      }
      const int k = s - (int)ss[lo];
      const int len = (int)rp[lo + 1] - (int)rp[lo];
      const int left = len - k * G;
      dsc = gs_pack((int)rp[lo] + k * G, left >= G ? G : (left > 0 ? left : 0), s + 1 == (int)ss[lo + 1]);
    }
    step[s] = dsc;
  }
  wave_lds_sync();
  // the step table is built: ss now lists the non-empty rows in order (ss[k] = local index of the k-th),
  // which is where the k-th row end of the table belongs; one more entry for the null steps past the end.
  // Without SPARSE_ROWS every row owns a step and the k-th row end belongs to row k.
  if constexpr (sparse_rows) {
#pragma unroll
    for (int ci = 0; ci < CHUNKS; ++ci) {
      const int r = ci * ISP_WAVE + lane;
      if (rank[ci] >= 0) ss[rank[ci]] = (gs_u16)r;
      // the empty rows behind the spare entry: row r has r - (non-empty rows before it) empty rows before it
      else if (rank[ci] >= -1 - GS_MAX_ROWS) ss[n_live + 1 + r - (-1 - rank[ci])] = (gs_u16)r;
    }
    if (lane == 0) ss[n_live] = 0;
    wave_lds_sync();
  }
  if (n_live_out) *n_live_out = n_live;
  return n_padded;
}

// Sum over the LPG consecutive lanes of a group, result in every lane of the group.  Lane
// exchanges inside 16 lanes are DPP modifiers (no LDS traffic); xor 16 is a ds_swizzle, xor 32 a
// bpermute.
template <int LPG>
__device__ inline float group_allreduce(float v) {
  // quad_perm [1,0,3,2] and [2,3,0,1]: xor 1, xor 2
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
  // row_half_mirror (reverse within 8 lanes): pairs the two quads of an 8-lane half
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));
  if constexpr (LPG >= 16)  // row_mirror (reverse within 16 lanes)
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));
  if constexpr (LPG >= 32)  // swap halves of 32 lanes: swizzle bit mode, xor mask 0x10
    v += __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));
  if constexpr (LPG >= 64) v += __shfl_xor(v, 32);
  return v;
}

// Sum W values per lane over the G = 64 / LPG groups (lanes with equal lane % LPG), leaving the sums spread over
// the groups instead of complete in one: a stage that pairs lanes `O` apart splits the values in two halves,
// each lane of a pair keeps one half and receives the partner's share of it, so the stages move W/2 + W/4 + ...
// values instead of W each.  Afterwards the lane holds, in v[0 .. R), R = max(1, W / G), the finished sums of
// its values idx0 .. idx0 + R (idx0 is returned).  With more groups than values (G > W) the last stages add
// single values both ways and the groups whose lane number has a bit of (64 / W - 1) & ~(LPG - 1) set hold
// copies: group_owner<LPG, W>(lane) says which lanes hold the ones to store.  The order of the additions is
// fixed, so results repeat bit for bit.
template <int O, int LPG, int N, int W>
__device__ inline void group_reduce_stage(float (&v)[W], int lane, int& idx0) {
  if constexpr (O >= LPG) {
    if constexpr (N > 1) {
      const bool up = (lane & O) != 0;
#pragma unroll
      for (int c = 0; c < N / 2; ++c) {
        const float send = up ? v[c] : v[c + N / 2];
        const float keep = up ? v[c + N / 2] : v[c];
        v[c] = keep + __shfl_xor(send, O);
      }
      idx0 += up ? N / 2 : 0;
      group_reduce_stage<O / 2, LPG, N / 2, W>(v, lane, idx0);
    } else {
      v[0] += __shfl_xor(v[0], O);
      group_reduce_stage<O / 2, LPG, 1, W>(v, lane, idx0);
    }
  }
}
template <int LPG, int W>
__device__ inline int group_reduce_scatter(float (&v)[W], int lane) {
  int idx0 = 0;
  group_reduce_stage<ISP_WAVE / 2, LPG, W, W>(v, lane, idx0);
  return idx0;
}
template <int LPG, int W>
__device__ inline bool group_owner(int lane) {
  return (lane & ((ISP_WAVE / W - 1) & ~(LPG - 1))) == 0;
}

}  // namespace isp_dev
