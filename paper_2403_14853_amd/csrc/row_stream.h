// Row-streaming skeleton shared by SpMM and the FusedMM kernels (gfx950, wave64).
//
// One wavefront owns one work item: either a block of whole short rows or one segment of a hub
// row.  The item's nonzeros form one contiguous range of the CSR arrays; the wave reads them 64
// at a time (lane l holds entry p + l), broadcasts each (column, value) pair through
// v_readlane into scalar registers, and gathers the addressed dense row with all 64 lanes
// spread across the feature dimension (VEC consecutive floats per lane, T column groups of
// 64*VEC).  U gathers are issued back to back before the first is consumed so that each wave
// keeps several 64*VEC*4-byte requests in flight.  A row's result is written when its last
// nonzero has been added; a hub segment's result goes to the handle's partial-sum scratch and is
// combined by a second, fixed-order kernel (no floating-point atomics anywhere).
#pragma once
#include <type_traits>
#include "isp_internal.h"

namespace isp_dev {

template <int VEC> struct vec_of;
template <> struct vec_of<1> { using type = float; };
template <> struct vec_of<2> { using type = float2; };
template <> struct vec_of<4> { using type = float4; };

template <int VEC>
__device__ inline void load_vec(const float* __restrict__ p, float (&o)[VEC]) {
  using V = typename vec_of<VEC>::type;
  const V v = *reinterpret_cast<const V*>(p);
  if constexpr (VEC == 1) { o[0] = v; }
  else if constexpr (VEC == 2) { o[0] = v.x; o[1] = v.y; }
  else { o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w; }
}

template <int VEC>
__device__ inline void store_vec(float* __restrict__ p, const float (&o)[VEC]) {
  using V = typename vec_of<VEC>::type;
  V v;
  if constexpr (VEC == 1) { v = o[0]; }
  else if constexpr (VEC == 2) { v.x = o[0]; v.y = o[1]; }
  else { v.x = o[0]; v.y = o[1]; v.z = o[2]; v.w = o[3]; }
  *reinterpret_cast<V*>(p) = v;
}

__device__ inline int bcast_i(int v, int src_lane) { return __builtin_amdgcn_readlane(v, src_lane); }
__device__ inline float bcast_f(float v, int src_lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}

// Sum over the 64 lanes, result in every lane (xor butterfly).
__device__ inline float wave_allreduce(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Per-entry facts handed to a policy's edge function (all wave-uniform).
struct edge_info {
  int col;      // column index of the entry (row of the gathered operand)
  int perm;     // perm[p] when the policy asked for it, else 0
  int64_t pos;  // position p of the entry in the CSR arrays
};

// What a work item covers.
struct item_range {
  int64_t p, p_end;      // nonzero range
  int row, row_last;     // block items: rows [row, row_last); segment items: [seg, seg + 1)
  int src_row;           // matrix row the nonzeros belong to at the start (segment: the hub row)
  bool is_seg, skip;
};

__device__ inline item_range locate_item(const isp_view& A, const int64_t* __restrict__ indptr, int item) {
  (void)indptr;
  item_range r;
  const int4 q = A.item_desc[item];  // item is wave-uniform: one scalar load
  r.is_seg = item >= A.n_blocks;
  r.p = q.x;
  r.p_end = q.y;
  r.row = q.z;
  if (!r.is_seg) {
    // a block made of one hub row is empty here (its nonzeros are covered by segment items): end row -1
    r.skip = q.w < 0;
    r.row_last = q.w;
    r.src_row = q.z;
  } else {
    r.skip = false;
    r.row_last = q.z + 1;  // (row = the segment's number, which names its partial row)
    r.src_row = q.w;       // the hub row
  }
  return r;
}

// A policy may declare  static constexpr bool HAS_SKIP = true  and carry args::live (one byte per stored
// entry of the matrix being streamed): entries whose byte live[p] is 0 are passed over - nothing is gathered
// for them and edge() is not called.
template <class P, class = void>
struct policy_has_skip : std::false_type {};
template <class P>
struct policy_has_skip<P, std::void_t<decltype(P::HAS_SKIP)>> : std::bool_constant<P::HAS_SKIP> {};

// Policy P supplies:
//   static constexpr int VEC, T, NG, U;  static constexpr bool HAS_VAL, ACCUMULATE;
//   struct args { const float* src[NG]; int64_t ld[NG]; ... };
//   static constexpr bool NEEDS_PERM (also read perm[p] per entry), HAS_FINISH (call finish before a row is stored)
//   struct row_state;  static void row_begin(args, row_state&, int row, cols...)
//   static void edge(args, row_state&, float a, x[NG][T][VEC], acc[T][VEC], on[T], edge_info)
//   static void finish(args, row_state&, acc[T][VEC], out_row, is_seg, row_len, side, col[T], on[T])
template <class P>
__device__ inline void stream_item(const isp_view& A, const int64_t* __restrict__ indptr,
                                   const int32_t* __restrict__ indices, const float* __restrict__ values,
                                   const typename P::args& pa, int d, int k0, float* __restrict__ Y, int64_t ldy,
                                   int store_group = -1, int group_cnt = 1) {
  // store_group >= 0 (operations that need whole rows per entry, at widths beyond a partial row): a hub
  // segment computes with every column group of 64 * VEC columns but stores only groups [store_group,
  // store_group + group_cnt), into group_cnt consecutive partial rows (segment s owns rows s * group_cnt ...);
  // the host picks group_cnt so that all segments' rows fit the scratch and launches once per run of groups.
  // Row blocks write whole output rows, so they run in the launch that starts at group 0 only
  constexpr int VEC = P::VEC, T = P::T, NG = P::NG, U = P::U;
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  const int item = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * ISP_WAVES_PER_WG + (threadIdx.x >> 6)));
  if (item >= A.n_blocks + A.n_seg) return;
  item_range it = locate_item(A, indptr, item);
  if (it.skip) return;
  if (store_group > 0 && !it.is_seg) return;
  if (!it.is_seg) store_group = -1;

  int col[T];      // first feature column of this lane in each group, relative to the matrix
  bool on[T];
#pragma unroll
  for (int tt = 0; tt < T; ++tt) {
    col[tt] = k0 + (tt * ISP_WAVE + lane) * VEC;
    on[tt] = col[tt] < d;
  }
  // where results go: Y rows for block items, partial rows for segments
  float* __restrict__ out = it.is_seg ? A.partials : Y;
  const int64_t ldo = it.is_seg ? (int64_t)ISP_PARTIAL_TILE * (store_group >= 0 ? group_cnt : 1) : ldy;
  // partial rows hold only the current column tile (of it, only the stored groups, one row each)
  const int out_k0 = it.is_seg ? k0 + (store_group > 0 ? store_group * ISP_WAVE * VEC : 0) : 0;

  int row = it.row;
  const int row_last = it.row_last;
  int64_t p = it.p;
  const int64_t p_end = it.p_end;
  const int64_t never = INT64_MAX;
  int64_t row_end, row_end_next;
  int64_t row_start = p;
  if (it.is_seg) { row_end = p_end; row_end_next = never; }
  else {
    row_end = indptr[row + 1];
    row_end_next = (row + 1 < row_last) ? indptr[row + 2] : never;
  }

  float acc[T][VEC];
#pragma unroll
  for (int tt = 0; tt < T; ++tt)
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[tt][v] = 0.f;

  typename P::row_state rs;
  int src_row = it.src_row;

  auto write_row = [&]() {
    if constexpr (P::HAS_FINISH)
      P::finish(pa, rs, acc, row, it.is_seg, row_end - row_start,
                it.is_seg ? A.partials + (int64_t)row * ISP_PARTIAL_TILE : nullptr, col, on, k0);
#pragma unroll
    for (int tt = 0; tt < T; ++tt) {
      if (on[tt] && (store_group < 0 || (tt >= store_group && tt < store_group + group_cnt))) {
        float* o = out + (int64_t)row * ldo + (col[tt] - out_k0);
        if (P::ACCUMULATE && !it.is_seg) {
          float old[VEC];
          load_vec<VEC>(o, old);
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[tt][v] += old[v];
        }
        store_vec<VEC>(o, acc[tt]);
      }
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[tt][v] = 0.f;
    }
  };
  auto next_row = [&]() {
    ++row;
    ++src_row;
    row_start = row_end;
    row_end = row_end_next;
    row_end_next = (row + 1 < row_last) ? indptr[row + 2] : never;
  };

  // leading empty rows
  while (row < row_last && row_end == p) { write_row(); next_row(); }
  if (row < row_last) P::row_begin(pa, rs, src_row, col, on);

  while (p < p_end) {
    const int64_t left = p_end - p;
    const int cnt = left < ISP_WAVE ? (int)left : ISP_WAVE;
    int c = 0, pm = 0;
    float a = 1.f;
    bool dead = false;
    if (lane < cnt) {
      c = __builtin_nontemporal_load(indices + p + lane);
      if (P::HAS_VAL) a = __builtin_nontemporal_load(values + p + lane);
      if constexpr (P::NEEDS_PERM) pm = __builtin_nontemporal_load(pa.perm + p + lane);
      if constexpr (policy_has_skip<P>::value) dead = __builtin_nontemporal_load(pa.live + p + lane) == 0;
    }
    const unsigned long long dead_mask = policy_has_skip<P>::value ? __ballot(dead) : 0ull;  // bit t: entry p + t
    if constexpr (policy_has_skip<P>::value) {
      if (it.is_seg) {
        // a hub segment is one row with no row end inside, and nearly all of its entries are passed over:
        // visit the live ones only, U at a time
        unsigned long long todo = ~dead_mask & (cnt == ISP_WAVE ? ~0ull : ((1ull << cnt) - 1ull));
        while (todo) {
          int idx[U];
          float x[U][NG][T][VEC];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            idx[u] = todo ? (int)__builtin_ctzll(todo) : -1;
            todo &= todo - 1ull;  // (0 stays 0)
          }
#pragma unroll
          for (int u = 0; u < U; ++u) {
            if (idx[u] >= 0) {
              const int cj = bcast_i(c, idx[u]);
#pragma unroll
              for (int g = 0; g < NG; ++g) {
                const float* __restrict__ src = pa.src[g] + (int64_t)cj * pa.ld[g];
#pragma unroll
                for (int tt = 0; tt < T; ++tt) {
                  if (on[tt]) load_vec<VEC>(src + col[tt], x[u][g][tt]);
                  else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) x[u][g][tt][v] = 0.f;
                  }
                }
              }
            }
          }
#pragma unroll
          for (int u = 0; u < U; ++u) {
            if (idx[u] >= 0) {
              edge_info ei;
              ei.col = bcast_i(c, idx[u]);
              ei.perm = P::NEEDS_PERM ? bcast_i(pm, idx[u]) : 0;
              ei.pos = p + idx[u];
              P::edge(pa, rs, P::HAS_VAL ? bcast_f(a, idx[u]) : 1.f, x[u], acc, on, ei);
            }
          }
        }
        p += cnt;
        if (p == p_end) write_row();  // the segment's row ends with its last entry
        continue;
      }
    }
    for (int t = 0; t < cnt; t += U) {
      float x[U][NG][T][VEC];
      const bool full = t + U <= cnt;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if ((full || t + u < cnt) && !((dead_mask >> (t + u)) & 1ull)) {
          const int cj = bcast_i(c, t + u);
#pragma unroll
          for (int g = 0; g < NG; ++g) {
            const float* __restrict__ src = pa.src[g] + (int64_t)cj * pa.ld[g];
#pragma unroll
            for (int tt = 0; tt < T; ++tt) {
              if (on[tt]) load_vec<VEC>(src + col[tt], x[u][g][tt]);
              else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) x[u][g][tt][v] = 0.f;
              }
            }
          }
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (full || t + u < cnt) {
          if (!((dead_mask >> (t + u)) & 1ull)) {
            const float av = P::HAS_VAL ? bcast_f(a, t + u) : 1.f;
            edge_info ei;
            ei.col = bcast_i(c, t + u);
            ei.perm = P::NEEDS_PERM ? bcast_i(pm, t + u) : 0;
            ei.pos = p + t + u;
            P::edge(pa, rs, av, x[u], acc, on, ei);
          }
          if (p + t + u + 1 == row_end) {
            write_row();
            next_row();
            while (row < row_last && row_end == p + t + u + 1) { write_row(); next_row(); }
            if (row < row_last) P::row_begin(pa, rs, src_row, col, on);
          }
        }
      }
    }
    p += cnt;
  }
}

// Fixed-order combination of hub-segment partial sums: one wave per hub row adds its segments'
// partial rows in segment order and writes (or, with ACCUMULATE, adds to) the output row.
// stride / slot: segment s's partial row is row s * stride + slot of the scratch (1 / 0 unless the segments
// stored several column groups each).
template <int VEC, int T, bool ACCUMULATE>
__device__ inline void hub_fixup(const isp_view& A, int d, int k0, float* __restrict__ Y, int64_t ldy, int stride = 1,
                                 int slot = 0) {
  const int lane = threadIdx.x & (ISP_WAVE - 1);
  const int h = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * ISP_WAVES_PER_WG + (threadIdx.x >> 6)));
  if (h >= A.n_hub) return;
  const int s0 = A.hub_seg_ptr[h], s1 = A.hub_seg_ptr[h + 1];
  const int row = A.hub_rows[h];
#pragma unroll
  for (int tt = 0; tt < T; ++tt) {
    const int rel = (tt * ISP_WAVE + lane) * VEC;
    if (k0 + rel >= d) continue;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    int s = s0;
    for (; s + 8 <= s1; s += 8) {  // eight partial rows in flight, added in segment order
      float t[8][VEC];
#pragma unroll
      for (int u = 0; u < 8; ++u) load_vec<VEC>(A.partials + ((int64_t)(s + u) * stride + slot) * ISP_PARTIAL_TILE + rel, t[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] += t[u][v];
    }
    for (; s < s1; ++s) {
      float t[VEC];
      load_vec<VEC>(A.partials + ((int64_t)s * stride + slot) * ISP_PARTIAL_TILE + rel, t);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] += t[v];
    }
    float* o = Y + (int64_t)row * ldy + k0 + rel;
    if (ACCUMULATE) {
      float old[VEC];
      load_vec<VEC>(o, old);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[v] += old[v];
    }
    store_vec<VEC>(o, acc);
  }
}

// The same combination with one workgroup per hub row, for SpMM: a row cut into more than 32 segments
// (a vertex adjacent to a large share of the graph) is split four ways, each wavefront adds a contiguous
// quarter of the partial rows in order and the quarters are added in order - a fixed summation tree, so
// still deterministic.  Shorter rows are summed by the first wavefront alone, in segment order.
// MEAN: the sum is divided by the row's length (hub rows are never empty).
template <int VEC, int T, bool MEAN>
__device__ inline void hub_fixup_wg(const isp_view& A, int d, int k0, float* __restrict__ Y, int64_t ldy) {
  __shared__ float part[ISP_WAVES_PER_WG][T][ISP_WAVE][VEC];
  const int lane = threadIdx.x & (ISP_WAVE - 1), w = threadIdx.x >> 6;
  const int h = blockIdx.x;
  const int s0 = A.hub_seg_ptr[h], s1 = A.hub_seg_ptr[h + 1];
  const bool split = s1 - s0 > 32;  // uniform over the workgroup
  if (!split && w > 0) return;
  const int q = split ? (s1 - s0 + ISP_WAVES_PER_WG - 1) / ISP_WAVES_PER_WG : s1 - s0;
  const int a = s0 + w * q, b = (a + q < s1) ? a + q : s1;
  float acc[T][VEC];
#pragma unroll
  for (int tt = 0; tt < T; ++tt) {
    const int rel = (tt * ISP_WAVE + lane) * VEC;
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[tt][v] = 0.f;
    if (k0 + rel >= d) continue;
    int s = a;
    for (; s + 8 <= b; s += 8) {  // eight partial rows in flight, added in segment order
      float t[8][VEC];
#pragma unroll
      for (int u = 0; u < 8; ++u) load_vec<VEC>(A.partials + (int64_t)(s + u) * ISP_PARTIAL_TILE + rel, t[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[tt][v] += t[u][v];
    }
    for (; s < b; ++s) {
      float t[VEC];
      load_vec<VEC>(A.partials + (int64_t)s * ISP_PARTIAL_TILE + rel, t);
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[tt][v] += t[v];
    }
  }
  if (split) {
#pragma unroll
    for (int tt = 0; tt < T; ++tt)
#pragma unroll
      for (int v = 0; v < VEC; ++v) part[w][tt][lane][v] = acc[tt][v];
    __syncthreads();
    if (w > 0) return;
#pragma unroll
    for (int tt = 0; tt < T; ++tt)
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        float t = part[0][tt][lane][v];
#pragma unroll
        for (int ww = 1; ww < ISP_WAVES_PER_WG; ++ww) t += part[ww][tt][lane][v];
        acc[tt][v] = t;
      }
  }
  const int row = A.hub_rows[h];
  const float inv = MEAN ? A.inv_len[row] : 1.f;  // (= 1.f / (float)length, as the row blocks compute it)
#pragma unroll
  for (int tt = 0; tt < T; ++tt) {
    const int rel = (tt * ISP_WAVE + lane) * VEC;
    if (k0 + rel >= d) continue;
    if (MEAN) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[tt][v] *= inv;
    }
    store_vec<VEC>(Y + (int64_t)row * ldy + k0 + rel, acc[tt]);
  }
}

}  // namespace isp_dev
