// Device-wide exclusive prefix sums used by the CSR partition and the transpose
// (integer bookkeeping only).  Three launches: per-tile sums, a single-workgroup scan of the
// tile sums, per-tile scan with the tile offset added.
#include "isp_internal.h"

namespace {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

template <typename T>
__device__ inline T wave_inclusive_scan(T v, int lane) {
#pragma unroll
  for (int o = 1; o < ISP_WAVE; o <<= 1) {
    T t = __shfl_up(v, o);
    if (lane >= o) v += t;
  }
  return v;
}

// Exclusive scan of one value per thread across the workgroup; returns the exclusive prefix and
// writes the workgroup total to *total (same value in every thread).
template <typename T>
__device__ inline T block_exclusive_scan(T v, T* total) {
  __shared__ T wave_tot[SCAN_THREADS / ISP_WAVE];
  const int lane = threadIdx.x & (ISP_WAVE - 1), w = threadIdx.x / ISP_WAVE;
  T inc = wave_inclusive_scan(v, lane);
  __syncthreads();  // protect wave_tot against a previous call's readers
  if (lane == ISP_WAVE - 1) wave_tot[w] = inc;
  __syncthreads();
  T base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < SCAN_THREADS / ISP_WAVE; ++i) {
    if (i < w) base += wave_tot[i];
    tot += wave_tot[i];
  }
  *total = tot;
  return base + inc - v;
}

template <typename TI, typename TO>
__global__ void __launch_bounds__(SCAN_THREADS) scan_tile_sums(const TI* __restrict__ in, TO* __restrict__ tile_sum,
                                                               int64_t n) {
  const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
  TO s = 0;
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i)
    if (base + i < n) s += (TO)in[base + i];
  TO tot;
  block_exclusive_scan<TO>(s, &tot);
  if (threadIdx.x == 0) tile_sum[blockIdx.x] = tot;
}

// One workgroup: exclusive scan of tile_sum[0..nt) in place; grand total to *total_out.
template <typename TO>
__global__ void __launch_bounds__(SCAN_THREADS) scan_of_tile_sums(TO* __restrict__ tile_sum, int64_t nt,
                                                                  TO* __restrict__ total_out) {
  TO carry = 0;
  for (int64_t c = 0; c < nt; c += SCAN_THREADS) {
    const int64_t i = c + threadIdx.x;
    TO v = (i < nt) ? tile_sum[i] : (TO)0;
    TO tot;
    TO ex = block_exclusive_scan<TO>(v, &tot);
    if (i < nt) tile_sum[i] = carry + ex;
    carry += tot;
  }
  if (threadIdx.x == 0) *total_out = carry;
}

template <typename TI, typename TO>
__global__ void __launch_bounds__(SCAN_THREADS) scan_apply(const TI* __restrict__ in, TO* __restrict__ out,
                                                           const TO* __restrict__ tile_sum, int64_t n) {
  const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
  TO v[SCAN_ITEMS];
  TO s = 0;
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    v[i] = (base + i < n) ? (TO)in[base + i] : (TO)0;
    s += v[i];
  }
  TO tot;
  TO run = block_exclusive_scan<TO>(s, &tot) + tile_sum[blockIdx.x];
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    if (base + i < n) out[base + i] = run;
    run += v[i];
  }
}

template <typename TI, typename TO>
isp_status scan_impl(const TI* in, TO* out, int64_t n, void* tmp, hipStream_t s) {
  TO* tile_sum = (TO*)tmp;
  if (n <= 0) {  // only the total (zero) is written
    scan_of_tile_sums<TO><<<dim3(1), dim3(SCAN_THREADS), 0, s>>>(tile_sum, 0, out);
    ISP_LAUNCH_CHECK();
    return ISP_OK;
  }
  const int64_t nt = (n + SCAN_TILE - 1) / SCAN_TILE;
  scan_tile_sums<TI, TO><<<dim3((unsigned)nt), dim3(SCAN_THREADS), 0, s>>>(in, tile_sum, n);
  ISP_LAUNCH_CHECK();
  scan_of_tile_sums<TO><<<dim3(1), dim3(SCAN_THREADS), 0, s>>>(tile_sum, nt, out + n);
  ISP_LAUNCH_CHECK();
  scan_apply<TI, TO><<<dim3((unsigned)nt), dim3(SCAN_THREADS), 0, s>>>(in, out, tile_sum, n);
  ISP_LAUNCH_CHECK();
  return ISP_OK;
}

}  // namespace

size_t isp_scan_tmp_bytes(int64_t n) {
  const int64_t nt = (n + SCAN_TILE - 1) / SCAN_TILE;
  return isp_align((size_t)(nt + 1) * sizeof(int64_t));
}

isp_status isp_scan_i32_to_i64(const int32_t* in, int64_t* out, int64_t n, void* tmp, hipStream_t s) {
  return scan_impl<int32_t, int64_t>(in, out, n, tmp, s);
}

isp_status isp_scan_i32_to_i32(const int32_t* in, int32_t* out, int64_t n, void* tmp, hipStream_t s) {
  return scan_impl<int32_t, int32_t>(in, out, n, tmp, s);
}
