// Memory-system ceilings of the box, measured independently of the library: streaming float4
// reads and random 512-byte row gathers (the access pattern of SpMM at d = 128) over arrays of
// several footprints (L2-resident, Infinity-Cache-resident, HBM-resident).  Stand-alone program:
//   hipcc --offload-arch=gfx950 -O3 bw_probe.hip -o bw_probe && ./bw_probe
// (built as paper_2403_14853_amd/bw_probe by build.py).  Not part of the library or its ABI.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

__global__ void __launch_bounds__(256) k_stream(const float4* __restrict__ a, size_t n4, float* __restrict__ out) {
  float4 s = {0, 0, 0, 0};
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i + 3 * stride < n4; i += 4 * stride) {
    float4 v0 = a[i], v1 = a[i + stride], v2 = a[i + 2 * stride], v3 = a[i + 3 * stride];
    s.x += v0.x + v1.x + v2.x + v3.x; s.y += v0.y + v1.y + v2.y + v3.y;
    s.z += v0.z + v1.z + v2.z + v3.z; s.w += v0.w + v1.w + v2.w + v3.w;
  }
  for (; i < n4; i += stride) { float4 v = a[i]; s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w; }
  if (s.x + s.y + s.z + s.w == 1.2345f) out[0] = 1.f;
}

// each wave gathers rows idx[..] of 128 floats (float2 per lane), 8 rows in flight
__global__ void __launch_bounds__(256) k_gather(const float* __restrict__ X, const int* __restrict__ idx, size_t n_idx,
                                                float* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const size_t n_waves = ((size_t)gridDim.x * blockDim.x) >> 6;
  const size_t per = n_idx / n_waves;
  const int* my = idx + wave * per;
  float2 s = {0, 0};
  for (size_t t = 0; t + 8 <= per; t += 8) {
    float2 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = __builtin_amdgcn_readfirstlane(my[t + u]);
      v[u] = *reinterpret_cast<const float2*>(X + (size_t)r * 128 + lane * 2);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; }
  }
  if (s.x + s.y == 1.2345f) out[0] = 1.f;
}

// same gather with float4 per lane: one instruction fetches two rows (half a wave each), 8 in flight
__global__ void __launch_bounds__(256) k_gather4(const float* __restrict__ X, const int* __restrict__ idx, size_t n_idx,
                                                 float* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const size_t n_waves = ((size_t)gridDim.x * blockDim.x) >> 6;
  const size_t per = n_idx / n_waves;
  const int* my = idx + wave * per;
  float4 s = {0, 0, 0, 0};
  for (size_t t = 0; t + 16 <= per; t += 16) {
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = my[t + 2 * u + (lane >> 5)];
      v[u] = *reinterpret_cast<const float4*>(X + (size_t)r * 128 + (lane & 31) * 4);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
  }
  if (s.x + s.y + s.z + s.w == 1.2345f) out[0] = 1.f;
}

int main() {
  float* out; CK(hipMalloc(&out, 256));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  const size_t sizes_mb[] = {2, 8, 16, 32, 64, 128, 256, 512, 1280, 4096};
  for (size_t mb : sizes_mb) {
    const size_t bytes = mb << 20;
    float* a; CK(hipMalloc(&a, bytes)); CK(hipMemset(a, 0, bytes));
    const size_t n4 = bytes / 16;
    int reps = (int)((size_t)(16ull << 30) / bytes); if (reps < 4) reps = 4; if (reps > 2000) reps = 2000;
    for (int grid : {256 * 8, 256 * 32}) {
      for (int i = 0; i < 3; ++i) k_stream<<<grid, 256>>>((const float4*)a, n4, out);
      CK(hipEventRecord(e0));
      for (int i = 0; i < reps; ++i) k_stream<<<grid, 256>>>((const float4*)a, n4, out);
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1));
      printf("stream %5zu MB grid %5d: %.2f TB/s\n", mb, grid, (double)bytes * reps / (ms * 1e-3) / 1e12);
    }
    // random row gather over this array
    const size_t n_rows = bytes / 512;
    const size_t n_idx = 256ull * 32 * 4 * 2048;  // 67M gathers of 512 B = 34 GB
    std::vector<int> h(n_idx);
    unsigned long long z = 88172645463325252ull;
    for (size_t i = 0; i < n_idx; ++i) { z ^= z << 13; z ^= z >> 7; z ^= z << 17; h[i] = (int)(z % n_rows); }
    int* idx; CK(hipMalloc(&idx, n_idx * 4)); CK(hipMemcpy(idx, h.data(), n_idx * 4, hipMemcpyHostToDevice));
    k_gather<<<256 * 8, 256>>>(a, idx, n_idx, out);
    CK(hipEventRecord(e0));
    for (int i = 0; i < 3; ++i) k_gather<<<256 * 8, 256>>>(a, idx, n_idx, out);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    printf("gather %5zu MB: %.2f TB/s (512 B rows, float2 per lane, 8 in flight per wave, 8 waves/SIMD)\n", mb, (double)n_idx * 512 * 3 / (ms * 1e-3) / 1e12);
    k_gather4<<<256 * 8, 256>>>(a, idx, n_idx, out);
    CK(hipEventRecord(e0));
    for (int i = 0; i < 3; ++i) k_gather4<<<256 * 8, 256>>>(a, idx, n_idx, out);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    CK(hipEventElapsedTime(&ms, e0, e1));
    printf("gather4 %4zu MB: %.2f TB/s (512 B rows, float4 per lane, two rows per instruction)\n", mb, (double)n_idx * 512 * 3 / (ms * 1e-3) / 1e12);
    CK(hipFree(idx)); CK(hipFree(a));
    fflush(stdout);
  }
  return 0;
}
