// A consumer of the C ABI with nothing else around it: no Python, no PyTorch.  It allocates with the HIP
// runtime, runs SpMM, the cached-transpose backward and SDDMM on a small band graph, and compares with
// plain host loops.  Built next to the library (paper_2403_14853_amd/abi_example); prints "OK" and returns 0.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>
#include "isp.h"

#define HIP_OK(call)                                                                 \
  do {                                                                               \
    hipError_t e_ = (call);                                                          \
    if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 2; } \
  } while (0)
#define ISP_CALL(call)                                                               \
  do {                                                                               \
    isp_status s_ = (call);                                                          \
    if (s_ != ISP_OK) { fprintf(stderr, "%s -> %d: %s\n", #call, (int)s_, isp_last_error()); return 3; } \
  } while (0)

template <class T>
static T* to_device(const std::vector<T>& h) {
  T* d = nullptr;
  if (hipMalloc((void**)&d, h.size() * sizeof(T) + 16) != hipSuccess) return nullptr;
  if (hipMemcpy(d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
  return d;
}

int main() {
  const int64_t n = 5000;
  const int d = 48;
  // row i: columns i, i+1, i+7 (mod n), plus a hub row 0 that touches every third column
  std::vector<int64_t> indptr(n + 1, 0);
  std::vector<int32_t> indices;
  std::vector<float> values;
  for (int64_t i = 0; i < n; ++i) {
    if (i == 0) {
      for (int64_t j = 0; j < n; j += 3) { indices.push_back((int32_t)j); values.push_back(0.01f * (float)(j % 11)); }
    } else {
      const int64_t c[3] = {i, (i + 1) % n, (i + 7) % n};
      for (int k = 0; k < 3; ++k) { indices.push_back((int32_t)c[k]); values.push_back(1.f / (float)(k + 1)); }
    }
    indptr[i + 1] = (int64_t)indices.size();
  }
  const int64_t nnz = (int64_t)indices.size();
  std::vector<float> X(n * d), G(n * d);
  for (int64_t i = 0; i < n; ++i)
    for (int k = 0; k < d; ++k) {
      X[i * d + k] = 0.1f * (float)(i % 13) - 0.05f * (float)k;
      G[i * d + k] = 0.02f * (float)((i * 7 + k) % 17) - 0.1f;
    }

  int64_t* d_indptr = to_device(indptr);
  int32_t* d_indices = to_device(indices);
  float* d_values = to_device(values);
  float* d_X = to_device(X);
  float* d_G = to_device(G);
  float *d_Y = nullptr, *d_dX = nullptr, *d_dA = nullptr;
  HIP_OK(hipMalloc((void**)&d_Y, n * d * sizeof(float)));
  HIP_OK(hipMalloc((void**)&d_dX, n * d * sizeof(float)));
  HIP_OK(hipMalloc((void**)&d_dA, nnz * sizeof(float)));
  if (!d_indptr || !d_indices || !d_values || !d_X || !d_G) { fprintf(stderr, "allocation failed\n"); return 2; }

  size_t ws_bytes = 0, wt_bytes = 0;
  void *ws = nullptr, *wt = nullptr;
  ISP_CALL(isp_csr_build_workspace(n, n, nnz, &ws_bytes));
  HIP_OK(hipMalloc(&ws, ws_bytes));
  isp_csr_t* A = nullptr;
  ISP_CALL(isp_csr_build(n, n, nnz, d_indptr, d_indices, d_values, ws, ws_bytes, 0, nullptr, &A));
  ISP_CALL(isp_spmm(A, d_X, d, d, d_Y, d, nullptr));
  ISP_CALL(isp_csr_transpose_workspace(A, &wt_bytes));
  HIP_OK(hipMalloc(&wt, wt_bytes));
  const isp_csr_t* At = nullptr;
  int was_cached = -1;
  ISP_CALL(isp_csr_transpose_cached(A, wt, wt_bytes, nullptr, &At, &was_cached));
  if (was_cached != 0) { fprintf(stderr, "first transpose call reported a cache hit\n"); return 4; }
  ISP_CALL(isp_csr_transpose_cached(A, nullptr, 0, nullptr, &At, &was_cached));
  if (was_cached != 1) { fprintf(stderr, "second transpose call missed the cache\n"); return 4; }
  ISP_CALL(isp_spmm(At, d_G, d, d, d_dX, d, nullptr));
  ISP_CALL(isp_sddmm(A, d_G, d, d_X, d, d, 0, d_dA, nullptr));
  HIP_OK(hipDeviceSynchronize());

  std::vector<float> Y(n * d), dX(n * d), dA(nnz);
  HIP_OK(hipMemcpy(Y.data(), d_Y, Y.size() * sizeof(float), hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(dX.data(), d_dX, dX.size() * sizeof(float), hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(dA.data(), d_dA, dA.size() * sizeof(float), hipMemcpyDeviceToHost));

  // host loops
  std::vector<double> rY(n * d, 0.0), mY(n * d, 0.0), rdX(n * d, 0.0), mdX(n * d, 0.0);
  double worst = 0.0;
  for (int64_t i = 0; i < n; ++i)
    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {
      const int64_t j = indices[p];
      double dot = 0.0, mag = 0.0;
      for (int k = 0; k < d; ++k) {
        const double a = values[p];
        rY[i * d + k] += a * X[j * d + k];
        mY[i * d + k] += fabs(a * X[j * d + k]);
        rdX[j * d + k] += a * G[i * d + k];
        mdX[j * d + k] += fabs(a * G[i * d + k]);
        dot += (double)G[i * d + k] * X[j * d + k];
        mag += fabs((double)G[i * d + k] * X[j * d + k]);
      }
      const double r = fabs(dA[p] - dot) / (1e-5 * mag + 1e-6);
      worst = r > worst ? r : worst;
    }
  for (int64_t e = 0; e < n * d; ++e) {
    const double r1 = fabs(Y[e] - rY[e]) / (1e-5 * mY[e] + 1e-6), r2 = fabs(dX[e] - rdX[e]) / (1e-5 * mdX[e] + 1e-6);
    worst = r1 > worst ? r1 : worst;
    worst = r2 > worst ? r2 : worst;
  }
  isp_csr_destroy(A);
  printf("%s: n=%lld nnz=%lld d=%d, largest error / tolerance = %.3f (%s)\n", worst <= 1.0 ? "OK" : "MISMATCH",
         (long long)n, (long long)nnz, d, worst, isp_version());
  return worst <= 1.0 ? 0 : 1;
}
