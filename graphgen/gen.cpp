// Seeded synthetic-input generators: Erdos-Renyi and R-MAT edge lists, CSR assembly
// (symmetrise, dedupe, self-loops, random vertex relabelling), edge-value
// normalisations and dense feature fills.
//
// This file produces INPUTS only.  It contains none of the sparse-kernel arithmetic
// (no SpMM / SDDMM / transpose) and is shared by the CPU oracle's tests and the GPU
// library's tests and benchmark so both sides see byte-identical data.
//
// All randomness is counter based (a 64-bit mixing function applied to
// (seed, stream, counter)), so a seed yields the same graph for any thread count.
//
// Build: g++ -O2 -fopenmp -shared -fPIC gen.cpp -o libgraphgen.so
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#include <omp.h>

namespace {

inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// One 64-bit draw for (seed, stream, counter).
inline uint64_t draw(uint64_t seed, uint64_t stream, uint64_t ctr) {
  return mix64(mix64(seed * 0xD1342543DE82EF95ull + stream) ^ (ctr * 0xA24BAED4963EE407ull + 1));
}

inline double u01(uint64_t r) {  // (0,1)
  return ((double)(r >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

}  // namespace

extern "C" {

// R-MAT candidate edges.  For edge e and level l one 16-bit uniform picks the quadrant
// with probabilities (a, b, c, 1-a-b-c); no noise.  Endpoints >= n are marked rejected
// (u = v = -1).  u is the row bit string, v the column bit string.
void gg_rmat_edges(int scale, int64_t n, int64_t m, uint64_t seed, double a, double b, double c,
                   int32_t* u_out, int32_t* v_out) {
  const uint32_t ta = (uint32_t)std::lround(a * 65536.0);
  const uint32_t tb = ta + (uint32_t)std::lround(b * 65536.0);
  const uint32_t tc = tb + (uint32_t)std::lround(c * 65536.0);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    uint64_t u = 0, v = 0, bits = 0;
    int have = 0;
    uint64_t word = 0;
    for (int l = 0; l < scale; ++l) {
      if (have == 0) {
        bits = draw(seed, 1, (uint64_t)e * 8 + word);
        ++word;
        have = 4;
      }
      uint32_t r = (uint32_t)(bits & 0xFFFF);
      bits >>= 16;
      --have;
      uint64_t ub, vb;
      if (r < ta) { ub = 0; vb = 0; }
      else if (r < tb) { ub = 0; vb = 1; }
      else if (r < tc) { ub = 1; vb = 0; }
      else { ub = 1; vb = 1; }
      u = (u << 1) | ub;
      v = (v << 1) | vb;
    }
    if ((int64_t)u >= n || (int64_t)v >= n) { u_out[e] = -1; v_out[e] = -1; }
    else { u_out[e] = (int32_t)u; v_out[e] = (int32_t)v; }
  }
}

// G(n, m)-style Erdos-Renyi candidates: m ordered pairs drawn uniformly.
void gg_er_edges(int64_t n, int64_t m, uint64_t seed, int32_t* u_out, int32_t* v_out) {
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    u_out[e] = (int32_t)(draw(seed, 2, (uint64_t)e * 2) % (uint64_t)n);
    v_out[e] = (int32_t)(draw(seed, 2, (uint64_t)e * 2 + 1) % (uint64_t)n);
  }
}

// Seeded random permutation of 0..n-1 (Fisher-Yates with counter-based draws).
void gg_permutation(int64_t n, uint64_t seed, int32_t* perm) {
  for (int64_t i = 0; i < n; ++i) perm[i] = (int32_t)i;
  for (int64_t i = n - 1; i > 0; --i) {
    int64_t j = (int64_t)(draw(seed, 3, (uint64_t)i) % (uint64_t)(i + 1));
    std::swap(perm[i], perm[j]);
  }
}

// Assemble a CSR pattern from candidate pairs.
//   relabel   : optional vertex permutation applied to both endpoints (may be NULL)
//   symmetrise: also insert (v,u) for every (u,v)
//   self_loops: 1 = insert (i,i) for every i; 0 = no diagonal entries at all
// Candidate self-pairs and rejected pairs (u < 0) are dropped; duplicates are removed;
// every row's columns come out sorted ascending.
// indptr must hold n+1 entries, indices at least (symmetrise?2:1)*m + n entries.
// Returns nnz.
int64_t gg_build_csr(int64_t n, int64_t m, const int32_t* u, const int32_t* v, const int32_t* relabel,
                     int symmetrise, int self_loops, int64_t* indptr, int32_t* indices) {
  std::vector<int64_t> cnt((size_t)n + 1, 0);
  auto lab = [&](int32_t x) { return relabel ? relabel[x] : x; };
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    if (u[e] < 0 || u[e] == v[e]) continue;
    int32_t a = lab(u[e]), b = lab(v[e]);
#pragma omp atomic
    cnt[a]++;
    if (symmetrise) {
#pragma omp atomic
      cnt[b]++;
    }
  }
  if (self_loops)
    for (int64_t i = 0; i < n; ++i) cnt[i]++;
  std::vector<int64_t> off((size_t)n + 1);
  off[0] = 0;
  for (int64_t i = 0; i < n; ++i) off[i + 1] = off[i] + cnt[i];
  const int64_t total = off[n];
  std::vector<int32_t> raw((size_t)total);
  std::vector<int64_t> cur(off.begin(), off.end() - 1);
  if (self_loops)
    for (int64_t i = 0; i < n; ++i) raw[cur[i]++] = (int32_t)i;
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    if (u[e] < 0 || u[e] == v[e]) continue;
    int32_t a = lab(u[e]), b = lab(v[e]);
    int64_t q;
#pragma omp atomic capture
    q = cur[a]++;
    raw[q] = b;
    if (symmetrise) {
#pragma omp atomic capture
      q = cur[b]++;
      raw[q] = a;
    }
  }
  // per-row sort + unique (makes the result independent of the scatter order)
  std::vector<int64_t> newcnt((size_t)n, 0);
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < n; ++i) {
    int32_t* s = raw.data() + off[i];
    int32_t* t = raw.data() + off[i + 1];
    std::sort(s, t);
    newcnt[i] = std::unique(s, t) - s;
  }
  indptr[0] = 0;
  for (int64_t i = 0; i < n; ++i) indptr[i + 1] = indptr[i] + newcnt[i];
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < n; ++i)
    std::memcpy(indices + indptr[i], raw.data() + off[i], (size_t)newcnt[i] * sizeof(int32_t));
  return indptr[n];
}

// Edge values.  mode 0: all ones.  mode 1: GCN normalisation 1/sqrt(deg_i*deg_j) with
// deg = stored entries per row (the pattern has unit entries, so this is the row sum).
// mode 2: row mean 1/deg_i.  Computed in fp64, rounded once to fp32.
void gg_values(int64_t n, const int64_t* indptr, const int32_t* indices, int mode, float* values) {
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < n; ++i) {
    const double di = (double)(indptr[i + 1] - indptr[i]);
    for (int64_t p = indptr[i]; p < indptr[i + 1]; ++p) {
      if (mode == 0) values[p] = 1.0f;
      else if (mode == 2) values[p] = (float)(1.0 / di);
      else {
        const int32_t j = indices[p];
        const double dj = (double)(indptr[j + 1] - indptr[j]);
        values[p] = (float)(1.0 / std::sqrt(di * (dj > 0 ? dj : 1.0)));
      }
    }
  }
}

void gg_fill_uniform(float* out, int64_t count, uint64_t seed, double lo, double hi) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) out[i] = (float)(lo + (hi - lo) * u01(draw(seed, 4, (uint64_t)i)));
}

// Box-Muller on counter-based uniforms; element i uses draws (2*(i/2), 2*(i/2)+1).
void gg_fill_normal(float* out, int64_t count, uint64_t seed, double mean, double stddev) {
  const int64_t pairs = (count + 1) / 2;
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < pairs; ++k) {
    const double u1 = u01(draw(seed, 5, (uint64_t)k * 2));
    const double u2 = u01(draw(seed, 5, (uint64_t)k * 2 + 1));
    const double r = std::sqrt(-2.0 * std::log(u1));
    const double t = 6.283185307179586476925 * u2;
    out[2 * k] = (float)(mean + stddev * r * std::cos(t));
    if (2 * k + 1 < count) out[2 * k + 1] = (float)(mean + stddev * r * std::sin(t));
  }
}

int gg_max_threads(void) { return omp_get_max_threads(); }

}  // extern "C"
