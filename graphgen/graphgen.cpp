// Seeded synthetic input generator for CSR SpMM experiments.
//
// This file produces INPUTS only (graph structure in CSR, edge values, dense
// feature matrices).  It contains none of the SpMM arithmetic: both the CPU
// oracle and the GPU library are fed from here and share nothing else.
//
// Every random quantity is a pure function of (seed, stream, index) through a
// counter-based 64-bit mixer, so the output is identical for any thread count.
//
// Graph families (stand-ins for the paper's workloads: the citation graphs of
// Table IV, the random graphs of Section V-B and the SNAP range of Section V-A):
//   * Chung-Lu with power-law expected degrees, symmetric or directed
//   * R-MAT on a 2^scale grid
// Output is always plain CSR with sorted, duplicate-free column indices.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <unordered_set>
#include <vector>
#include <parallel/algorithm>
#include <omp.h>

namespace {

// ---------------------------------------------------------------- RNG ------
inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
// value #idx of stream #stream under `seed`
inline uint64_t rng_u64(uint64_t seed, uint64_t stream, uint64_t idx) {
  return mix64(mix64(seed * 0xD1342543DE82EF95ull + stream) ^ (idx * 0xA0761D6478BD642Full + 0x2545F4914F6CDD1Dull));
}
inline double u64_to_unit(uint64_t x) { return (double)(x >> 11) * (1.0 / 9007199254740992.0); }  // [0,1)

enum Stream : uint64_t {
  ST_PERM_A = 1, ST_PERM_B = 2, ST_EDGE_U = 3, ST_EDGE_V = 4, ST_EMPTY = 5,
  ST_RMAT = 6, ST_VALS = 7, ST_DENSE = 8
};

struct Csr {
  int64_t M = 0, K = 0, nnz = 0;
  std::vector<int32_t> rowptr;
  std::vector<int32_t> colind;
};

// Sorted unique (row<<32|col) keys -> CSR.
void keys_to_csr(std::vector<uint64_t>& keys, int64_t M, int64_t K, Csr* out) {
  __gnu_parallel::sort(keys.begin(), keys.end());
  keys.erase(std::unique(keys.begin(), keys.end()), keys.end());
  const int64_t nnz = (int64_t)keys.size();
  out->M = M; out->K = K; out->nnz = nnz;
  out->rowptr.assign((size_t)M + 1, 0);
  out->colind.resize((size_t)nnz);
  std::vector<int32_t>& rp = out->rowptr;
#pragma omp parallel for schedule(static)
  for (int64_t p = 0; p < nnz; ++p) out->colind[p] = (int32_t)(keys[p] & 0xFFFFFFFFull);
  // rowptr[r+1] = number of keys with row <= r : mark row ends, then fill gaps.
  // Sequential and simple: one pass over the keys.
  int64_t r = 0;
  for (int64_t p = 0; p < nnz; ++p) {
    const int64_t row = (int64_t)(keys[p] >> 32);
    while (r < row) rp[++r] = (int32_t)p;
  }
  while (r < M) rp[++r] = (int32_t)nnz;
}

// Seeded Fisher-Yates permutation of 0..M-1.
void permutation(int64_t M, uint64_t seed, uint64_t stream, std::vector<int32_t>* perm) {
  perm->resize((size_t)M);
  for (int64_t i = 0; i < M; ++i) (*perm)[i] = (int32_t)i;
  for (int64_t i = M - 1; i > 0; --i) {
    const uint64_t j = rng_u64(seed, stream, (uint64_t)i) % (uint64_t)(i + 1);
    std::swap((*perm)[i], (*perm)[j]);
  }
}

// Power-law expected-degree weights w_i = (i + i0)^(-1/(gamma-1)), i0 chosen by
// bisection so that max(w)/mean(w) == max_over_mean; returns the cumulative sums.
void powerlaw_cdf(int64_t M, double gamma, double max_over_mean, std::vector<double>* cdf) {
  const double ex = -1.0 / (gamma - 1.0);
  auto ratio = [&](double i0) {
    double s = 0.0;
    for (int64_t i = 0; i < M; ++i) s += std::pow((double)i + i0, ex);
    return std::pow(i0, ex) / (s / (double)M);
  };
  double lo = 1e-3, hi = (double)M * 64.0;  // ratio decreases with i0
  for (int it = 0; it < 60; ++it) {
    const double mid = std::sqrt(lo * hi);
    if (ratio(mid) > max_over_mean) lo = mid; else hi = mid;
  }
  const double i0 = std::sqrt(lo * hi);
  cdf->resize((size_t)M);
  double s = 0.0;
  for (int64_t i = 0; i < M; ++i) { s += std::pow((double)i + i0, ex); (*cdf)[i] = s; }
}

inline int64_t sample_cdf(const std::vector<double>& cdf, double u01) {
  const double x = u01 * cdf.back();
  int64_t lo = 0, hi = (int64_t)cdf.size() - 1;  // first index with cdf[idx] > x
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (cdf[mid] > x) hi = mid; else lo = mid + 1;
  }
  return lo;
}

}  // namespace

extern "C" {

// ---- CSR handle ------------------------------------------------------------
int64_t gg_csr_rows(const void* h) { return ((const Csr*)h)->M; }
int64_t gg_csr_cols(const void* h) { return ((const Csr*)h)->K; }
int64_t gg_csr_nnz(const void* h) { return ((const Csr*)h)->nnz; }
void gg_csr_copy(const void* h, int32_t* rowptr, int32_t* colind) {
  const Csr* c = (const Csr*)h;
  std::memcpy(rowptr, c->rowptr.data(), sizeof(int32_t) * c->rowptr.size());
  if (c->nnz) std::memcpy(colind, c->colind.data(), sizeof(int32_t) * (size_t)c->nnz);
}
void gg_csr_free(void* h) { delete (Csr*)h; }

// ---- Chung-Lu, symmetric ---------------------------------------------------
// Undirected edges {u,v}, u != v, endpoints drawn independently from the
// power-law weight distribution; each kept edge yields two non-zeros.
//  exact != 0 : candidates are taken in index order until exactly `edges`
//               distinct undirected edges exist (nnz == 2*edges exactly).
//  exact == 0 : exactly `edges` candidates are drawn; duplicates and self loops
//               are dropped afterwards (nnz <= 2*edges).
void* gg_chung_lu_symmetric(int64_t M, double gamma, double max_over_mean, int64_t edges,
                            int exact, uint64_t seed) {
  if (M <= 1 || edges < 0 || M >= (1ll << 31)) return nullptr;
  std::vector<double> cdf;
  powerlaw_cdf(M, gamma, max_over_mean, &cdf);
  std::vector<int32_t> perm;
  permutation(M, seed, ST_PERM_A, &perm);
  std::vector<uint64_t> keys;
  if (exact) {
    std::unordered_set<uint64_t> seen;
    seen.reserve((size_t)edges * 2);
    keys.reserve((size_t)edges * 2);
    for (uint64_t e = 0; (int64_t)seen.size() < edges; ++e) {
      const int64_t u = perm[sample_cdf(cdf, u64_to_unit(rng_u64(seed, ST_EDGE_U, e)))];
      const int64_t v = perm[sample_cdf(cdf, u64_to_unit(rng_u64(seed, ST_EDGE_V, e)))];
      if (u == v) continue;
      const uint64_t a = (uint64_t)std::min(u, v), b = (uint64_t)std::max(u, v);
      if (!seen.insert((a << 32) | b).second) continue;
      keys.push_back((a << 32) | b);
      keys.push_back((b << 32) | a);
    }
  } else {
    keys.resize((size_t)edges * 2);
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < edges; ++e) {
      const uint64_t u = (uint64_t)perm[sample_cdf(cdf, u64_to_unit(rng_u64(seed, ST_EDGE_U, (uint64_t)e)))];
      const uint64_t v = (uint64_t)perm[sample_cdf(cdf, u64_to_unit(rng_u64(seed, ST_EDGE_V, (uint64_t)e)))];
      // a self loop is marked with an impossible key and removed below
      keys[2 * e] = (u == v) ? ~0ull : ((u << 32) | v);
      keys[2 * e + 1] = (u == v) ? ~0ull : ((v << 32) | u);
    }
    keys.erase(std::remove(keys.begin(), keys.end(), ~0ull), keys.end());
  }
  Csr* out = new (std::nothrow) Csr;
  if (!out) return nullptr;
  keys_to_csr(keys, M, M, out);
  return out;
}

// ---- Chung-Lu, directed ----------------------------------------------------
// `edges` candidates (u -> v): the row u from an out-weight sequence and the
// column v from an independent in-weight sequence (own permutation each); self
// loops and duplicates dropped; then every row r with
// rng(seed, EMPTY, r) < empty_frac loses all its entries.
void* gg_chung_lu_directed(int64_t M, double gamma, double max_over_mean_out,
                           double max_over_mean_in, int64_t edges, double empty_frac,
                           uint64_t seed) {
  if (M <= 1 || edges < 0 || M >= (1ll << 31)) return nullptr;
  std::vector<double> cdf_out, cdf_in;
  powerlaw_cdf(M, gamma, max_over_mean_out, &cdf_out);
  powerlaw_cdf(M, gamma, max_over_mean_in, &cdf_in);
  std::vector<int32_t> perm_out, perm_in;
  permutation(M, seed, ST_PERM_A, &perm_out);
  permutation(M, seed, ST_PERM_B, &perm_in);
  std::vector<uint64_t> keys((size_t)edges);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < edges; ++e) {
    const uint64_t u = (uint64_t)perm_out[sample_cdf(cdf_out, u64_to_unit(rng_u64(seed, ST_EDGE_U, (uint64_t)e)))];
    const uint64_t v = (uint64_t)perm_in[sample_cdf(cdf_in, u64_to_unit(rng_u64(seed, ST_EDGE_V, (uint64_t)e)))];
    const bool dropped = (u == v) || (u64_to_unit(rng_u64(seed, ST_EMPTY, u)) < empty_frac);
    keys[e] = dropped ? ~0ull : ((u << 32) | v);
  }
  keys.erase(std::remove(keys.begin(), keys.end(), ~0ull), keys.end());
  Csr* out = new (std::nothrow) Csr;
  if (!out) return nullptr;
  keys_to_csr(keys, M, M, out);
  return out;
}

// ---- R-MAT -----------------------------------------------------------------
// `draws` accepted edges on a 2^scale grid with quadrant probabilities
// (a, b, c, 1-a-b-c); a draw whose row or column is >= M is rejected and
// redrawn with the next attempt number; duplicates merged; rows not permuted;
// then rows with rng(seed, EMPTY, r) < extra_empty_frac are emptied.
void* gg_rmat(int64_t M, int scale, double a, double b, double c, int64_t draws,
              double extra_empty_frac, uint64_t seed) {
  if (M <= 0 || scale < 1 || scale > 30 || (1ll << scale) < M || draws < 0) return nullptr;
  std::vector<uint64_t> keys((size_t)draws);
  const double ab = a + b, abc = a + b + c;
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < draws; ++e) {
    for (uint64_t attempt = 0;; ++attempt) {
      uint64_t row = 0, col = 0;
      for (int level = 0; level < scale; ++level) {
        const double u = u64_to_unit(
            rng_u64(seed, ST_RMAT + (attempt << 8), (uint64_t)e * 64u + (uint64_t)level));
        const unsigned quadrant = (u < a) ? 0u : (u < ab) ? 1u : (u < abc) ? 2u : 3u;
        row = (row << 1) | (quadrant >> 1);
        col = (col << 1) | (quadrant & 1u);
      }
      if ((int64_t)row < M && (int64_t)col < M) {
        const bool dropped = extra_empty_frac > 0.0 &&
                             u64_to_unit(rng_u64(seed, ST_EMPTY, row)) < extra_empty_frac;
        keys[e] = dropped ? ~0ull : ((row << 32) | col);
        break;
      }
    }
  }
  keys.erase(std::remove(keys.begin(), keys.end(), ~0ull), keys.end());
  Csr* out = new (std::nothrow) Csr;
  if (!out) return nullptr;
  keys_to_csr(keys, M, M, out);
  return out;
}

// ---- edge values -----------------------------------------------------------
// Symmetric normalisation of a square adjacency matrix: 1/sqrt(d_i * d_j) with
// d = number of stored entries of the row (computed in double, rounded once).
void gg_vals_sym_norm(int64_t M, const int32_t* rowptr, const int32_t* colind, float* vals) {
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < M; ++i) {
    const double di = (double)(rowptr[i + 1] - rowptr[i]);
    for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
      const int32_t j = colind[p];
      const double dj = (double)(rowptr[j + 1] - rowptr[j]);
      vals[p] = (float)(1.0 / std::sqrt(di * std::max(dj, 1.0)));
    }
  }
}
// uniform (0,1]: (u24 + 1) * 2^-24, exactly representable in fp32
void gg_fill_uniform_01(int64_t n, uint64_t seed, uint64_t stream, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    const uint32_t u24 = (uint32_t)(rng_u64(seed, ST_VALS + (stream << 8), (uint64_t)i) >> 40);
    out[i] = (float)((double)(u24 + 1u) * (1.0 / 16777216.0));
  }
}
// uniform on (-1,1): (2*u24 + 1 - 2^24) * 2^-24, an odd numerator: never zero, exact in fp32
void gg_fill_uniform_pm1(int64_t n, uint64_t seed, uint64_t stream, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    const int64_t u24 = (int64_t)(rng_u64(seed, ST_DENSE + (stream << 8), (uint64_t)i) >> 40);
    out[i] = (float)((double)(2 * u24 + 1 - 16777216) * (1.0 / 16777216.0));
  }
}
// standard normal by Box-Muller (one draw per element, cosine branch), rounded to fp32
void gg_fill_normal(int64_t n, uint64_t seed, uint64_t stream, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    const uint64_t x = rng_u64(seed, ST_DENSE + (stream << 8), 2 * (uint64_t)i);
    const uint64_t y = rng_u64(seed, ST_DENSE + (stream << 8), 2 * (uint64_t)i + 1);
    const double u1 = ((double)(x >> 11) + 1.0) * (1.0 / 9007199254740992.0);  // (0,1]
    const double u2 = u64_to_unit(y);
    float v = (float)(std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586476925 * u2));
    if (v == 0.0f) v = 1.0f / 16777216.0f;
    out[i] = v;
  }
}

int gg_max_threads(void) { return omp_get_max_threads(); }
void gg_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }

}  // extern "C"
