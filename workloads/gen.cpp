// Seeded synthetic inputs for the GCN hot path: graph patterns (CSR, no values),
// dense feature matrices, weights and labels.
//
// This file holds NO arithmetic of the method itself (no normalisation, no
// products): it only draws random structure and numbers.  Both the HIP path
// and the CPU oracle are fed from here; neither shares anything else.
//
// Every random quantity is a pure function of (seed, stream, index) through a
// splitmix64-style integer mix, so any element can be regenerated alone and
// the result does not depend on thread count.
//
// Graph recipes (stand-ins for the paper's Table 1 workloads, which are not
// reproduced here):
//   * Erdos-Renyi G(n,p), undirected, by geometric skipping per row.
//   * Chung-Lu with a truncated power-law expected-degree sequence (degree
//     quantiles, no sampling noise in the sequence), edges by the
//     Miller-Hagberg skipping method, then a random vertex relabelling
//     (the paper balances tiles with a random permutation, section
//     "Permutation").
//   * R-MAT(a,b,c,d) edge draws, symmetrised and deduplicated.
//   * A rectangular "row block" with power-law row degrees and Zipf-like
//     column popularity (one GPU's share of a 1-D row partition, section
//     "Partitioning").
// All patterns come out with sorted, duplicate-free rows and no self-loops
// (the block generator never emits (r,r) either).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
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

inline uint64_t draw(uint64_t seed, uint64_t stream, uint64_t index) {
  return mix64(mix64(mix64(seed) ^ stream) ^ index);
}

// uniform in the open interval (0,1), 53 bits
inline double u01(uint64_t h) { return ((double)(h >> 11) + 0.5) * (1.0 / 9007199254740992.0); }

struct Pattern {
  int64_t n_rows = 0, n_cols = 0;
  std::vector<int64_t> rowptr;
  std::vector<int32_t> colidx;
};

// Directed edge list (possibly with duplicates) -> CSR with sorted unique rows.
void build_csr(int64_t n_rows, int64_t n_cols, const std::vector<int32_t>& src,
               const std::vector<int32_t>& dst, Pattern* out) {
  const int64_t m = (int64_t)src.size();
  std::vector<int64_t> cnt(n_rows + 1, 0);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
#pragma omp atomic
    cnt[src[e] + 1]++;
  }
  for (int64_t i = 0; i < n_rows; ++i) cnt[i + 1] += cnt[i];
  std::vector<int32_t> tmp(m);
  std::vector<int64_t> cur(cnt.begin(), cnt.end() - 1);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    int64_t p;
#pragma omp atomic capture
    p = cur[src[e]]++;
    tmp[p] = dst[e];
  }
  std::vector<int64_t> ucnt(n_rows + 1, 0);
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t i = 0; i < n_rows; ++i) {
    int32_t* b = tmp.data() + cnt[i];
    int32_t* e = tmp.data() + cnt[i + 1];
    std::sort(b, e);
    ucnt[i + 1] = std::unique(b, e) - b;
  }
  for (int64_t i = 0; i < n_rows; ++i) ucnt[i + 1] += ucnt[i];
  out->n_rows = n_rows;
  out->n_cols = n_cols;
  out->rowptr = ucnt;
  out->colidx.resize(ucnt[n_rows]);
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t i = 0; i < n_rows; ++i) {
    std::memcpy(out->colidx.data() + ucnt[i], tmp.data() + cnt[i],
                sizeof(int32_t) * (size_t)(ucnt[i + 1] - ucnt[i]));
  }
}

// Upper-triangle adjacency lists -> both directions, relabelled by perm.
void symmetrise(int64_t n, const std::vector<int64_t>& off, const std::vector<int32_t>& nbr,
                const std::vector<int32_t>& perm, Pattern* out) {
  const int64_t m = off[n];
  std::vector<int32_t> src(2 * m), dst(2 * m);
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t u = 0; u < n; ++u) {
    const int32_t pu = perm.empty() ? (int32_t)u : perm[u];
    for (int64_t k = off[u]; k < off[u + 1]; ++k) {
      const int32_t pv = perm.empty() ? nbr[k] : perm[nbr[k]];
      src[2 * k] = pu; dst[2 * k] = pv;
      src[2 * k + 1] = pv; dst[2 * k + 1] = pu;
    }
  }
  build_csr(n, n, src, dst, out);
}

// Random permutation: rank of a hashed key (ties broken by index).
void random_perm(int64_t n, uint64_t seed, uint64_t stream, std::vector<int32_t>* perm) {
  std::vector<std::pair<uint64_t, int32_t>> key(n);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) key[i] = {draw(seed, stream, (uint64_t)i), (int32_t)i};
  std::sort(key.begin(), key.end());
  perm->resize(n);
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < n; ++r) (*perm)[key[r].second] = (int32_t)r;
}

// Neighbours v>u of row u for expected-degree weights w (descending), total S.
// Emits through f(v).  Skipping method of Miller and Hagberg (2011).
template <class Emit>
inline void chung_lu_row(int64_t u, int64_t n, const double* w, double S, uint64_t seed,
                         Emit&& f) {
  uint64_t t = 0;
  const uint64_t stream = 0x1000000000ull + (uint64_t)u;
  int64_t v = u + 1;
  if (v >= n) return;
  double p = std::min(w[u] * w[v] / S, 1.0);
  while (v < n && p > 0.0) {
    if (p != 1.0) {
      const double r = u01(draw(seed, stream, t++));
      const double skip = std::floor(std::log(r) / std::log1p(-p));
      if (skip >= (double)(n - v)) break;
      v += (int64_t)skip;
    }
    if (v < n) {
      const double q = std::min(w[u] * w[v] / S, 1.0);
      const double r = u01(draw(seed, stream, t++));
      if (r < q / p) f((int32_t)v);
      p = q;
      ++v;
    }
  }
}

// Quantile degree sequence of a power law pdf ~ d^-gamma on [dmin,dmax], descending.
void powerlaw_sequence(int64_t n, double gamma, double dmin, double dmax, double* w) {
  const double e = 1.0 - gamma;
  const double a = std::pow(dmin, e), b = std::pow(dmax, e);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    const double q = 1.0 - ((double)i + 0.5) / (double)n;  // descending degrees
    w[i] = std::pow(a - q * (a - b), 1.0 / e);
  }
}

double powerlaw_mean(int64_t n, double gamma, double dmin, double dmax) {
  std::vector<double> w(n);
  powerlaw_sequence(n, gamma, dmin, dmax, w.data());
  double s = 0;
  for (int64_t i = 0; i < n; ++i) s += w[i];
  return s / (double)n;
}

double solve_dmin(int64_t n, double gamma, double dmax, double mean) {
  double lo = 1e-3, hi = dmax;
  for (int it = 0; it < 60; ++it) {
    const double mid = 0.5 * (lo + hi);
    if (powerlaw_mean(std::min<int64_t>(n, 200000), gamma, mid, dmax) < mean) lo = mid; else hi = mid;
  }
  return 0.5 * (lo + hi);
}

}  // namespace

extern "C" {

struct wl_pattern;  // opaque

int64_t wl_pattern_rows(const wl_pattern* p) { return ((const Pattern*)p)->n_rows; }
int64_t wl_pattern_cols(const wl_pattern* p) { return ((const Pattern*)p)->n_cols; }
int64_t wl_pattern_nnz(const wl_pattern* p) { return (int64_t)((const Pattern*)p)->colidx.size(); }
// rowptr is written as int32 (the library's index type); fails (returns -1) at nnz >= 2^31.
int wl_pattern_export(const wl_pattern* p_, int32_t* rowptr, int32_t* colidx) {
  const Pattern* p = (const Pattern*)p_;
  if (p->colidx.size() >= (size_t)INT32_MAX) return -1;
  for (int64_t i = 0; i <= p->n_rows; ++i) rowptr[i] = (int32_t)p->rowptr[i];
  std::memcpy(colidx, p->colidx.data(), sizeof(int32_t) * p->colidx.size());
  return 0;
}
void wl_pattern_free(wl_pattern* p) { delete (Pattern*)p; }

// Undirected Erdos-Renyi G(n,p).
wl_pattern* wl_erdos_renyi(int64_t n, double p, uint64_t seed) {
  std::vector<int64_t> off(n + 1, 0);
  std::vector<int32_t> nbr;
  const double lq = std::log1p(-p);
  for (int pass = 0; pass < 2; ++pass) {
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t u = 0; u < n; ++u) {
      uint64_t t = 0;
      int64_t v = u, c = 0;
      for (;;) {
        const double r = u01(draw(seed, 0x2000000000ull + (uint64_t)u, t++));
        const double skip = std::floor(std::log(r) / lq);
        if (skip >= (double)(n - v)) break;
        v += 1 + (int64_t)skip;
        if (v >= n) break;
        if (pass) nbr[off[u] + c] = (int32_t)v;
        ++c;
      }
      if (!pass) off[u + 1] = c;
    }
    if (!pass) {
      for (int64_t i = 0; i < n; ++i) off[i + 1] += off[i];
      nbr.resize(off[n]);
    }
  }
  Pattern* out = new Pattern;
  symmetrise(n, off, nbr, {}, out);
  return (wl_pattern*)out;
}

// Chung-Lu, truncated power-law expected degrees; target_nnz counts directed entries.
// relabel != 0 applies a random vertex permutation; 0 keeps degree-descending order.
wl_pattern* wl_chung_lu(int64_t n, double target_nnz, double gamma, double dmax, int relabel,
                        uint64_t seed) {
  const double mean = target_nnz / (double)n;
  const double dmin = solve_dmin(n, gamma, dmax, mean);
  std::vector<double> w(n);
  powerlaw_sequence(n, gamma, dmin, dmax, w.data());
  double S = 0;
  for (int64_t i = 0; i < n; ++i) S += w[i];
  std::vector<int64_t> off(n + 1, 0);
  std::vector<int32_t> nbr;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t u = 0; u < n; ++u) {
    int64_t c = 0;
    chung_lu_row(u, n, w.data(), S, seed, [&](int32_t) { ++c; });
    off[u + 1] = c;
  }
  for (int64_t i = 0; i < n; ++i) off[i + 1] += off[i];
  nbr.resize(off[n]);
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t u = 0; u < n; ++u) {
    int64_t c = off[u];
    chung_lu_row(u, n, w.data(), S, seed, [&](int32_t v) { nbr[c++] = v; });
  }
  std::vector<int32_t> perm;
  if (relabel) random_perm(n, seed, 0x3000000000ull, &perm);
  Pattern* out = new Pattern;
  symmetrise(n, off, nbr, perm, out);
  return (wl_pattern*)out;
}

// R-MAT: n = 2^scale vertices, n_draws undirected edge draws, self-loops dropped,
// symmetrised, deduplicated, randomly relabelled.
wl_pattern* wl_rmat(int scale, int64_t n_draws, double a, double b, double c, uint64_t seed) {
  const int64_t n = (int64_t)1 << scale;
  std::vector<int32_t> perm;
  random_perm(n, seed, 0x3000000000ull, &perm);
  std::vector<int32_t> src(2 * n_draws), dst(2 * n_draws);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < n_draws; ++e) {
    int64_t u = 0, v = 0;
    for (int l = 0; l < scale; ++l) {
      const double r = u01(draw(seed, 0x4000000000ull + (uint64_t)l, (uint64_t)e));
      const int quad = r < a ? 0 : (r < a + b ? 1 : (r < a + b + c ? 2 : 3));
      u = (u << 1) | (quad >> 1);
      v = (v << 1) | (quad & 1);
    }
    if (u == v) v = (u + 1 + (int64_t)(draw(seed, 0x4100000000ull, (uint64_t)e) % (uint64_t)(n - 1))) % n;
    src[2 * e] = perm[u]; dst[2 * e] = perm[v];
    src[2 * e + 1] = perm[v]; dst[2 * e + 1] = perm[u];
  }
  Pattern* out = new Pattern;
  build_csr(n, n, src, dst, out);
  return (wl_pattern*)out;
}

// Rectangular row block: n_rows x n_cols, ~target_nnz entries.  Row degrees follow
// a truncated power law (exponent gamma_r, cap dmax); each entry's column is drawn
// from a Zipf-like popularity (rank^-alpha by inverse CDF) over n_cols, scattered by
// a multiplicative hash so popular columns are not adjacent.  (r,r) is never emitted.
wl_pattern* wl_row_block(int64_t n_rows, int64_t n_cols, double target_nnz, double gamma_r,
                         double dmax, double alpha, uint64_t seed) {
  const double mean = target_nnz / (double)n_rows;
  const double dmin = solve_dmin(n_rows, gamma_r, dmax, mean);
  std::vector<double> w(n_rows);
  powerlaw_sequence(n_rows, gamma_r, dmin, dmax, w.data());
  std::vector<int32_t> perm;
  random_perm(n_rows, seed, 0x3000000000ull, &perm);
  std::vector<int64_t> off(n_rows + 1, 0);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n_rows; ++i) {
    // stochastic rounding keeps the mean
    const double d = w[i];
    const double fl = std::floor(d);
    off[perm[i] + 1] = (int64_t)fl + (u01(draw(seed, 0x5000000000ull, (uint64_t)i)) < d - fl ? 1 : 0);
  }
  for (int64_t i = 0; i < n_rows; ++i) off[i + 1] += off[i];
  const int64_t m = off[n_rows];
  std::vector<int32_t> src(m), dst(m);
  const double e1 = 1.0 - alpha;
  const double hiN = std::pow((double)n_cols + 1.0, e1);
  // odd multiplier coprime with n_cols for most sizes; map rank -> column
  const uint64_t mult = 0x9E3779B97F4A7C15ull % (uint64_t)n_cols | 1ull;
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t r = 0; r < n_rows; ++r) {
    for (int64_t k = off[r]; k < off[r + 1]; ++k) {
      const double u = u01(draw(seed, 0x6000000000ull, (uint64_t)k));
      // inverse CDF of pdf ~ x^-alpha on [1, n_cols+1)
      double x = std::pow(1.0 + u * (hiN - 1.0), 1.0 / e1);
      int64_t rank = (int64_t)x - 1;
      if (rank < 0) rank = 0;
      if (rank >= n_cols) rank = n_cols - 1;
      int64_t col = (int64_t)(((unsigned __int128)rank * mult) % (uint64_t)n_cols);
      if (col == r) col = (col + 1) % n_cols;
      src[k] = (int32_t)r;
      dst[k] = (int32_t)col;
    }
  }
  Pattern* out = new Pattern;
  build_csr(n_rows, n_cols, src, dst, out);
  return (wl_pattern*)out;
}

// out[i] ~ N(0,1), i = first..first+count-1 of the (seed,stream) sequence.  Box-Muller
// in double on two uniforms per value, rounded once to fp32.
void wl_normal_f32(uint64_t seed, uint64_t stream, int64_t first, int64_t count, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    const uint64_t j = (uint64_t)(first + i);
    const double u1 = u01(draw(seed, stream, 2 * j));
    const double u2 = u01(draw(seed, stream, 2 * j + 1));
    out[i] = (float)(std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586476925 * u2));
  }
}

// out[i] ~ U(lo,hi)
void wl_uniform_f32(uint64_t seed, uint64_t stream, int64_t first, int64_t count, double lo,
                    double hi, float* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i)
    out[i] = (float)(lo + (hi - lo) * u01(draw(seed, stream, (uint64_t)(first + i))));
}

// out[i] uniform over {0..n_classes-1}
void wl_labels_i32(uint64_t seed, uint64_t stream, int64_t count, int32_t n_classes, int32_t* out) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i)
    out[i] = (int32_t)(draw(seed, stream, (uint64_t)i) % (uint64_t)n_classes);
}

}  // extern "C"
