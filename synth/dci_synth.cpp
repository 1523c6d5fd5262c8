// Seeded synthetic inputs for the dual-cache GNN inference path: R-MAT graphs in
// CSR-by-destination form, Gaussian feature rows, distinct seed (test) nodes and
// Glorot-uniform layer weights.
//
// This file holds input generators only.  It contains none of the method's
// arithmetic (no sampling, counting, cache filling, gathering or model code) and
// is used by both the CPU oracle's tests and the GPU path's tests so that both
// see identical bytes.  Its random numbers come from a splitmix64-style counter
// hash, deliberately unrelated to the Philox generator the sampler is defined on.
//
// Every value is a pure function of (seed, index), so results do not depend on
// the number of worker threads.
//
// Shapes follow the paper's dataset table (Table II: node / edge / feature /
// class counts) with a power-law degree profile standing in for the real graphs.

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// One 64-bit word per (seed, a, b) triple.
inline uint64_t word(uint64_t seed, uint64_t a, uint64_t b) {
  return mix64(mix64(seed ^ mix64(a)) ^ (b * 0xD6E8FEB86659FD93ull));
}

struct Perm {  // seeded bijection of [0, n) by a 4-round Feistel network + cycle walking
  uint64_t n, seed, half_mask;
  int half_bits;
  Perm(uint64_t n_, uint64_t seed_) : n(n_), seed(seed_) {
    int bits = 1;
    while ((1ull << bits) < n) ++bits;
    half_bits = (bits + 1) / 2;
    half_mask = (1ull << half_bits) - 1;
  }
  inline uint64_t once(uint64_t x) const {
    uint64_t l = x >> half_bits, r = x & half_mask;
    for (int round = 0; round < 4; ++round) {
      uint64_t f = word(seed, r, (uint64_t)round) & half_mask;
      uint64_t nl = r, nr = l ^ f;
      l = nl;
      r = nr;
    }
    return (l << half_bits) | r;
  }
  inline uint64_t operator()(uint64_t x) const {
    uint64_t y = once(x);
    while (y >= n) y = once(y);
    return y;
  }
};

struct Rmat {
  int64_t N;
  int scale;
  uint32_t ta, tb, tc;  // cumulative 16-bit thresholds of quadrants a, b, c
  uint64_t seed;
  Perm perm;
  Rmat(int64_t N_, double a, double b, double c, uint64_t seed_)
      : N(N_), seed(seed_), perm((uint64_t)N_, seed_ ^ 0x5bd1e995ull) {
    scale = 1;
    while ((1ll << scale) < N) ++scale;
    ta = (uint32_t)std::llround(a * 65536.0);
    tb = (uint32_t)std::llround((a + b) * 65536.0);
    tc = (uint32_t)std::llround((a + b + c) * 65536.0);
  }
  // Edge i as (src, dst) after the vertex relabel.  An attempt whose raw endpoint
  // falls outside [0, N) is redrawn with the next attempt number.
  inline void edge(int64_t i, int64_t* src, int64_t* dst) const {
    for (uint64_t attempt = 0;; ++attempt) {
      uint64_t s = 0, d = 0, w = 0;
      for (int level = 0; level < scale; ++level) {
        if ((level & 3) == 0) w = word(seed, (uint64_t)i, attempt * 8 + (uint64_t)(level >> 2));
        uint32_t r = (uint32_t)(w & 0xFFFF);
        w >>= 16;
        uint64_t sb, db;
        if (r < ta) { sb = 0; db = 0; }
        else if (r < tb) { sb = 0; db = 1; }
        else if (r < tc) { sb = 1; db = 0; }
        else { sb = 1; db = 1; }
        s = (s << 1) | sb;
        d = (d << 1) | db;
      }
      if ((int64_t)s < N && (int64_t)d < N) {
        *src = (int64_t)perm(s);
        *dst = (int64_t)perm(d);
        return;
      }
    }
  }
};

template <class Fn>
void parallel_chunks(int64_t n, int nthreads, int64_t chunk, Fn fn) {
  if (nthreads < 1) nthreads = 1;
  std::atomic<int64_t> next(0);
  auto worker = [&]() {
    for (;;) {
      int64_t lo = next.fetch_add(chunk);
      if (lo >= n) break;
      int64_t hi = std::min(n, lo + chunk);
      fn(lo, hi);
    }
  };
  std::vector<std::thread> pool;
  for (int t = 1; t < nthreads; ++t) pool.emplace_back(worker);
  worker();
  for (auto& th : pool) th.join();
}

}  // namespace

extern "C" {

// R-MAT multigraph with exactly E directed edges (duplicates and self loops kept),
// stored by destination: the in-neighbours of node v are
// indices[indptr[v] .. indptr[v+1]), sorted ascending.  Returns 0, or -1 on bad
// arguments.
int32_t synth_rmat_csr(int64_t N, int64_t E, double a, double b, double c, uint64_t seed,
                       int64_t* indptr, int64_t* indices, int32_t nthreads) {
  if (N <= 0 || E < 0 || !indptr || (!indices && E > 0) || a < 0 || b < 0 || c < 0 || a + b + c > 1.0)
    return -1;
  Rmat g(N, a, b, c, seed);
  std::memset(indptr, 0, sizeof(int64_t) * (size_t)(N + 1));
  // pass 1: in-degree histogram
  parallel_chunks(E, nthreads, 1 << 16, [&](int64_t lo, int64_t hi) {
    for (int64_t i = lo; i < hi; ++i) {
      int64_t s, d;
      g.edge(i, &s, &d);
      __atomic_fetch_add(&indptr[d + 1], 1, __ATOMIC_RELAXED);
    }
  });
  for (int64_t v = 0; v < N; ++v) indptr[v + 1] += indptr[v];
  // pass 2: scatter (order within a list is fixed by the sort below)
  std::vector<int64_t> cursor(indptr, indptr + N);
  int64_t* cur = cursor.data();
  parallel_chunks(E, nthreads, 1 << 16, [&](int64_t lo, int64_t hi) {
    for (int64_t i = lo; i < hi; ++i) {
      int64_t s, d;
      g.edge(i, &s, &d);
      int64_t at = __atomic_fetch_add(&cur[d], 1, __ATOMIC_RELAXED);
      indices[at] = s;
    }
  });
  parallel_chunks(N, nthreads, 1 << 10, [&](int64_t lo, int64_t hi) {
    for (int64_t v = lo; v < hi; ++v) std::sort(indices + indptr[v], indices + indptr[v + 1]);
  });
  return 0;
}

// fp32 rows ~ N(0,1) (Box-Muller on two hashed uniforms per pair of values).
int32_t synth_features(int64_t N, int32_t F, uint64_t seed, float* out, int32_t nthreads) {
  if (N < 0 || F <= 0 || !out) return -1;
  const int64_t total = N * (int64_t)F;
  const int64_t pairs = (total + 1) / 2;
  parallel_chunks(pairs, nthreads, 1 << 16, [&](int64_t lo, int64_t hi) {
    for (int64_t p = lo; p < hi; ++p) {
      uint64_t w0 = word(seed, (uint64_t)p, 0), w1 = word(seed, (uint64_t)p, 1);
      double u0 = ((double)(w0 >> 11) + 1.0) * (1.0 / 9007199254740993.0);  // (0,1)
      double u1 = (double)(w1 >> 11) * (1.0 / 9007199254740992.0);          // [0,1)
      double r = std::sqrt(-2.0 * std::log(u0));
      double t = 6.283185307179586476925286766559 * u1;
      out[2 * p] = (float)(r * std::cos(t));
      if (2 * p + 1 < total) out[2 * p + 1] = (float)(r * std::sin(t));
    }
  });
  return 0;
}

// S distinct node ids, uniform over [0, N): the first S images of a seeded bijection.
int32_t synth_seeds(int64_t N, int64_t S, uint64_t seed, int64_t* out) {
  if (N <= 0 || S < 0 || S > N || !out) return -1;
  Perm p((uint64_t)N, seed);
  for (int64_t i = 0; i < S; ++i) out[i] = (int64_t)p((uint64_t)i);
  return 0;
}

// Glorot-uniform [rows, cols] matrix: U(-a, a), a = sqrt(6 / (rows + cols)).
// `stream` separates the matrices drawn from one seed.
int32_t synth_glorot(int64_t rows, int64_t cols, uint64_t seed, uint64_t stream, float* out) {
  if (rows <= 0 || cols <= 0 || !out) return -1;
  const double a = std::sqrt(6.0 / (double)(rows + cols));
  for (int64_t i = 0; i < rows * cols; ++i) {
    double u = (double)(word(seed ^ mix64(stream + 0x1234), (uint64_t)i, 7) >> 11) * (1.0 / 9007199254740992.0);
    out[i] = (float)((2.0 * u - 1.0) * a);
  }
  return 0;
}

// U(-a, a) vector (used for biases so that they are not all zero).
int32_t synth_uniform(int64_t n, double a, uint64_t seed, uint64_t stream, float* out) {
  if (n < 0 || !out) return -1;
  for (int64_t i = 0; i < n; ++i) {
    double u = (double)(word(seed ^ mix64(stream + 0x9876), (uint64_t)i, 11) >> 11) * (1.0 / 9007199254740992.0);
    out[i] = (float)((2.0 * u - 1.0) * a);
  }
  return 0;
}

}  // extern "C"
