// Seeded synthetic dynamic-graph generator (host only, no method arithmetic).
//
// Produces the inputs that both the CPU oracle and the HIP path are fed with: a sequence of
// undirected, duplicate-free, loop-free graph snapshots in canonical CSR (both directions stored,
// columns strictly ascending) and dense fp32 feature matrices.  They stand in for the dynamic
// graph datasets of the paper's Table 1 (power-law social / e-commerce graphs whose topology
// changes slowly between adjacent snapshots, Section 3.1 "Topology overlap").
//
// Nothing here normalises, intersects or aggregates anything: it only draws random structure.
//
// Random numbers: one documented generator so that seeds reproduce across compilers.
//   next()  : splitmix64 (state += 0x9E3779B97F4A7C15; output = finaliser of the state)
//   u01()   : (next() >> 11) * 2^-53, a double in [0,1)
//   below(n): multiply-high of next() by n (tiny bias < n/2^64, irrelevant here)
//   feature : value(seed, t, idx) = ((mix(key) >> 40) - 2^23) * 2^-23, 24 random bits mapped to
//             a float in [-1, 1) that is exactly representable, key = seed, t, idx hashed together.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

struct Rng {
  uint64_t s;
  explicit Rng(uint64_t seed) : s(mix64(seed ^ 0xD1B54A32D192ED03ull)) {}
  uint64_t next() {
    s += 0x9E3779B97F4A7C15ull;
    return mix64(s);
  }
  double u01() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
  uint64_t below(uint64_t n) { return (uint64_t)(((unsigned __int128)next() * n) >> 64); }
};

// Open-addressing set of 64-bit edge keys (lo << 32 | hi with lo < hi).
struct EdgeSet {
  std::vector<uint64_t> tab;
  uint64_t mask = 0;
  static constexpr uint64_t EMPTY = ~0ull;
  void reset(size_t expect) {
    size_t cap = 64;
    while (cap < expect * 2 + 16) cap <<= 1;
    tab.assign(cap, EMPTY);
    mask = cap - 1;
  }
  // returns true when the key was absent (and is now present)
  bool insert(uint64_t key) {
    uint64_t h = mix64(key) & mask;
    while (true) {
      uint64_t v = tab[h];
      if (v == EMPTY) { tab[h] = key; return true; }
      if (v == key) return false;
      h = (h + 1) & mask;
    }
  }
};

inline uint64_t edge_key(uint32_t a, uint32_t b) {
  return a < b ? ((uint64_t)a << 32) | b : ((uint64_t)b << 32) | a;
}

// Endpoint samplers ---------------------------------------------------------------------------

// Chung-Lu: both endpoints drawn independently with probability proportional to the expected
// degree w_i = c * (i + i0)^(-1/(gamma-1)); i0 is the smallest offset with w_max <= sqrt(sum w),
// the usual condition for the model's edge probabilities w_i w_j / sum w to stay below one.
struct ChungLu {
  std::vector<double> prob;     // alias table (Vose)
  std::vector<uint32_t> alias;
  uint32_t n = 0;
  void init(uint32_t n_, double gamma, double mean_deg) {
    n = n_;
    const double alpha = 1.0 / (gamma - 1.0);
    const double total = (double)n * mean_deg;
    auto wsum = [&](double i0) {
      double s = 0.0;
      for (uint32_t i = 0; i < n; ++i) s += std::pow((double)i + i0, -alpha);
      return s;
    };
    auto ok = [&](double i0) {
      double c = total / wsum(i0);
      return c * std::pow(i0, -alpha) <= std::sqrt(total);
    };
    double lo = 1.0, hi = 1.0;
    if (!ok(lo)) {
      hi = 2.0;
      while (!ok(hi)) hi *= 2.0;
      for (int it = 0; it < 40; ++it) {
        double mid = 0.5 * (lo + hi);
        if (ok(mid)) hi = mid; else lo = mid;
      }
    }
    const double i0 = hi;
    std::vector<double> w(n);
    double s = 0.0;
    for (uint32_t i = 0; i < n; ++i) { w[i] = std::pow((double)i + i0, -alpha); s += w[i]; }
    // Vose alias construction on p_i * n
    prob.assign(n, 0.0);
    alias.assign(n, 0);
    std::vector<uint32_t> small, large;
    small.reserve(n); large.reserve(n);
    for (uint32_t i = 0; i < n; ++i) {
      w[i] = w[i] / s * (double)n;
      (w[i] < 1.0 ? small : large).push_back(i);
    }
    while (!small.empty() && !large.empty()) {
      uint32_t a = small.back(); small.pop_back();
      uint32_t g = large.back(); large.pop_back();
      prob[a] = w[a]; alias[a] = g;
      w[g] = (w[g] + w[a]) - 1.0;
      (w[g] < 1.0 ? small : large).push_back(g);
    }
    for (uint32_t i : large) { prob[i] = 1.0; alias[i] = i; }
    for (uint32_t i : small) { prob[i] = 1.0; alias[i] = i; }
  }
  uint32_t draw(Rng &r) const {
    uint32_t i = (uint32_t)r.below(n);
    return r.u01() < prob[i] ? i : alias[i];
  }
  void draw_edge(Rng &r, uint32_t &u, uint32_t &v) const { u = draw(r); v = draw(r); }
};

// R-MAT: recursive quadrant choice with probabilities (a, b, c, d) on a 2^scale grid.
struct Rmat {
  double a = 0, ab = 0, abc = 0;
  int scale = 0;
  void init(uint32_t n, double a_, double b_, double c_) {
    a = a_; ab = a_ + b_; abc = a_ + b_ + c_;
    scale = 0;
    while ((1ull << scale) < n) ++scale;
  }
  void draw_edge(Rng &r, uint32_t &u, uint32_t &v) const {
    uint32_t x = 0, y = 0;
    for (int l = 0; l < scale; ++l) {
      double p = r.u01();
      uint32_t bx = p >= ab ? 1u : 0u;             // lower half of the quadrant grid (c or d)
      uint32_t by = (p >= a && p < ab) || p >= abc ? 1u : 0u;  // right half (b or d)
      x = (x << 1) | bx;
      y = (y << 1) | by;
    }
    u = x; v = y;
  }
};

template <class Model>
void add_fresh_edges(const Model &m, Rng &r, uint32_t n, size_t count, EdgeSet &set,
                     std::vector<uint64_t> &edges) {
  size_t added = 0;
  while (added < count) {
    uint32_t u, v;
    m.draw_edge(r, u, v);
    if (u >= n || v >= n || u == v) continue;
    uint64_t key = edge_key(u, v);
    if (!set.insert(key)) continue;
    edges.push_back(key);
    ++added;
  }
}

void emit_csr(uint32_t n, const std::vector<uint64_t> &edges, int32_t *rowptr, int32_t *col) {
  std::vector<int64_t> cnt((size_t)n + 1, 0);
  for (uint64_t k : edges) {
    ++cnt[(uint32_t)(k >> 32) + 1];
    ++cnt[(uint32_t)k + 1];
  }
  for (uint32_t i = 0; i < n; ++i) cnt[i + 1] += cnt[i];
  for (uint32_t i = 0; i <= n; ++i) rowptr[i] = (int32_t)cnt[i];
  std::vector<int64_t> pos(cnt.begin(), cnt.end() - 1);
  for (uint64_t k : edges) {
    uint32_t a = (uint32_t)(k >> 32), b = (uint32_t)k;
    col[pos[a]++] = (int32_t)b;
    col[pos[b]++] = (int32_t)a;
  }
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < (int64_t)n; ++i) std::sort(col + rowptr[i], col + rowptr[i + 1]);
}

template <class Model>
int run(const Model &m, uint32_t n, int64_t n_edges, int n_snap, int64_t churn_edges,
        uint64_t seed, int32_t *rowptr_out, int32_t *col_out) {
  Rng r(seed);
  EdgeSet set;
  std::vector<uint64_t> edges;
  edges.reserve((size_t)n_edges);
  set.reset((size_t)n_edges);
  add_fresh_edges(m, r, n, (size_t)n_edges, set, edges);
  for (int t = 0; t < n_snap; ++t) {
    if (t > 0 && churn_edges > 0) {
      // remove a uniform random subset (partial Fisher-Yates to the front), then refill
      for (int64_t q = 0; q < churn_edges; ++q) {
        size_t pick = (size_t)q + (size_t)r.below((uint64_t)(n_edges - q));
        std::swap(edges[(size_t)q], edges[pick]);
      }
      edges.erase(edges.begin(), edges.begin() + churn_edges);
      set.reset((size_t)n_edges);
      for (uint64_t k : edges) set.insert(k);
      add_fresh_edges(m, r, n, (size_t)churn_edges, set, edges);
    }
    emit_csr(n, edges, rowptr_out + (size_t)t * ((size_t)n + 1),
             col_out + (size_t)t * (size_t)(2 * n_edges));
  }
  return 0;
}

}  // namespace

extern "C" {

// model 0: Chung-Lu (p0 = power-law exponent gamma, p1 = mean degree)
// model 1: R-MAT    (p0 = a, p1 = b, p2 = c; d = 1 - a - b - c)
// Writes n_snap CSRs back to back: rowptr_out[n_snap][n+1], col_out[n_snap][2*n_edges].
// Snapshot t+1 = snapshot t minus churn_edges uniformly chosen undirected edges plus the same
// number of fresh edges of the same model that are absent after the removal.
// Returns 0, or -1 on invalid arguments.
int pipad_synth_graphs(int model, int32_t n, int64_t n_edges, int32_t n_snap, int64_t churn_edges,
                       double p0, double p1, double p2, uint64_t seed, int32_t *rowptr_out,
                       int32_t *col_out) {
  if (n < 2 || n_edges < 0 || n_snap < 1 || churn_edges < 0 || churn_edges > n_edges) return -1;
  if (2 * n_edges >= (int64_t)1 << 31) return -1;
  if ((double)n_edges > 0.25 * (double)n * ((double)n - 1.0)) return -1;  // rejection would stall
  if (!rowptr_out || (n_edges > 0 && !col_out)) return -1;
  if (model == 0) {
    ChungLu m;
    m.init((uint32_t)n, p0, p1);
    return run(m, (uint32_t)n, n_edges, n_snap, churn_edges, seed, rowptr_out, col_out);
  }
  if (model == 1) {
    Rmat m;
    m.init((uint32_t)n, p0, p1, p2);
    return run(m, (uint32_t)n, n_edges, n_snap, churn_edges, seed, rowptr_out, col_out);
  }
  return -1;
}

// Fills out[count] with the features idx0 .. idx0+count-1 of stream (seed, t): iid, uniform on
// the 2^24 floats m * 2^-23 - 1 (m = 0 .. 2^24-1), i.e. [-1, 1).  Counter based, so any slice
// can be produced independently and in parallel.
void pipad_synth_features(uint64_t seed, int32_t t, int64_t idx0, int64_t count, float *out) {
  const uint64_t stream = mix64(seed * 0x9E3779B97F4A7C15ull + (uint64_t)(uint32_t)t + 1ull);
#pragma omp parallel for schedule(static)
  for (int64_t q = 0; q < count; ++q) {
    uint64_t h = mix64(stream ^ ((uint64_t)(idx0 + q) * 0xD6E8FEB86659FD93ull));
    int32_t m = (int32_t)(h >> 40);  // 24 bits
    out[q] = (float)(m - 8388608) * (1.0f / 8388608.0f);
  }
}

}  // extern "C"
