// CPU oracle for frame-parallel GCN neighbour aggregation.  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, plain statement of what the hot path computes.  It exists so that the
// HIP library can be checked element by element; it is never part of the product path, shares no
// code with it, and is only called from tests, the smoke check and the benchmark's CPU-baseline
// leg.
//
// What it follows:
//  * Section 2.1, Eq. 1: a GNN layer aggregates the features of N(v) united with {v}; the GCN
//    aggregation is taken in its symmetric-normalised form A^ = D^-1/2 (A + I) D^-1/2 with
//    D = row sums of A + I.  (The text says "mean"; the symmetric form is the reading fixed for
//    this build.)
//  * Section 4.1 "Overlap-aware data transfer" / Section 4.2 "Dimension-aware parallel GNN": the
//    topology of a snapshot group is regrouped as ONE overlap part shared by all snapshots plus one
//    exclusive part per snapshot.  The overlap is read as the exact set intersection of the
//    directed edge sets of all k snapshots; exclusive_t = E_t minus overlap.
//
// The method reproduces A^_t X_t exactly (overlap + exclusive_t = E_t), so aggregation here is
// the plain definition, one snapshot at a time, with no overlap split at all.
//
// Storage: every snapshot is an edge list of directed (row, col) pairs.  Input lists may be
// unsorted and may hold duplicates and diagonal entries: they are sorted, de-duplicated and the
// diagonal is dropped first (self-loops are implicit and added by the normalisation).
// Arithmetic: double accumulation; weights 1/sqrt(d_i d_j) in double; result rounded to float once.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <utility>
#include <vector>

namespace {

using Edge = std::pair<int32_t, int32_t>;  // (row, col); std::pair orders by row, then col

std::vector<Edge> canonical_edges(int64_t nnz, const int32_t *rows, const int32_t *cols) {
  std::vector<Edge> e;
  e.reserve((size_t)nnz);
  for (int64_t q = 0; q < nnz; ++q)
    if (rows[q] != cols[q]) e.emplace_back(rows[q], cols[q]);
  std::sort(e.begin(), e.end());
  e.erase(std::unique(e.begin(), e.end()), e.end());
  return e;
}

bool in_range(int32_t n, int64_t nnz, const int32_t *rows, const int32_t *cols) {
  for (int64_t q = 0; q < nnz; ++q)
    if (rows[q] < 0 || rows[q] >= n || cols[q] < 0 || cols[q] >= n) return false;
  return true;
}

struct Frame {
  int32_t n = 0, k = 0;
  std::vector<Edge> common;
  std::vector<std::vector<Edge>> excl;
};

void edges_to_csr(int32_t n, const std::vector<Edge> &e, int32_t *rowptr, int32_t *col) {
  for (int32_t i = 0; i <= n; ++i) rowptr[i] = 0;
  for (const Edge &p : e) ++rowptr[p.first + 1];
  for (int32_t i = 0; i < n; ++i) rowptr[i + 1] += rowptr[i];
  for (size_t q = 0; q < e.size(); ++q) col[q] = e[q].second;  // e is sorted by (row, col)
}

}  // namespace

extern "C" {

// ---- overlap / exclusive decomposition (Section 4.1, 4.2) -----------------------------------

// Builds the decomposition of k snapshots given as edge lists (host pointers).
// nnz[t] pairs in rows[t][..], cols[t][..].  Returns an opaque handle, or NULL on bad arguments.
void *pipad_oracle_overlap_create(int32_t n, int32_t k, const int64_t *nnz,
                                  const int32_t *const *rows, const int32_t *const *cols) {
  if (n < 0 || k < 1 || !nnz || !rows || !cols) return nullptr;
  for (int32_t t = 0; t < k; ++t)
    if (nnz[t] < 0 || !in_range(n, nnz[t], rows[t], cols[t])) return nullptr;
  Frame *f = new Frame;
  f->n = n;
  f->k = k;
  std::vector<std::vector<Edge>> snaps((size_t)k);
  for (int32_t t = 0; t < k; ++t) snaps[(size_t)t] = canonical_edges(nnz[t], rows[t], cols[t]);
  // overlap = edges present in every snapshot: fold set_intersection over t
  f->common = snaps[0];
  for (int32_t t = 1; t < k; ++t) {
    std::vector<Edge> next;
    std::set_intersection(f->common.begin(), f->common.end(), snaps[(size_t)t].begin(),
                          snaps[(size_t)t].end(), std::back_inserter(next));
    f->common.swap(next);
  }
  // exclusive_t = E_t \ overlap
  f->excl.resize((size_t)k);
  for (int32_t t = 0; t < k; ++t)
    std::set_difference(snaps[(size_t)t].begin(), snaps[(size_t)t].end(), f->common.begin(),
                        f->common.end(), std::back_inserter(f->excl[(size_t)t]));
  return f;
}

void pipad_oracle_overlap_destroy(void *h) { delete static_cast<Frame *>(h); }

// t = -1: the overlap part; 0 <= t < k: exclusive part of snapshot t.  Returns -1 on bad t.
int64_t pipad_oracle_overlap_nnz(const void *h, int32_t t) {
  const Frame *f = static_cast<const Frame *>(h);
  if (!f || t < -1 || t >= f->k) return -1;
  return (int64_t)(t < 0 ? f->common.size() : f->excl[(size_t)t].size());
}

// Writes the selected part as CSR: rowptr[n+1], col[nnz], columns ascending within a row.
int pipad_oracle_overlap_csr(const void *h, int32_t t, int32_t *rowptr, int32_t *col) {
  const Frame *f = static_cast<const Frame *>(h);
  if (!f || t < -1 || t >= f->k || !rowptr) return -1;
  edges_to_csr(f->n, t < 0 ? f->common : f->excl[(size_t)t], rowptr, col);
  return 0;
}

// ---- aggregation (Eq. 1 with the symmetric GCN normalisation) --------------------------------

// One snapshot: Y = D^-1/2 (A + I) D^-1/2 X with A given as an edge list.
//   X: n rows of F floats, row stride ldx (elements).  Y (float, stride ldy), Yd (double, dense
//   n*F) and B (double, dense n*F) are each optional (NULL to skip):
//     Yd[i][f] = sum_j a^_ij x_jf                (double, unrounded)
//     Y [i][f] = (float) Yd[i][f]
//     B [i][f] = sum_j |a^_ij| |x_jf|            (the scale of the parity tolerance)
//   threads <= 1: single thread.  Otherwise rows are split statically into `threads` ranges.
// Returns the number of threads used (>= 1), or -1 on bad arguments.
int pipad_oracle_aggregate(int32_t n, int64_t nnz, const int32_t *rows, const int32_t *cols,
                           int32_t F, const float *X, int64_t ldx, float *Y, int64_t ldy,
                           double *Yd, double *B, int32_t threads) {
  if (n < 0 || nnz < 0 || F < 1 || ldx < F || (Y && ldy < F)) return -1;
  if (nnz > 0 && (!rows || !cols)) return -1;
  if (n > 0 && !X) return -1;
  if (!in_range(n, nnz, rows, cols)) return -1;
  // A + I as an edge list: canonical off-diagonal pairs plus (i, i) for every i
  std::vector<Edge> e = canonical_edges(nnz, rows, cols);
  for (int32_t i = 0; i < n; ++i) e.emplace_back(i, i);
  std::sort(e.begin(), e.end());
  // d_i = number of pairs in row i (row sum of A + I)
  std::vector<double> d((size_t)n, 0.0);
  for (const Edge &p : e) d[(size_t)p.first] += 1.0;

  const int nthreads = std::max(1, std::min<int>(threads, n > 0 ? n : 1));
  auto work = [&](int32_t row_lo, int32_t row_hi) {
    std::vector<double> acc((size_t)F), bnd((size_t)F);
    auto it = std::lower_bound(e.begin(), e.end(), Edge(row_lo, INT32_MIN));
    for (int32_t i = row_lo; i < row_hi; ++i) {
      std::fill(acc.begin(), acc.end(), 0.0);
      std::fill(bnd.begin(), bnd.end(), 0.0);
      for (; it != e.end() && it->first == i; ++it) {
        const int32_t j = it->second;
        const double w = 1.0 / std::sqrt(d[(size_t)i] * d[(size_t)j]);
        const float *xj = X + (int64_t)j * ldx;
        for (int32_t f = 0; f < F; ++f) {
          acc[(size_t)f] += w * (double)xj[f];
          bnd[(size_t)f] += std::fabs(w) * std::fabs((double)xj[f]);
        }
      }
      for (int32_t f = 0; f < F; ++f) {
        if (Y) Y[(int64_t)i * ldy + f] = (float)acc[(size_t)f];
        if (Yd) Yd[(int64_t)i * F + f] = acc[(size_t)f];
        if (B) B[(int64_t)i * F + f] = bnd[(size_t)f];
      }
    }
  };
  if (nthreads == 1) {
    work(0, n);
  } else {
    std::vector<std::thread> pool;
    for (int w = 0; w < nthreads; ++w) {
      int32_t lo = (int32_t)((int64_t)n * w / nthreads);
      int32_t hi = (int32_t)((int64_t)n * (w + 1) / nthreads);
      pool.emplace_back(work, lo, hi);
    }
    for (auto &th : pool) th.join();
  }
  return nthreads;
}

int pipad_oracle_hardware_threads(void) {
  unsigned c = std::thread::hardware_concurrency();
  return c ? (int)c : 1;
}

}  // extern "C"
