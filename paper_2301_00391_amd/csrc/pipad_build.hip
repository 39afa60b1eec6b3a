// pipad_frame_build_overlap: overlap extraction for a frame of k CSR snapshots on gfx950.
//
// Section 4.1 ("Overlap-aware data transfer") regroups the topology of a snapshot group as one
// overlap part plus one exclusive part per snapshot; Section 4.3 makes this the job of a data
// preparation module that runs once.  Here it runs on the GPU, edge-parallel, in five steps:
//
//   mark     one lane per stored entry of snapshot 0: find its row, then binary-search its column
//            in the same row of every other snapshot.  An entry found everywhere is a common
//            edge: a flag is set for it at the position where each snapshot holds it (a byte
//            per stored entry, packed into one bit per entry afterwards).
//   count    popcount per 64-entry word of every output part (common = set bits of snapshot 0's
//            bitmap, delta_t = clear bits of snapshot t's bitmap) and one exclusive prefix sum
//            over all words.
//   rowptr   output row pointers are read off the prefix sums at the input row starts.
//   scatter  every selected entry is written to prefix[word] + (set bits below it in its word),
//            which keeps the ascending column order of the input (stable compaction); the
//            per-entry column scales are written alongside.
//   lists    rows binned by length into the work lists of the aggregation (short, mid, hub; very
//            long rows cut into units), and the entries of the hub rows stored a second time,
//            grouped by column class, with their scales.
//
// All integer work; the outputs are unique, so they are bit-exact regardless of scheduling (the
// marks are plain byte stores with one writer each; the only atomics are integer additions that
// sum up sizes).
#include <algorithm>
#include <cstring>

#include "pipad_internal.h"

#ifndef PIPAD_DENSE_FACTOR
#define PIPAD_DENSE_FACTOR 3  // exclusive entries from all / this on take the lane-per-entry scatter
#endif

namespace pipad {
namespace {

struct Snaps {
  const int32_t *rowptr[PIPAD_MAX_K];
  const int32_t *col[PIPAD_MAX_K];
  int32_t nnz[PIPAD_MAX_K];
};

struct Parts {  // part 0 = common (from snapshot 0), part 1+t = delta_t
  uint64_t *bits[PIPAD_MAX_K];       // bitmap of snapshot t, ceil(nnz_t/64) words
  uint8_t *flag8[PIPAD_MAX_K];       // t >= 1: one byte per stored entry, set by k_mark
  uint32_t word_off[PIPAD_MAX_K + 2];  // first word of each part in the concatenated prefix array
  int32_t *rowptr_out[PIPAD_MAX_K + 1];
  int32_t *col_out[PIPAD_MAX_K + 1];
  float *wc[PIPAD_MAX_K];  // column scales of the common entries, one array per snapshot
  float *wd[PIPAD_MAX_K];  // column scales of the exclusive entries of snapshot t
};

__host__ __device__ inline int part_snapshot(int part) { return part == 0 ? 0 : part - 1; }

// Selected entries of word w of a part, as a bit mask.
__device__ inline uint64_t selected_word(const Parts &p, const Snaps &s, int part, uint32_t w) {
  const int t = part_snapshot(part);
  uint64_t b = p.bits[t][w];
  if (part == 0) return b;
  const int64_t left = (int64_t)s.nnz[t] - (int64_t)w * 64;
  const uint64_t valid = left >= 64 ? ~0ull : ((1ull << left) - 1ull);
  return ~b & valid;
}

// ---- validation -----------------------------------------------------------------------------
// One wave per (snapshot, row): row pointer sanity, then column range / order / diagonal.
__global__ __launch_bounds__(kBlock) void k_validate(Snaps s, int32_t n, int32_t k, int *bad) {
  const int64_t unit = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  const int lane = threadIdx.x % kWave;
  if (unit >= (int64_t)k * n) return;
  // (one unit per wave: saying so lets the snapshot's pointers come through the scalar unit)
  const int t = __builtin_amdgcn_readfirstlane((int)(unit / n));
  const int32_t i = __builtin_amdgcn_readfirstlane((int32_t)(unit % n));
  const int32_t *rp = s.rowptr[t];
  const int32_t a = rp[i], b = rp[i + 1];
  bool ok = a >= 0 && b >= a && b <= s.nnz[t];
  if (i == 0 && a != 0) ok = false;
  if (i == n - 1 && b != s.nnz[t]) ok = false;
  if (ok) {
    const int32_t *col = s.col[t];
    for (int32_t e = a + lane; e < b; e += kWave) {
      const int32_t c = col[e];
      if (c < 0 || c >= n || c == i) ok = false;
      if (e > a && col[e - 1] >= c) ok = false;
    }
  }
  if (!ok) *bad = 1;
}

// ---- mark -----------------------------------------------------------------------------------
// Last row i in [lo, hi] with rowptr[i] <= e, given rowptr[lo] <= e < rowptr[hi + 1].
__device__ inline int32_t row_of_entry(const int32_t *rp, int32_t lo, int32_t hi, int32_t e) {
  while (lo < hi) {
    const int32_t mid = lo + ((hi - lo + 1) >> 1);
    if (rp[mid] <= e) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Position of column c in the ascending run col[a, b), or -1, given that col[g] == v != c for some
// g in [a, b).  The search gallops outwards from g, so it costs O(log distance): adjacent
// snapshots differ in few entries, so the offset of a column within its row barely moves from one
// snapshot to the next.
__device__ inline int32_t gallop_from(const int32_t *col, int32_t a, int32_t b, int32_t g,
                                      int32_t v, int32_t c) {
  int32_t lo, hi;  // the answer, if any, is the lower bound of c within [lo, hi)
  if (v < c) {
    int32_t prev = g, step = 1, cur;
    while (true) {
      cur = g + step;
      if (cur >= b) { cur = b; break; }
      if (col[cur] >= c) break;
      prev = cur;
      step <<= 1;
    }
    lo = prev + 1;
    hi = cur;
  } else {
    int32_t next = g, step = 1, cur;
    while (true) {
      cur = g - step;
      if (cur < a) { cur = a - 1; break; }
      if (col[cur] < c) break;
      next = cur;
      step <<= 1;
    }
    lo = cur + 1;
    hi = next;
  }
  while (lo < hi) {
    const int32_t mid = lo + ((hi - lo) >> 1);
    if (col[mid] < c) lo = mid + 1; else hi = mid;
  }
  return (lo < b && col[lo] == c) ? lo : -1;
}

// wave_row[w] = row that holds entry 64*w of snapshot 0, for w in [0, ceil(nnz0/64)); one extra
// slot at the end receives n - 1.  One thread per row writes the (usually zero or one) slots whose
// entry falls into its row, so k_mark needs no search over the whole row-pointer array.
__global__ __launch_bounds__(kBlock) void k_wave_rows(const int32_t *rp0, int32_t n, int32_t nnz0,
                                                       int32_t *wave_row) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  const int32_t a = rp0[i], b = rp0[i + 1];
  for (int64_t w = ((int64_t)a + kWave - 1) / kWave; w * kWave < b; ++w) wave_row[w] = (int32_t)i;
  if (i == n - 1) wave_row[((int64_t)nnz0 + kWave - 1) / kWave] = n - 1;
}

// One lane per stored entry of snapshot 0.  The row of a wave's first entry and an upper bound for
// the row of its last one come from wave_row; every lane then only searches between those two.
//
// Finding the entries' columns in the other snapshots: the 64 entries of a wave are a contiguous
// stretch of snapshot 0 in (row, column) order, so their matches lie in a contiguous stretch of
// every other snapshot, about as long and - adjacent snapshots differ little - at about the same
// offset from the start of the first lane's row.  The wave stages that stretch (kMarkWindow
// columns per snapshot, two coalesced loads) in LDS and every lane searches its own row's part of
// the window there.  A lane whose row reaches beyond the window on a side where its column could
// lie falls back to probing global memory: first at the same relative offset, then galloping.
constexpr int kMarkGroup = 8;     // snapshots staged together (bounds registers and LDS)
constexpr int kMarkWindow = 128;  // columns per snapshot staged by a wave
constexpr int kMarkMargin = 32;   // window columns in front of the first lane's guessed place

template <int KMAX>
__global__ __launch_bounds__(kBlock) void k_mark(Snaps s, Parts p, int32_t n, int32_t k,
                                                  const int32_t *wave_row) {
  __shared__ int32_t win[kWavesPerBlock][kMarkGroup][kMarkWindow];
  const int64_t e64 = (int64_t)blockIdx.x * kBlock + threadIdx.x;  // wave-aligned: 64 | kBlock
  const int lane = threadIdx.x % kWave;
  const int wv = threadIdx.x / kWave;
  const int32_t nnz0 = s.nnz[0];
  const bool in = e64 < nnz0;
  const int32_t e = in ? (int32_t)e64 : nnz0 - 1;
  const int32_t *rp0 = s.rowptr[0];
  const int64_t nwaves0 = ((int64_t)nnz0 + kWave - 1) / kWave;
  const int64_t w = min(e64 / kWave, nwaves0 - 1);  // waves past the end repeat the last one
  // (clamped, so that a row-pointer array that is not a valid offset array cannot send the search
  // out of range: its slots may then be unwritten)
  const int32_t r_first = min(max(wave_row[w], 0), n - 1);
  const int32_t r_last = min(max(wave_row[w + 1], r_first), n - 1);  // next wave's first row, or n - 1
  const int32_t c = s.col[0][e];
  // Row of the entry: the wave stages the row pointers of its candidate rows in LDS (one round
  // trip to memory instead of one per step of a search) when they are few enough.
  int32_t i, row_start;
  const int32_t nrows = r_last - r_first + 1;
  if (nrows == 1) {
    i = r_first;
    row_start = rp0[i];
  } else if (nrows < kMarkWindow) {
    int32_t *rs = win[wv][0];
    const int32_t a0 = r_first + lane, a1 = a0 + kWave;
    rs[lane] = a0 <= r_last ? rp0[a0] : INT32_MAX;
    rs[lane + kWave] = a1 <= r_last ? rp0[a1] : INT32_MAX;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    int32_t cnt = 0;  // number of staged row pointers <= e (at least 1, fewer than kMarkWindow)
#pragma unroll
    for (int step = kMarkWindow / 2; step >= 1; step >>= 1)
      if (rs[cnt + step - 1] <= e) cnt += step;
    cnt = max(cnt, 1);
    i = r_first + cnt - 1;
    row_start = rs[cnt - 1];
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  } else {
    i = row_of_entry(rp0, r_first, r_last, e);
    row_start = rp0[i];
  }
  const int32_t rel = e - row_start;  // offset of the entry within its row: the first guess
  bool found = in;
  int32_t pos[KMAX];
#pragma unroll
  for (int t = 0; t < KMAX; ++t) pos[t] = 0;
  constexpr int G = kMarkGroup, W = kMarkWindow;
#pragma unroll
  for (int t0 = 1; t0 < KMAX; t0 += G) {
    if (t0 < k && __any(found)) {
      int32_t lo[G], hi[G], P[G];
      {
        int32_t v0[G], v1[G];
#pragma unroll
        for (int u = 0; u < G; ++u) {
          const int t = t0 + u;
          lo[u] = hi[u] = P[u] = 0;
          v0[u] = v1[u] = INT32_MAX;
          if (t < KMAX && t < k) {
            lo[u] = s.rowptr[t][i];
            hi[u] = s.rowptr[t][i + 1];
          }
        }
#pragma unroll
        for (int u = 0; u < G; ++u) {
          const int t = t0 + u;
          if (t < KMAX && t < k) {
            P[u] = max(__shfl(lo[u] + rel, 0) - kMarkMargin, 0);
            const int32_t a0 = P[u] + lane, a1 = a0 + kWave;
            if (a0 < s.nnz[t]) v0[u] = s.col[t][a0];
            if (a1 < s.nnz[t]) v1[u] = s.col[t][a1];
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");  // earlier readers of win are done
#pragma unroll
        for (int u = 0; u < G; ++u) {
          win[wv][u][lane] = v0[u];
          win[wv][u][lane + kWave] = v1[u];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      }
      // The row's part of the window holds the match, if there is one, unless the row goes on in
      // front of the window with columns that may still reach c, or likewise behind it.  The
      // search is branch-free: window slots in front of the row's part count as smaller than c,
      // slots behind it as larger, which keeps the predicate monotone over the whole window.
      uint32_t outside = 0;  // snapshots this lane has to look up in global memory
#pragma unroll
      for (int u = 0; u < G; ++u) {
        const int t = t0 + u;
        if (t < KMAX && t < k) {
          const int32_t *wu = win[wv][u];
          const int32_t s0 = max(lo[u], P[u]) - P[u], s1 = min(hi[u], P[u] + W) - P[u];
          // (bitwise operators on purpose: every LDS read is unconditional, no branches)
          const int32_t w_first = wu[0], w_last = wu[W - 1];
          const bool front_ok = (lo[u] >= P[u]) | ((P[u] < hi[u]) & (w_first <= c));
          const bool back_ok = (hi[u] <= P[u] + W) | ((P[u] + W - 1 >= lo[u]) & (w_last >= c));
          int32_t a = 0;  // slots counted as smaller than c, capped at W - 1
#pragma unroll
          for (int step = W / 2; step >= 1; step >>= 1) {
            const int32_t idx = a + step - 1;
            const int32_t v = wu[idx];
            const bool below = (idx < s0) | ((idx < s1) & (v < c));
            a += below ? step : 0;
          }
          const int32_t v_at = wu[a];
          const bool hit = (a < s1) & (v_at == c);
          const bool inwin = front_ok & back_ok;
          pos[t] = P[u] + a;
          if (hi[u] <= lo[u]) found = false;
          else if (!inwin) outside |= 1u << u;
          else found = found && hit;
        }
      }
      if (outside != 0 && found) {
#pragma unroll
        for (int u = 0; u < G; ++u) {
          const int t = t0 + u;
          if (t < KMAX && t < k && (outside >> u & 1u) && found) {
            const int32_t g = min(max(lo[u] + rel, lo[u]), hi[u] - 1);
            const int32_t v = s.col[t][g];
            pos[t] = v == c ? g : gallop_from(s.col[t], lo[u], hi[u], g, v, c);
            found = pos[t] >= 0;
          }
        }
      }
    }
  }
  const uint64_t word = __ballot(found);
  if (lane == 0 && in) p.bits[0][e64 >> 6] = word;
  if (found) {
    // plain byte stores (every byte has one writer); positions ascend with the lane, so the
    // stores of a wave fall into a few cache lines
#pragma unroll
    for (int t = 1; t < KMAX; ++t)
      if (t < k) p.flag8[t][pos[t]] = 1;
  }
}

// Packs the byte flags (0 or 1) of snapshots 1 .. k-1 into bitmaps (grid.y = t - 1).  A wave takes
// 4096 flags in four coalesced 1 KB loads; a lane squeezes its 16 flags into 16 bits and four
// neighbouring lanes merge into one word.  Flags behind a snapshot's last entry are padding inside
// the cleared flag area, so they read as zero.
constexpr int kPackPerWave = 4096;

__device__ inline uint32_t squeeze4(uint32_t x) {  // bytes b0..b3 in {0, 1} -> b0 | b1<<1 | b2<<2 | b3<<3
  return (x * 0x01020408u) >> 24 & 0xfu;
}

__global__ __launch_bounds__(kBlock) void k_pack(Snaps s, Parts p) {
  const int t = blockIdx.y + 1;
  const int32_t nnz = s.nnz[t];
  const int lane = threadIdx.x % kWave;
  const int64_t base = ((int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave) * kPackPerWave;
  if (base >= nnz) return;  // whole wave
#pragma unroll
  for (int j = 0; j < kPackPerWave / (16 * kWave); ++j) {
    const int64_t off = base + (int64_t)(j * kWave + lane) * 16;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (off < nnz) v = *reinterpret_cast<const uint4 *>(p.flag8[t] + off);
    const uint32_t bits16 =
        squeeze4(v.x) | squeeze4(v.y) << 4 | squeeze4(v.z) << 8 | squeeze4(v.w) << 12;
    unsigned long long part = (unsigned long long)bits16 << (16 * (lane & 3));
    part |= __shfl_xor(part, 1);
    part |= __shfl_xor(part, 2);
    if ((lane & 3) == 0 && off < nnz) p.bits[t][off >> 6] = part;
  }
}

// ---- count ----------------------------------------------------------------------------------
// grid.y = part; cnt[word_off[part] + w] = number of selected entries in word w.
__global__ __launch_bounds__(kBlock) void k_popcount(Snaps s, Parts p, uint32_t *cnt, uint32_t m) {
  const int part = blockIdx.y;
  if (part == 0 && blockIdx.x == 0 && threadIdx.x == 0) cnt[m - 1] = 0;  // the trailing word
  const uint32_t nw = p.word_off[part + 1] - p.word_off[part];
  const uint32_t w = blockIdx.x * kBlock + threadIdx.x;
  if (w < nw) cnt[p.word_off[part] + w] = (uint32_t)__popcll(selected_word(p, s, part, w));
}

// ---- exclusive prefix sum over uint32 (three launches) ---------------------------------------
constexpr int kScanItems = 8;
constexpr int kScanTile = kBlock * kScanItems;

// Exclusive scan of one value per thread across the workgroup; returns the prefix, sets total.
__device__ inline uint32_t block_exclusive_scan(uint32_t v, uint32_t &total) {
  __shared__ uint32_t wave_sum[kWavesPerBlock];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  uint32_t inc = v;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const uint32_t up = __shfl_up(inc, d, kWave);
    if (lane >= d) inc += up;
  }
  __syncthreads();  // protects wave_sum against the previous call's readers
  if (lane == kWave - 1) wave_sum[wave] = inc;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kWavesPerBlock; ++w) {
    const uint32_t x = wave_sum[w];
    if (w < wave) before += x;
    all += x;
  }
  total = all;
  return before + inc - v;
}

// Up to kScanBatch arrays of one length are scanned by the same three launches (grid.y = array).
constexpr int kScanBatch = 3;
struct ScanBatch {
  uint32_t *data[kScanBatch];
  uint32_t *bsum[kScanBatch];  // ceil(m / kScanTile) words each
};

__global__ __launch_bounds__(kBlock) void k_scan_reduce(ScanBatch b, uint32_t m) {
  const uint32_t *data = b.data[blockIdx.y];
  const uint32_t base = blockIdx.x * (uint32_t)kScanTile + threadIdx.x * kScanItems;
  uint32_t s = 0;
#pragma unroll
  for (int q = 0; q < kScanItems; ++q)
    if (base + q < m) s += data[base + q];
  uint32_t total;
  block_exclusive_scan(s, total);
  if (threadIdx.x == 0) b.bsum[blockIdx.y][blockIdx.x] = total;
}

__global__ __launch_bounds__(kBlock) void k_scan_blocksums(ScanBatch b, uint32_t nb) {
  uint32_t *bsum = b.bsum[blockIdx.x];
  uint32_t carry = 0;
  for (uint32_t base = 0; base < nb; base += kBlock) {
    const uint32_t idx = base + threadIdx.x;
    const uint32_t v = idx < nb ? bsum[idx] : 0u;
    uint32_t total;
    const uint32_t pre = block_exclusive_scan(v, total);
    if (idx < nb) bsum[idx] = carry + pre;
    carry += total;
  }
}

__global__ __launch_bounds__(kBlock) void k_scan_apply(ScanBatch b, uint32_t m) {
  uint32_t *data = b.data[blockIdx.y];
  const uint32_t base = blockIdx.x * (uint32_t)kScanTile + threadIdx.x * kScanItems;
  uint32_t v[kScanItems];
  uint32_t s = 0;
#pragma unroll
  for (int q = 0; q < kScanItems; ++q) {
    v[q] = base + q < m ? data[base + q] : 0u;
    s += v[q];
  }
  uint32_t total;
  uint32_t pre = block_exclusive_scan(s, total) + b.bsum[blockIdx.y][blockIdx.x];
#pragma unroll
  for (int q = 0; q < kScanItems; ++q) {
    if (base + q < m) data[base + q] = pre;
    pre += v[q];
  }
}

// In-place exclusive scans of `count` arrays data[j][0..m); bsum holds count * ceil(m / kScanTile)
// words.
int exclusive_scan(uint32_t *const *data, int count, uint32_t m, uint32_t *bsum, hipStream_t st) {
  if (m == 0 || count == 0) return PIPAD_OK;
  const uint32_t nb = (m + kScanTile - 1) / kScanTile;
  ScanBatch b;
  for (int j = 0; j < kScanBatch; ++j) {
    b.data[j] = data[j < count ? j : 0];
    b.bsum[j] = bsum + (size_t)(j < count ? j : 0) * nb;
  }
  hipLaunchKernelGGL(k_scan_reduce, dim3(nb, count), dim3(kBlock), 0, st, b, m);
  hipLaunchKernelGGL(k_scan_blocksums, dim3(count), dim3(kBlock), 0, st, b, nb);
  hipLaunchKernelGGL(k_scan_apply, dim3(nb, count), dim3(kBlock), 0, st, b, m);
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

int exclusive_scan(uint32_t *data, uint32_t m, uint32_t *bsum, hipStream_t st) {
  return exclusive_scan(&data, 1, m, bsum, st);
}

// ---- row pointers of every part ---------------------------------------------------------------
// grid.y = part; thread per row boundary i in [0, n].  pre = scanned popcounts (all parts
// concatenated, one trailing word); differences are taken in uint32 so that a wrapped running
// total over all parts cannot corrupt a single part (each part has < 2^31 entries).
__global__ __launch_bounds__(kBlock) void k_rowptr(Snaps s, Parts p, const uint32_t *pre,
                                                    int32_t n) {
  const int part = blockIdx.y;
  const int t = part_snapshot(part);
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i > n) return;
  const uint32_t r = (uint32_t)s.rowptr[t][i];
  const uint32_t w = r >> 6, bit = r & 63u;
  const uint32_t off = p.word_off[part];
  uint32_t v = pre[off + w] - pre[off];
  if (bit) v += (uint32_t)__popcll(selected_word(p, s, part, w) & ((1ull << bit) - 1ull));
  p.rowptr_out[part][i] = (int32_t)v;
}

// ---- per-row metadata: D^-1/2 ------------------------------------------------------------------
// dinv_t[i] = (1 + |row i of snapshot t|)^-1/2, evaluated in double and rounded once.
__global__ __launch_bounds__(kBlock) void k_dinv(Snaps s, int32_t n, int32_t k, float *dinv,
                                                  float *dinv_nk) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  for (int t = 0; t < k; ++t) {
    const int32_t len = s.rowptr[t][i + 1] - s.rowptr[t][i];
    const float v = (float)(1.0 / sqrt((double)(len + 1)));
    dinv[(int64_t)t * n + i] = v;
    dinv_nk[i * k + t] = v;  // node-major copy for the scatter step (one line per node)
  }
}

// ---- row classes --------------------------------------------------------------------------------
// Length L(i) = common + longest exclusive row decides the class (see pipad_frame); the three
// arrays written here are turned into list positions by exclusive prefix sums.  split_total[p]
// receives the number of entries that the hub rows hold in part p (0 = common, 1 + t = exclusive
// part of snapshot t): the sizes of the class-grouped copies.  Integer atomics, one per
// workgroup and part, so the result does not depend on scheduling.
struct PartRows {
  const int32_t *rowptr[PIPAD_MAX_K + 1];  // common, then the k exclusive parts
};

__global__ __launch_bounds__(kBlock) void k_classify(PartRows p, int32_t n, int32_t k,
                                                      uint32_t *shortflag, uint32_t *hubflag,
                                                      uint32_t *nseg, uint32_t *split_total,
                                                      int32_t short_max, int32_t mid_max,
                                                      int32_t threshold, int32_t segment) {
  __shared__ uint32_t sums[PIPAD_MAX_K + 1];
  for (int q = threadIdx.x; q <= k; q += kBlock) sums[q] = 0;
  __syncthreads();
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i == n) {  // trailing entries of the arrays that get scanned
    shortflag[n] = 0;
    hubflag[n] = 0;
    nseg[n] = 0;
  } else if (i < n) {
    const int32_t lc = p.rowptr[0][i + 1] - p.rowptr[0][i];
    int32_t ldmax = 0;
    for (int q = 1; q <= k; ++q) ldmax = max(ldmax, p.rowptr[q][i + 1] - p.rowptr[q][i]);
    const int64_t total = (int64_t)lc + ldmax;
    const int cls = row_class(total, short_max, mid_max);
    shortflag[i] = cls == 0 ? 1u : 0u;
    hubflag[i] = cls == 2 ? 1u : 0u;
    nseg[i] = cls == 2 ? hub_units(total, threshold, segment) : 0u;
    if (cls == 2)
      for (int q = 0; q <= k; ++q) {  // (the few split rows read their row pointers a second time)
        const int32_t len = p.rowptr[q][i + 1] - p.rowptr[q][i];
        if (len) atomicAdd(&sums[q], (uint32_t)len);
      }
  }
  __syncthreads();
  for (int q = threadIdx.x; q <= k; q += kBlock)
    if (sums[q]) atomicAdd(&split_total[q], sums[q]);
}

// Turns the scanned class arrays into the row lists and the hub units.
// Every row is in exactly one class, so its position in the mid list is i - (#short before i)
// - (#hub before i).  A hub row that is not cut is one unit covering its whole entry list.
__global__ __launch_bounds__(kBlock) void k_row_lists(int32_t n, const uint32_t *shortidx,
                                                       const uint32_t *hubidx,
                                                       const uint32_t *segoff, int32_t segment,
                                                       int32_t *rows_short, int32_t *rows_long,
                                                       int32_t *hub_rows, int32_t *hub_item_off,
                                                       int32_t *item_row, int32_t *item_v0,
                                                       int32_t *item_v1) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i > n) return;
  if (i == n) {
    hub_item_off[hubidx[n]] = (int32_t)segoff[n];
    return;
  }
  const uint32_t si = shortidx[i], hi = hubidx[i];
  if (shortidx[i + 1] != si) {
    rows_short[si] = (int32_t)i;
  } else if (hubidx[i + 1] != hi) {
    const uint32_t first = segoff[i], last = segoff[i + 1];
    hub_rows[hi] = (int32_t)i;
    hub_item_off[hi] = (int32_t)first;
    for (uint32_t q = first; q < last; ++q) {
      item_row[q] = (int32_t)i;
      const int64_t v0 = (int64_t)(q - first) * segment;
      item_v0[q] = last - first == 1 ? 0 : (int32_t)v0;
      item_v1[q] = last - first == 1 ? INT32_MAX : (int32_t)min(v0 + segment, (int64_t)INT32_MAX);
    }
  } else {
    rows_long[(uint32_t)i - si - hi] = (int32_t)i;
  }
}

// ---- class-grouped copies of the split rows' entries ----------------------------------------------
struct SplitArgs {
  int32_t n, n_units, k;
  int32_t sub_log2;
  int32_t team_log2;                       // delta fill: lanes per (unit, snapshot) team
  const int32_t *item_row, *item_v0, *item_v1;
  const int32_t *rowptr[PIPAD_MAX_K + 1];  // parts: common, then exclusive
  const int32_t *col[PIPAD_MAX_K + 1];
  const float *dinv_nk;                    // [n][k]
  const float *wd[PIPAD_MAX_K];            // canonical scales of the exclusive parts
  uint32_t *ulen;                          // [(k + 1) * n_units + 1]: lengths, then (scanned) starts
  uint32_t *sptr;
  int32_t *scol;
  float *swc[PIPAD_MAX_K];
  float *swd;
  uint32_t total_c;
};

// Entries [*a, *b) of part p's column array that unit u covers.
__device__ inline void unit_range(const SplitArgs &g, int p, int32_t u, int32_t *a, int32_t *b) {
  const int32_t row = g.item_row[u], v0 = g.item_v0[u], v1 = g.item_v1[u];
  const int32_t cs = g.rowptr[0][row], lc = g.rowptr[0][row + 1] - cs;
  if (p == 0) {
    *a = cs + min(v0, lc);
    *b = cs + min(v1, lc);
  } else {
    const int32_t ds = g.rowptr[p][row], ld = g.rowptr[p][row + 1] - ds;
    *a = ds + min(max(v0 - lc, 0), ld);
    *b = ds + min(max(v1 - lc, 0), ld);
  }
}

// ulen[p * n_units + u] = entries of unit u in part p (the trailing word is cleared).
__global__ __launch_bounds__(kBlock) void k_unit_len(SplitArgs g) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t m = (int64_t)(g.k + 1) * g.n_units;
  if (e > m) return;
  if (e == m) { g.ulen[m] = 0; return; }
  const int p = (int)(e / g.n_units);
  int32_t a, b;
  unit_range(g, p, (int32_t)(e - (int64_t)p * g.n_units), &a, &b);
  g.ulen[e] = (uint32_t)(b - a);
}

// The class-grouped copy of one part of one unit by a team of TL = 1 << tl_log2 lanes (all of
// them active and in step; lanes below `lane0` belong to other teams).  First pass: entries per
// class; second pass: a stable scatter - a ballot per class gives every lane its rank among the
// team's lanes of that class - which takes the entries' column scales along.
template <int NC>
__device__ inline void split_fill_part(const SplitArgs &g, int p, int32_t u, int tl_log2, int lane) {
  const int tl = 1 << tl_log2;
  const int q = lane & (tl - 1);      // lane within the team
  const int lane0 = lane - q;
  const uint64_t team_mask = (tl == kWave ? ~0ull : ((1ull << tl) - 1ull)) << lane0;
  int32_t a, b;
  unit_range(g, p, u, &a, &b);
  const int32_t *col = g.col[p];
#ifndef PIPAD_FILL_CHUNKS
#define PIPAD_FILL_CHUNKS 8
#endif
  constexpr int UN = PIPAD_FILL_CHUNKS;  // chunks in flight per pass
  uint32_t cnt[NC];
#pragma unroll
  for (int x = 0; x < NC; ++x) cnt[x] = 0;
  for (int32_t e0 = a + q; e0 < b; e0 += UN * tl) {
    int32_t cv[UN];
#pragma unroll
    for (int j = 0; j < UN; ++j) cv[j] = e0 + j * tl < b ? col[e0 + j * tl] : -1;
#pragma unroll
    for (int j = 0; j < UN; ++j) {
      const uint32_t c = cv[j] >= 0 ? column_class(cv[j], g.sub_log2) : (uint32_t)NC;
#pragma unroll
      for (int x = 0; x < NC; ++x) cnt[x] += c == (uint32_t)x ? 1u : 0u;
    }
  }
  uint32_t run[NC];  // next free position of every class (the same in all lanes of the team)
  uint32_t next = g.ulen[(int64_t)p * g.n_units + u];
  const int64_t v = ((int64_t)p * g.n_units + u) * NC;
#pragma unroll
  for (int x = 0; x < NC; ++x) {
    uint32_t c = cnt[x];
    for (int m = tl >> 1; m >= 1; m >>= 1) c += __shfl_xor(c, m, kWave);
    run[x] = next;
    if (q == 0) g.sptr[v + x] = next;
    next += c;
  }
  const float *wd_t = g.wd[p > 0 ? p - 1 : 0];
  for (int32_t base = a; base < b; base += UN * tl) {
    int32_t cv[UN];
    uint32_t pos[UN];
#pragma unroll
    for (int j = 0; j < UN; ++j) {
      const int32_t e = base + j * tl + q;
      cv[j] = e < b ? col[e] : -1;
    }
#pragma unroll
    for (int j = 0; j < UN; ++j) {
      const uint32_t cl = cv[j] >= 0 ? column_class(cv[j], g.sub_log2) : (uint32_t)NC;
      pos[j] = 0;
#pragma unroll
      for (int x = 0; x < NC; ++x) {
        const uint64_t mask = __ballot(cl == (uint32_t)x) & team_mask;
        if (cl == (uint32_t)x) pos[j] = run[x] + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        run[x] += (uint32_t)__popcll(mask);
      }
    }
    if (p == 0) {
      // (the k scales of an overlap entry follow in k_split_scales, one lane per grouped entry)
    } else {
      float wv[UN];
#pragma unroll
      for (int j = 0; j < UN; ++j) wv[j] = cv[j] >= 0 ? wd_t[base + j * tl + q] : 0.f;
#pragma unroll
      for (int j = 0; j < UN; ++j)
        if (cv[j] >= 0) g.swd[pos[j] - g.total_c] = wv[j];
    }
#pragma unroll
    for (int j = 0; j < UN; ++j)
      if (cv[j] >= 0) g.scol[pos[j]] = cv[j];
  }
}

// Column scales of the grouped overlap entries: swc[t][e] = dinv_t[scol[e]], one lane per entry,
// a node's k scales from the node-major copy of D^-1/2 (one line per node).
__global__ __launch_bounds__(kBlock) void k_split_scales(SplitArgs g) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= g.total_c) return;
  const float *row = g.dinv_nk + (int64_t)g.scol[e] * g.k;
  if ((g.k & 3) == 0) {
    for (int t = 0; t < g.k; t += 4) {
      const float4 w4 = *reinterpret_cast<const float4 *>(row + t);
      g.swc[t][e] = w4.x; g.swc[t + 1][e] = w4.y; g.swc[t + 2][e] = w4.z; g.swc[t + 3][e] = w4.w;
    }
  } else {
    for (int t = 0; t < g.k; ++t) g.swc[t][e] = row[t];
  }
}

// One wave per unit: first the overlap part with the whole wave, then the k exclusive parts side
// by side, a team of 64 / (k rounded up to a power of two) lanes per snapshot (the exclusive parts
// of a unit are short where the overlap is large, and where it is small there are k of them to
// keep the wave busy).
template <int NC>
__global__ __launch_bounds__(kBlock) void k_split_fill(SplitArgs g) {
  const int lane = threadIdx.x % kWave;
  const int64_t id = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  if (id == 0 && lane == 0)
    g.sptr[(int64_t)(g.k + 1) * g.n_units * NC] = g.ulen[(int64_t)(g.k + 1) * g.n_units];
  if (id >= g.n_units) return;
  const int32_t u = __builtin_amdgcn_readfirstlane((int32_t)id);
  split_fill_part<NC>(g, 0, u, 6, lane);
  for (int t0 = 0; t0 < g.k; t0 += kWave >> g.team_log2) {
    const int t = t0 + (lane >> g.team_log2);
    if (t < g.k) split_fill_part<NC>(g, 1 + t, u, g.team_log2, lane);
  }
}

// ---- scatter ----------------------------------------------------------------------------------
// Every selected entry is written to prefix[word] + (selected entries below it in its word), which
// keeps the ascending column order of the input.  Besides the column index, the column scale
// dinv_t[column] of the entry is stored: for a common entry once per snapshot, for an exclusive
// entry for its own snapshot (dinv of one snapshot is 4 bytes per node: cache-resident).
//
// Common part: one lane per stored entry of snapshot 0 (most of them are selected); the entry's k
// column scales come from the node-major copy of D^-1/2 (one line per node).
// KV > 0: k == 4 * KV, a node's k scales are read as KV 16-byte pieces; KV == 0: any k, one by one.
// The scales of a hub row's entries are never read from here (the aggregation takes them from the
// class-grouped copy, k_split_scales): a wave whose 64 entries all lie in one hub row - most waves
// of such a row - skips them.  wave_row / hubidx: as written by k_wave_rows and the scan of
// k_classify's hub flags.
template <int KV>
__global__ __launch_bounds__(kBlock) void k_scatter_common(Snaps s, Parts p, const uint32_t *pre,
                                                            const float *dinv_nk, int32_t k,
                                                            const int32_t *wave_row,
                                                            const uint32_t *hubidx, int32_t n) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= s.nnz[0]) return;
  const uint32_t w = (uint32_t)(e >> 6), bit = (uint32_t)(e & 63);
  const uint64_t sel = p.bits[0][w];
  if (!((sel >> bit) & 1ull)) return;
  const uint32_t dst = pre[w] - pre[0] + (uint32_t)__popcll(sel & ((1ull << bit) - 1ull));
  const int32_t c = s.col[0][e];
  p.col_out[0][dst] = c;
  const int32_t r0 = wave_row[w], r1 = wave_row[w + 1];  // rows of this and of the next wave's first entry
  if (r0 == r1) {
    const int32_t r = min(max(r0, 0), n - 1);
    if (hubidx[r + 1] != hubidx[r]) return;
  }
  if (KV > 0) {
    const float4 *row = reinterpret_cast<const float4 *>(dinv_nk) + (int64_t)c * KV;
    float4 v[KV > 0 ? KV : 1];
#pragma unroll
    for (int q = 0; q < KV; ++q) v[q] = row[q];
#pragma unroll
    for (int q = 0; q < KV; ++q) {
      p.wc[4 * q + 0][dst] = v[q].x;
      p.wc[4 * q + 1][dst] = v[q].y;
      p.wc[4 * q + 2][dst] = v[q].z;
      p.wc[4 * q + 3][dst] = v[q].w;
    }
  } else {
    for (int u = 0; u < k; ++u) p.wc[u][dst] = dinv_nk[(int64_t)c * k + u];
  }
}

// Exclusive parts (grid.y = snapshot): usually few entries are selected.  A wave takes 64
// consecutive 64-entry words; its selected entries are consecutive in the output, so lane l takes
// the l-th, l + 64-th, ... of them: it finds the word (a search over the words' running counts)
// and the bit (the r-th set bit of that word), and the wave's stores are contiguous.
__device__ inline int nth_set_bit(uint64_t x, int r) {  // position of the r-th (0-based) set bit
  int pos = 0;
#pragma unroll
  for (int width = 32; width >= 1; width >>= 1) {
    const int c = __popcll(x & (((1ull << width) - 1ull) << pos));
    if (r >= c) {
      r -= c;
      pos += width;
    }
  }
  return pos;
}

__global__ __launch_bounds__(kBlock) void k_scatter_delta(Snaps s, Parts p, const uint32_t *pre,
                                                           const float *dinv, int32_t n) {
  const int t = blockIdx.y;
  const int part = 1 + t;
  const int lane = threadIdx.x % kWave;
  const uint32_t nw = p.word_off[part + 1] - p.word_off[part];
  const uint32_t w0 = (blockIdx.x * kWavesPerBlock + threadIdx.x / kWave) * kWave;  // first word of the wave
  if (w0 >= nw) return;
  const uint32_t w = w0 + lane;
  const uint64_t sel = w < nw ? selected_word(p, s, part, w) : 0ull;
  const uint32_t off = p.word_off[part];
  const uint32_t dst0 = pre[off + w0] - pre[off];
  int incl = __popcll(sel);  // running count of selected entries up to and including this word
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int up = __shfl_up(incl, d, kWave);
    if (lane >= d) incl += up;
  }
  const int total = __shfl(incl, kWave - 1, kWave);
  const int excl = incl - __popcll(sel);
  const uint32_t sel_lo = (uint32_t)sel, sel_hi = (uint32_t)(sel >> 32);
  const int32_t *col = s.col[t] + (int64_t)w0 * 64;
  const float *dinv_t = dinv + (int64_t)t * n;
  for (int j0 = 0; j0 < total; j0 += kWave) {
    const int j = min(j0 + lane, total - 1);
    int wj = 0;  // the word that holds selected entry j: the first whose running count exceeds j
#pragma unroll
    for (int step = kWave >> 1; step >= 1; step >>= 1)
      if (__shfl(incl, wj + step - 1, kWave) <= j) wj += step;
    const int r = j - __shfl(excl, wj, kWave);
    const uint64_t x = (uint64_t)(uint32_t)__shfl((int)sel_lo, wj, kWave) |
                       ((uint64_t)(uint32_t)__shfl((int)sel_hi, wj, kWave) << 32);
    const int32_t c = col[wj * 64 + nth_set_bit(x, r)];
    const float d = dinv_t[c];
    if (j0 + lane < total) {
      p.col_out[part][dst0 + j] = c;
      p.wd[t][dst0 + j] = d;
    }
  }
}

// Exclusive parts when most entries are selected (little overlap): one lane per stored entry.
__global__ __launch_bounds__(kBlock) void k_scatter_delta_dense(Snaps s, Parts p,
                                                                 const uint32_t *pre,
                                                                 const float *dinv, int32_t n) {
  const int t = blockIdx.y;
  const int part = 1 + t;
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= s.nnz[t]) return;
  const uint32_t w = (uint32_t)(e >> 6), bit = (uint32_t)(e & 63);
  const uint64_t sel = selected_word(p, s, part, w);
  if (!((sel >> bit) & 1ull)) return;
  const uint32_t off = p.word_off[part];
  const uint32_t dst = pre[off + w] - pre[off] + (uint32_t)__popcll(sel & ((1ull << bit) - 1ull));
  const int32_t c = s.col[t][e];
  p.col_out[part][dst] = c;
  p.wd[t][dst] = dinv[(int64_t)t * n + c];
}

// Collects the data-dependent sizes into one small buffer for a single copy to the host:
// out[0 .. k+1] = prefix at the start of every part (and the end of the last), then the numbers
// of hub rows, hub units and short rows, then the k + 1 split totals.
__global__ void k_totals(Parts p, const uint32_t *pre, int32_t k, int32_t n,
                         const uint32_t *hubidx, const uint32_t *segoff,
                         const uint32_t *shortidx, const uint32_t *split_total, uint32_t *out) {
  const int q = threadIdx.x;
  if (q <= k + 1) out[q] = pre[p.word_off[q]];
  if (q <= k) out[k + 5 + q] = split_total[q];
  if (q == 0) {
    out[k + 2] = hubidx[n];
    out[k + 3] = segoff[n];
    out[k + 4] = shortidx[n];
  }
}

}  // namespace

int scan_exclusive(uint32_t *const *data, int count, uint32_t m, uint32_t *bsum, hipStream_t st) {
  return exclusive_scan(data, count, m, bsum, st);
}

size_t scan_block_words(uint32_t m) { return ((size_t)m + kScanTile - 1) / kScanTile; }

// A few pinned host words per thread for the sizes a build reads back (allocated at the thread's
// first build, kept until the process ends); null when pinned memory cannot be had.
static uint32_t *pinned_words() {
  thread_local uint32_t *buf = nullptr;
  thread_local bool tried = false;
  if (!tried) {
    tried = true;
    void *ptr = nullptr;
    if (hipHostMalloc(&ptr, sizeof(uint32_t) * (2 * PIPAD_MAX_K + 8), hipHostMallocPortable) == hipSuccess)
      buf = static_cast<uint32_t *>(ptr);
    else
      (void)hipGetLastError();
  }
  return buf;
}

void frame_take_options(pipad_frame *f) {
  const int64_t lim = (int64_t)1 << 30;  // thresholds beyond any int32 row length mean "never"
  f->opt = options();
  f->short_max = (int32_t)std::clamp<int64_t>(f->opt.short_max, 0, lim);
  f->mid_max = (int32_t)std::clamp<int64_t>(f->opt.mid_max, f->short_max, lim);
  f->hub_threshold = (int32_t)std::clamp<int64_t>(f->opt.hub_threshold, 1, lim);
  f->hub_segment = (int32_t)std::clamp<int64_t>(f->opt.hub_segment, 1, lim);
  f->sub_log2 = f->opt.sub_classes >= 4 ? 2 : f->opt.sub_classes >= 2 ? 1 : 0;
  f->nclass = kClasses << f->sub_log2;
}

int launch_classify(const pipad_frame *f, uint32_t *shortflag, uint32_t *hubflag, uint32_t *nseg,
                    uint32_t *split_total, hipStream_t st) {
  PartRows p;
  std::memset(&p, 0, sizeof(p));
  p.rowptr[0] = f->rowptr_c;
  for (int t = 0; t < f->k; ++t) p.rowptr[1 + t] = f->rowptr_d[t];
  PIPAD_HIP(hipMemsetAsync(split_total, 0, sizeof(uint32_t) * (size_t)(f->k + 1), st));
  hipLaunchKernelGGL(k_classify, grid1((int64_t)f->n + 1, kBlock), dim3(kBlock), 0, st, p, f->n, f->k,
                     shortflag, hubflag, nseg, split_total, f->short_max, f->mid_max,
                     f->hub_threshold, f->hub_segment);
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

void launch_row_lists(int32_t n, const uint32_t *shortidx, const uint32_t *hubidx,
                      const uint32_t *segoff, pipad_frame *f, hipStream_t st) {
  hipLaunchKernelGGL(k_row_lists, grid1((int64_t)n + 1, kBlock), dim3(kBlock), 0, st, n, shortidx,
                     hubidx, segoff, f->hub_segment, f->rows_short, f->rows_long, f->hub_rows,
                     f->hub_item_off, f->item_row, f->item_v0, f->item_v1);
}

int set_list_sizes(pipad_frame *f, uint32_t n_hub, uint32_t n_items, uint32_t n_short,
                   const uint32_t *split_total) {
  f->n_hub = (int32_t)n_hub;
  f->n_items = (int32_t)n_items;
  f->n_short = (int32_t)n_short;
  f->n_long = f->n - f->n_short - f->n_hub;
  f->n_units = f->n_items;
  f->split_all = 0;
  for (int q = 0; q <= f->k; ++q) {
    f->split_total[q] = split_total[q];
    f->split_all += split_total[q];
  }
  if (f->split_all >= ((int64_t)1 << 31) ||
      (int64_t)(f->k + 1) * f->n_units * f->nclass >= ((int64_t)1 << 31))
    return PIPAD_ERR_TOO_LARGE;
  return PIPAD_OK;
}

void want_lists(Arena &a, pipad_frame *f, uint32_t **ulen, uint32_t **ubsum) {
  a.want(&f->rows_short, (size_t)f->n_short);
  a.want(&f->rows_long, (size_t)f->n_long);
  a.want(&f->hub_rows, (size_t)f->n_hub);
  a.want(&f->hub_item_off, (size_t)f->n_hub + 1);
  a.want(&f->item_row, (size_t)f->n_items);
  a.want(&f->item_v0, (size_t)f->n_items);
  a.want(&f->item_v1, (size_t)f->n_items);
  const size_t nu = (size_t)(f->k + 1) * f->n_units;
  a.want(&f->sptr, nu * f->nclass + 1);
  a.want(&f->scol, (size_t)f->split_all);
  for (int t = 0; t < f->k; ++t) a.want(&f->swc[t], (size_t)f->split_total[0]);
  a.want(&f->swd, (size_t)(f->split_all - f->split_total[0]));
  a.want(ulen, nu + 1);
  a.want(ubsum, scan_block_words((uint32_t)(nu + 1)) + 1);
}

int build_split_arrays(pipad_frame *f, uint32_t *ulen, uint32_t *bsum, hipStream_t st) {
  if (f->n_units == 0) return PIPAD_OK;
  SplitArgs g;
  std::memset(&g, 0, sizeof(g));
  g.n = f->n;
  g.n_units = f->n_units;
  g.k = f->k;
  g.sub_log2 = f->sub_log2;
  g.team_log2 = 6;
  while (g.team_log2 > 0 && (kWave >> g.team_log2) < f->k) --g.team_log2;  // 64 / team lanes >= k
  g.item_row = f->item_row;
  g.item_v0 = f->item_v0;
  g.item_v1 = f->item_v1;
  g.rowptr[0] = f->rowptr_c;
  g.col[0] = f->col_c;
  g.dinv_nk = f->dinv_nk;
  for (int t = 0; t < f->k; ++t) {
    g.rowptr[1 + t] = f->rowptr_d[t];
    g.col[1 + t] = f->col_d[t];
    g.wd[t] = f->wd[t];
    g.swc[t] = f->swc[t];
  }
  g.ulen = ulen;
  g.sptr = f->sptr;
  g.scol = f->scol;
  g.swd = f->swd;
  g.total_c = (uint32_t)f->split_total[0];
  const int64_t nu = (int64_t)(f->k + 1) * f->n_units;
  hipLaunchKernelGGL(k_unit_len, grid1(nu + 1, kBlock), dim3(kBlock), 0, st, g);
  PIPAD_HIP(hipGetLastError());
  {
    uint32_t *one = ulen;
    const int rc = exclusive_scan(&one, 1, (uint32_t)(nu + 1), bsum, st);
    if (rc != PIPAD_OK) return rc;
  }
  auto fill = f->sub_log2 == 0 ? k_split_fill<8> : f->sub_log2 == 1 ? k_split_fill<16> : k_split_fill<32>;
  hipLaunchKernelGGL(fill, grid1(f->n_units, kWavesPerBlock), dim3(kBlock), 0, st, g);
  if (g.total_c > 0)
    hipLaunchKernelGGL(k_split_scales, grid1(g.total_c, kBlock), dim3(kBlock), 0, st, g);
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

int build_overlap(int32_t n, int32_t k, const pipad_csr_t *snaps, uint32_t flags,
                  pipad_alloc_fn alloc, void *alloc_ctx, hipStream_t st, pipad_frame **out) {
  Snaps s;
  std::memset(&s, 0, sizeof(s));
  for (int t = 0; t < k; ++t) {
    s.rowptr[t] = snaps[t].rowptr;
    s.col[t] = snaps[t].colidx;
    s.nnz[t] = snaps[t].nnz;
  }

  pipad_frame *f = new (std::nothrow) pipad_frame;
  if (!f) return PIPAD_ERR_ALLOC;
  f->n = n;
  f->k = k;
  f->own_memory = alloc == nullptr;
  frame_take_options(f);
  Allocator A{alloc, alloc_ctx, f};
  f->alloc = alloc;
  f->alloc_ctx = alloc_ctx;
  void *temp = nullptr;  // temporaries: from the callback (kept by the caller) or hipMalloc'd here
  // every exit path below goes through fail() or the success return
  auto fail = [&](int code) {
    if (temp && !alloc) (void)hipFree(temp);
    release(f);
    return code;
  };
  if (hipGetDevice(&f->device) != hipSuccess) return fail(hip_fail(hipGetLastError(), "hipGetDevice"));
  {
    // set-up of pipad_frame_aggregate_static on this device: look up the fixed scratch array's
    // address now, so that the entry point itself has nothing left to initialise
    float *unused_ptr = nullptr;
    size_t unused_floats = 0;
    (void)static_scratch(&unused_ptr, &unused_floats);
  }

  // ---- sizes known up front: row pointers and D^-1/2 (persistent), all temporaries
  Parts p;
  std::memset(&p, 0, sizeof(p));
  uint32_t nw[PIPAD_MAX_K];
  for (int t = 0; t < k; ++t) {
    nw[t] = (uint32_t)(((int64_t)s.nnz[t] + 63) / 64);

  }
  // parts: common uses snapshot 0's words, delta_t uses snapshot t's words
  int64_t m64 = nw[0];
  for (int t = 0; t < k; ++t) m64 += nw[t];
  m64 += 1;  // trailing word so that prefix[end of last part] exists
  if (m64 >= ((int64_t)1 << 31)) return fail(PIPAD_ERR_TOO_LARGE);
  const uint32_t m = (uint32_t)m64;
  p.word_off[0] = 0;
  p.word_off[1] = nw[0];
  for (int t = 0; t < k; ++t) p.word_off[2 + t] = p.word_off[1 + t] + nw[t];
  const uint32_t scan_len_rows = (uint32_t)n + 1;

  Arena keep1;
  keep1.want(&f->rowptr_c, (size_t)n + 1);
  for (int t = 0; t < k; ++t) keep1.want(&f->rowptr_d[t], (size_t)n + 1);
  keep1.want(&f->dinv, (size_t)k * n);
  keep1.want(&f->dinv_nk, (size_t)k * n);
  {
    void *base = A.get(keep1.total);
    if (!base) return fail(PIPAD_ERR_ALLOC);
    keep1.assign(base);
  }
  p.rowptr_out[0] = f->rowptr_c;
  for (int t = 0; t < k; ++t) p.rowptr_out[1 + t] = f->rowptr_d[t];

  Arena tmp;
  size_t flag_bytes = 0;  // byte flags of snapshots 1 .. k-1 come first and are cleared together
  for (int t = 1; t < k; ++t) {
    tmp.want(&p.flag8[t], (size_t)s.nnz[t]);
    flag_bytes = tmp.total;
  }
  for (int t = 0; t < k; ++t) tmp.want(&p.bits[t], (size_t)nw[t]);
  uint32_t *pre = nullptr, *bsum = nullptr, *shortidx = nullptr, *hubidx = nullptr,
           *segoff = nullptr, *totals = nullptr, *split_total = nullptr;
  int *dflags = nullptr;
  tmp.want(&pre, (size_t)m);
  tmp.want(&bsum, std::max(((size_t)m + kScanTile - 1) / kScanTile,
                           3 * (((size_t)scan_len_rows + kScanTile - 1) / kScanTile)) + 1);
  tmp.want(&shortidx, (size_t)scan_len_rows);
  tmp.want(&hubidx, (size_t)scan_len_rows);
  tmp.want(&segoff, (size_t)scan_len_rows);
  int32_t *wave_row = nullptr;
  tmp.want(&wave_row, (size_t)nw[0] + 2);
  tmp.want(&totals, (size_t)2 * PIPAD_MAX_K + 8);
  tmp.want(&split_total, (size_t)PIPAD_MAX_K + 1);
  tmp.want(&dflags, (size_t)64);
  if (alloc) {
    temp = alloc(tmp.total, alloc_ctx);
    f->temp_ptr = temp;
    f->temp_bytes = temp ? tmp.total : 0;
  } else if (hipMalloc(&temp, tmp.total) != hipSuccess) {
    (void)hipGetLastError();
    temp = nullptr;
  }
  if (!temp) return fail(PIPAD_ERR_ALLOC);
  tmp.assign(temp);

  auto hipcheck = [&](hipError_t e, const char *what) { return e == hipSuccess ? 0 : hip_fail(e, what); };
#define PIPAD_TRY(call)                                   \
  do {                                                    \
    int rc__ = hipcheck((call), #call);                   \
    if (rc__ != 0) return fail(rc__);                     \
  } while (0)

  if (flag_bytes) PIPAD_TRY(hipMemsetAsync(temp, 0, flag_bytes, st));

  if ((flags & PIPAD_VALIDATE) && n > 0) {
    PIPAD_TRY(hipMemsetAsync(dflags, 0, 256, st));
    hipLaunchKernelGGL(k_validate, grid1((int64_t)k * n, kWavesPerBlock), dim3(kBlock), 0, st, s, n,
                       k, dflags);
    int bad = 0;
    PIPAD_TRY(hipGetLastError());
    PIPAD_TRY(hipMemcpyAsync(&bad, dflags, sizeof(int), hipMemcpyDeviceToHost, st));
    PIPAD_TRY(hipStreamSynchronize(st));
    if (bad) return fail(PIPAD_ERR_BAD_CSR);
  }

  if (s.nnz[0] > 0) {
    hipLaunchKernelGGL(k_wave_rows, grid1(n, kBlock), dim3(kBlock), 0, st, s.rowptr[0], n, s.nnz[0],
                       wave_row);
    // instances by the largest k they handle: fewer snapshots, fewer registers, more waves per CU
    auto mark = k <= 8 ? k_mark<8> : k <= 16 ? k_mark<16> : k_mark<PIPAD_MAX_K>;
    hipLaunchKernelGGL(mark, grid1(s.nnz[0], kBlock), dim3(kBlock), 0, st, s, p, n, k, wave_row);
  }
  {
    int32_t max_later = 0;
    for (int t = 1; t < k; ++t) max_later = std::max(max_later, s.nnz[t]);
    if (max_later > 0)
      hipLaunchKernelGGL(k_pack, grid1(max_later, kPackPerWave * kWavesPerBlock, k - 1), dim3(kBlock), 0,
                         st, s, p);
  }
  uint32_t max_nw = 0;
  for (int t = 0; t < k; ++t) max_nw = std::max(max_nw, nw[t]);
  if (max_nw > 0)
    hipLaunchKernelGGL(k_popcount, grid1(max_nw, kBlock, k + 1), dim3(kBlock), 0, st, s, p, pre, m);
  else
    PIPAD_TRY(hipMemsetAsync(pre, 0, sizeof(uint32_t) * (size_t)m, st));  // no entries at all
  PIPAD_TRY(hipGetLastError());
  {
    int rc = exclusive_scan(pre, m, bsum, st);
    if (rc != 0) return fail(rc);
  }
  hipLaunchKernelGGL(k_rowptr, grid1((int64_t)n + 1, kBlock, k + 1), dim3(kBlock), 0, st, s, p,
                     pre, n);
  PIPAD_TRY(hipGetLastError());
  {
    const int rc = launch_classify(f, shortidx, hubidx, segoff, split_total, st);
    if (rc != 0) return fail(rc);
  }
  {
    uint32_t *three[3] = {shortidx, hubidx, segoff};
    const int rc = exclusive_scan(three, 3, scan_len_rows, bsum, st);
    if (rc != 0) return fail(rc);
  }

  // ---- the one host synchronisation: sizes of the data-dependent outputs.  The host waits for
  // an event behind the copy, and D^-1/2 - which nothing before this point needs - is computed
  // behind that event, while the host sizes and requests the output buffers.
  uint32_t stack_totals[2 * PIPAD_MAX_K + 8];
  uint32_t *host_totals = pinned_words();
  hipLaunchKernelGGL(k_totals, dim3(1), dim3(kWave), 0, st, p, pre, k, n, hubidx, segoff, shortidx,
                     split_total, totals);
  PIPAD_TRY(hipGetLastError());
  hipEvent_t copied = nullptr;
  if (host_totals && hipEventCreateWithFlags(&copied, hipEventDisableTiming) != hipSuccess) {
    (void)hipGetLastError();
    copied = nullptr;
  }
  if (!copied) host_totals = stack_totals;
  {
    const hipError_t ce = hipMemcpyAsync(host_totals, totals, sizeof(uint32_t) * (size_t)(2 * k + 6),
                                         hipMemcpyDeviceToHost, st);
    if (ce != hipSuccess && copied) (void)hipEventDestroy(copied);
    PIPAD_TRY(ce);
  }
  if (copied) {
    hipError_t e = hipEventRecord(copied, st);
    if (e == hipSuccess && n > 0)
      hipLaunchKernelGGL(k_dinv, grid1(n, kBlock), dim3(kBlock), 0, st, s, n, k, f->dinv, f->dinv_nk);
    if (e == hipSuccess) e = hipEventSynchronize(copied);
    (void)hipEventDestroy(copied);
    PIPAD_TRY(e);
    PIPAD_TRY(hipGetLastError());
  } else {
    PIPAD_TRY(hipStreamSynchronize(st));
    if (n > 0)
      hipLaunchKernelGGL(k_dinv, grid1(n, kBlock), dim3(kBlock), 0, st, s, n, k, f->dinv, f->dinv_nk);
    PIPAD_TRY(hipGetLastError());
  }

  f->nnz_c = (int32_t)(host_totals[1] - host_totals[0]);
  for (int t = 0; t < k; ++t) f->nnz_d[t] = (int32_t)(host_totals[2 + t] - host_totals[1 + t]);
  {
    const int rc = set_list_sizes(f, host_totals[k + 2], host_totals[k + 3], host_totals[k + 4],
                                  host_totals + k + 5);
    if (rc != 0) return fail(rc);
  }

  Arena keep2;
  keep2.want(&f->col_c, (size_t)f->nnz_c);
  for (int t = 0; t < k; ++t) {
    keep2.want(&f->col_d[t], (size_t)f->nnz_d[t]);
    keep2.want(&f->wc[t], (size_t)f->nnz_c);
    keep2.want(&f->wd[t], (size_t)f->nnz_d[t]);
  }
  uint32_t *ulen = nullptr, *ubsum = nullptr;
  want_lists(keep2, f, &ulen, &ubsum);
  {
    void *base = A.get(keep2.total);
    if (!base) return fail(PIPAD_ERR_ALLOC);
    keep2.assign(base);
  }
  p.col_out[0] = f->col_c;
  for (int t = 0; t < k; ++t) {
    p.col_out[1 + t] = f->col_d[t];
    p.wc[t] = f->wc[t];
    p.wd[t] = f->wd[t];
  }

  if (s.nnz[0] > 0) {
    auto scatter = k == 4 ? k_scatter_common<1> : k == 8 ? k_scatter_common<2>
                 : k == 16 ? k_scatter_common<4> : k_scatter_common<0>;
    hipLaunchKernelGGL(scatter, grid1(s.nnz[0], kBlock), dim3(kBlock), 0, st, s, p, pre, f->dinv_nk, k,
                       wave_row, hubidx, n);
  }
  {
    int64_t all = 0, excl = 0;
    int32_t max_nnz = 0;
    for (int t = 0; t < k; ++t) {
      all += s.nnz[t];
      excl += f->nnz_d[t];
      max_nnz = std::max(max_nnz, s.nnz[t]);
    }
    if (excl * PIPAD_DENSE_FACTOR > all) {  // mostly selected: a lane per entry
      hipLaunchKernelGGL(k_scatter_delta_dense, grid1(max_nnz, kBlock, k), dim3(kBlock), 0, st, s, p,
                         pre, f->dinv, n);
    } else if (max_nw > 0) {
      hipLaunchKernelGGL(k_scatter_delta, grid1(max_nw, kBlock, k), dim3(kBlock), 0, st, s, p, pre,
                         f->dinv, n);
    }
  }
  launch_row_lists(n, shortidx, hubidx, segoff, f, st);
  PIPAD_TRY(hipGetLastError());
  {
    const int rc = build_split_arrays(f, ulen, ubsum, st);
    if (rc != 0) return fail(rc);
  }
  if (!alloc) {
    PIPAD_TRY(hipStreamSynchronize(st));  // the temporaries are freed next
    (void)hipFree(temp);
    temp = nullptr;
  }
#undef PIPAD_TRY
  *out = f;
  return PIPAD_OK;
}

void destroy_frame(pipad_frame *f) { release(f); }

}  // namespace pipad
