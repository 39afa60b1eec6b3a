// pipad_frame_build_overlap: overlap extraction for a frame of k CSR snapshots on gfx950.
//
// Section 4.1 ("Overlap-aware data transfer") regroups the topology of a snapshot group as one
// overlap part plus one exclusive part per snapshot; Section 4.3 makes this the job of a data
// preparation module that runs once.  Here it runs on the GPU, edge-parallel, in four steps:
//
//   mark     one lane per stored entry of snapshot 0: find its row, then binary-search its column
//            in the same row of every other snapshot.  An entry found everywhere is a common
//            edge: its bit is set in a per-snapshot bitmap (one bit per stored entry) at the
//            position where each snapshot holds it.
//   count    popcount per 64-entry word of every output part (common = set bits of snapshot 0's
//            bitmap, delta_t = clear bits of snapshot t's bitmap) and one exclusive prefix sum
//            over all words.
//   rowptr   output row pointers are read off the prefix sums at the input row starts.
//   scatter  every selected entry is written to prefix[word] + (set bits below it in its word),
//            which keeps the ascending column order of the input (stable compaction).
//
// All integer work; the outputs are unique, so they are bit-exact regardless of scheduling (the
// only atomics are integer ORs into the bitmaps).
#include <algorithm>
#include <cstring>

#include "pipad_internal.h"

namespace pipad {
namespace {

struct Snaps {
  const int32_t *rowptr[PIPAD_MAX_K];
  const int32_t *col[PIPAD_MAX_K];
  int32_t nnz[PIPAD_MAX_K];
};

struct Parts {  // part 0 = common (from snapshot 0), part 1+t = delta_t
  uint64_t *bits[PIPAD_MAX_K];       // bitmap of snapshot t, ceil(nnz_t/64) words
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
  const int t = (int)(unit / n);
  const int32_t i = (int32_t)(unit % n);
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
__global__ __launch_bounds__(kBlock) void k_mark(Snaps s, Parts p, int32_t n, int32_t k) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;  // wave-aligned: 64 | kBlock
  const int32_t nnz0 = s.nnz[0];
  const bool in = e < nnz0;
  bool found = in;
  int32_t pos[PIPAD_MAX_K];
  if (in) {
    const int32_t c = s.col[0][e];
    // row of entry e: the last i with rowptr0[i] <= e (skips empty rows)
    int32_t lo = 0, hi = n;  // invariant: rowptr0[lo] <= e < rowptr0[hi]
    const int32_t *rp0 = s.rowptr[0];
    while (hi - lo > 1) {
      const int32_t mid = lo + ((hi - lo) >> 1);
      if (rp0[mid] <= (int32_t)e) lo = mid; else hi = mid;
    }
    const int32_t i = lo;
#pragma unroll
    for (int t = 1; t < PIPAD_MAX_K; ++t) {
      pos[t] = 0;
      if (t < k && found) {
        const int32_t *col = s.col[t];
        int32_t a = s.rowptr[t][i];
        const int32_t b = s.rowptr[t][i + 1];
        int32_t len = b - a;
        while (len > 0) {  // lower_bound(c)
          const int32_t half = len >> 1;
          if (col[a + half] < c) { a += half + 1; len -= half + 1; } else { len = half; }
        }
        if (a < b && col[a] == c) pos[t] = a; else found = false;
      }
    }
  }
  const uint64_t word = __ballot(found);
  if (threadIdx.x % kWave == 0 && e < nnz0) p.bits[0][e >> 6] = word;
  if (found) {
#pragma unroll
    for (int t = 1; t < PIPAD_MAX_K; ++t) {
      if (t < k) {
        uint32_t *w32 = reinterpret_cast<uint32_t *>(p.bits[t]);
        atomicOr(&w32[pos[t] >> 5], 1u << (pos[t] & 31));
      }
    }
  }
}

// ---- count ----------------------------------------------------------------------------------
// grid.y = part; cnt[word_off[part] + w] = number of selected entries in word w.
__global__ __launch_bounds__(kBlock) void k_popcount(Snaps s, Parts p, uint32_t *cnt) {
  const int part = blockIdx.y;
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

__global__ __launch_bounds__(kBlock) void k_scan_reduce(const uint32_t *data, uint32_t m,
                                                         uint32_t *bsum) {
  const uint32_t base = blockIdx.x * (uint32_t)kScanTile + threadIdx.x * kScanItems;
  uint32_t s = 0;
#pragma unroll
  for (int q = 0; q < kScanItems; ++q)
    if (base + q < m) s += data[base + q];
  uint32_t total;
  block_exclusive_scan(s, total);
  if (threadIdx.x == 0) bsum[blockIdx.x] = total;
}

__global__ __launch_bounds__(kBlock) void k_scan_blocksums(uint32_t *bsum, uint32_t nb) {
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

__global__ __launch_bounds__(kBlock) void k_scan_apply(uint32_t *data, uint32_t m,
                                                        const uint32_t *bsum) {
  const uint32_t base = blockIdx.x * (uint32_t)kScanTile + threadIdx.x * kScanItems;
  uint32_t v[kScanItems];
  uint32_t s = 0;
#pragma unroll
  for (int q = 0; q < kScanItems; ++q) {
    v[q] = base + q < m ? data[base + q] : 0u;
    s += v[q];
  }
  uint32_t total;
  uint32_t pre = block_exclusive_scan(s, total) + bsum[blockIdx.x];
#pragma unroll
  for (int q = 0; q < kScanItems; ++q) {
    if (base + q < m) data[base + q] = pre;
    pre += v[q];
  }
}

// In-place exclusive scan of data[0..m); bsum must hold ceil(m / kScanTile) words.
int exclusive_scan(uint32_t *data, uint32_t m, uint32_t *bsum, hipStream_t st) {
  if (m == 0) return PIPAD_OK;
  const uint32_t nb = (m + kScanTile - 1) / kScanTile;
  hipLaunchKernelGGL(k_scan_reduce, dim3(nb), dim3(kBlock), 0, st, data, m, bsum);
  hipLaunchKernelGGL(k_scan_blocksums, dim3(1), dim3(kBlock), 0, st, bsum, nb);
  hipLaunchKernelGGL(k_scan_apply, dim3(nb), dim3(kBlock), 0, st, data, m, bsum);
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
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

// ---- per-row metadata: D^-1/2, length classes ---------------------------------------------------
// dinv_t[i] = (1 + |row i of snapshot t|)^-1/2, evaluated in double and rounded once.
// Length L(i) = common + longest exclusive row decides the class (see pipad_frame): the three
// arrays written here are turned into list positions by exclusive prefix sums.
__global__ __launch_bounds__(kBlock) void k_rowmeta(Snaps s, Parts p, int32_t n, int32_t k,
                                                     float *dinv, uint32_t *shortflag,
                                                     uint32_t *hubflag, uint32_t *nseg,
                                                     int32_t short_max, int32_t threshold,
                                                     int32_t segment) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i > n) return;
  if (i == n) {  // trailing entries of the arrays that get scanned
    shortflag[n] = 0;
    hubflag[n] = 0;
    nseg[n] = 0;
    return;
  }
  const int32_t lc = p.rowptr_out[0][i + 1] - p.rowptr_out[0][i];
  int32_t ldmax = 0;
  for (int t = 0; t < k; ++t) {
    const int32_t len = s.rowptr[t][i + 1] - s.rowptr[t][i];
    dinv[(int64_t)t * n + i] = (float)(1.0 / sqrt((double)(len + 1)));
    ldmax = max(ldmax, len - lc);
  }
  const int64_t total = (int64_t)lc + ldmax;
  const bool hub = total > threshold;
  shortflag[i] = total <= short_max ? 1u : 0u;
  hubflag[i] = hub ? 1u : 0u;
  nseg[i] = hub ? (uint32_t)((total + segment - 1) / segment) : 0u;
}

// Turns the scanned class arrays into the row lists and the (row, segment) work items.
// Every row is in exactly one class, so its position in the long list is i - (#short before i)
// - (#hub before i).
__global__ __launch_bounds__(kBlock) void k_row_lists(int32_t n, const uint32_t *shortidx,
                                                       const uint32_t *hubidx,
                                                       const uint32_t *segoff, int32_t *rows_short,
                                                       int32_t *rows_long, int32_t *hub_rows,
                                                       int32_t *hub_item_off, int32_t *item_row,
                                                       int32_t *item_seg) {
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
      item_seg[q] = (int32_t)(q - first);
    }
  } else {
    rows_long[(uint32_t)i - si - hi] = (int32_t)i;
  }
}

// ---- scatter ----------------------------------------------------------------------------------
// grid.y = part; one lane per stored entry of the part's snapshot.
// Besides the column index, the column scale dinv_t[column] of the entry is stored: for a common
// entry once per snapshot, for an exclusive entry for its own snapshot.
__global__ __launch_bounds__(kBlock) void k_scatter(Snaps s, Parts p, const uint32_t *pre,
                                                     const float *dinv, int32_t n, int32_t k) {
  const int part = blockIdx.y;
  const int t = part_snapshot(part);
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= s.nnz[t]) return;
  const uint32_t w = (uint32_t)(e >> 6), bit = (uint32_t)(e & 63);
  const uint64_t sel = selected_word(p, s, part, w);
  if (!((sel >> bit) & 1ull)) return;
  const uint32_t off = p.word_off[part];
  const uint32_t dst = pre[off + w] - pre[off] + (uint32_t)__popcll(sel & ((1ull << bit) - 1ull));
  const int32_t c = s.col[t][e];
  p.col_out[part][dst] = c;
  if (part == 0) {
    for (int u = 0; u < k; ++u) p.wc[u][dst] = dinv[(int64_t)u * n + c];
  } else {
    p.wd[t][dst] = dinv[(int64_t)t * n + c];
  }
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Allocator {
  pipad_alloc_fn fn;
  void *ctx;
  pipad_frame *frame;
  // Returns nullptr on failure.  bytes == 0 still returns a valid (tiny) buffer.
  void *get(size_t bytes) {
    bytes = std::max<size_t>(bytes, 256);
    void *ptr = nullptr;
    if (fn) {
      ptr = fn(bytes, ctx);
    } else {
      if (hipMalloc(&ptr, bytes) != hipSuccess) {
        (void)hipGetLastError();
        ptr = nullptr;
      }
      if (ptr) frame->owned.push_back(ptr);
    }
    return ptr;
  }
};

void release(pipad_frame *f) {
  if (!f) return;
  if (f->own_memory)
    for (void *ptr : f->owned) (void)hipFree(ptr);
  if (f->partial && f->own_memory) (void)hipFree(f->partial);
  delete f;
}

inline dim3 grid1(int64_t items, int per_block, int y = 1) {
  return dim3((unsigned)((items + per_block - 1) / per_block), (unsigned)y);
}

}  // namespace

int build_overlap(int32_t n, int32_t k, const pipad_csr_t *snaps, uint32_t flags,
                  pipad_alloc_fn alloc, void *alloc_ctx, hipStream_t st, pipad_frame **out) {
  Snaps s;
  std::memset(&s, 0, sizeof(s));
  int64_t total_words = 0;
  for (int t = 0; t < k; ++t) {
    s.rowptr[t] = snaps[t].rowptr;
    s.col[t] = snaps[t].colidx;
    s.nnz[t] = snaps[t].nnz;
  }

  pipad_frame *f = new pipad_frame;
  f->n = n;
  f->k = k;
  f->own_memory = alloc == nullptr;
  f->short_max = (int32_t)std::max<int64_t>(0, options().short_max);
  f->hub_threshold = (int32_t)std::max<int64_t>(f->short_max, options().hub_threshold);
  f->hub_segment = (int32_t)std::max<int64_t>(1, options().hub_segment);
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

  // ---- persistent buffers whose size is known up front
  Parts p;
  std::memset(&p, 0, sizeof(p));
  const size_t rp_bytes = ((size_t)n + 1) * sizeof(int32_t);
  f->rowptr_c = static_cast<int32_t *>(A.get(rp_bytes));
  if (!f->rowptr_c) return fail(PIPAD_ERR_ALLOC);
  p.rowptr_out[0] = f->rowptr_c;
  for (int t = 0; t < k; ++t) {
    f->rowptr_d[t] = static_cast<int32_t *>(A.get(rp_bytes));
    if (!f->rowptr_d[t]) return fail(PIPAD_ERR_ALLOC);
    p.rowptr_out[1 + t] = f->rowptr_d[t];
  }
  f->dinv = static_cast<float *>(A.get((size_t)k * (size_t)std::max(n, 1) * sizeof(float)));
  if (!f->dinv) return fail(PIPAD_ERR_ALLOC);

  // ---- temporaries, one allocation: bitmaps, prefix array, scan block sums, hub scans, flags
  uint32_t nw[PIPAD_MAX_K];
  for (int t = 0; t < k; ++t) {
    nw[t] = (uint32_t)(((int64_t)s.nnz[t] + 63) / 64);
    total_words += nw[t];
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

  const size_t bits_bytes = align_up((size_t)total_words * 8, 256);
  const size_t pre_bytes = align_up((size_t)m * 4, 256);
  const uint32_t scan_len_rows = (uint32_t)n + 1;
  const size_t bsum_words = (std::max<size_t>(m, scan_len_rows) + kScanTile - 1) / kScanTile + 1;
  const size_t bsum_bytes = align_up(bsum_words * 4, 256);
  const size_t rows_bytes = align_up((size_t)scan_len_rows * 4, 256);
  const size_t temp_bytes = bits_bytes + pre_bytes + bsum_bytes + 3 * rows_bytes + 256;
  if (alloc) {
    temp = alloc(temp_bytes, alloc_ctx);
  } else if (hipMalloc(&temp, temp_bytes) != hipSuccess) {
    (void)hipGetLastError();
    temp = nullptr;
  }
  if (!temp) return fail(PIPAD_ERR_ALLOC);
  char *cur = static_cast<char *>(temp);
  uint64_t *bits_all = reinterpret_cast<uint64_t *>(cur); cur += bits_bytes;
  uint32_t *pre = reinterpret_cast<uint32_t *>(cur); cur += pre_bytes;
  uint32_t *bsum = reinterpret_cast<uint32_t *>(cur); cur += bsum_bytes;
  uint32_t *shortidx = reinterpret_cast<uint32_t *>(cur); cur += rows_bytes;
  uint32_t *hubidx = reinterpret_cast<uint32_t *>(cur); cur += rows_bytes;
  uint32_t *segoff = reinterpret_cast<uint32_t *>(cur); cur += rows_bytes;
  int *dflags = reinterpret_cast<int *>(cur);  // [0] = validation verdict
  {
    uint64_t *b = bits_all;
    for (int t = 0; t < k; ++t) { p.bits[t] = b; b += nw[t]; }
  }
  auto hipcheck = [&](hipError_t e, const char *what) { return e == hipSuccess ? 0 : hip_fail(e, what); };
#define PIPAD_TRY(call)                                   \
  do {                                                    \
    int rc__ = hipcheck((call), #call);                   \
    if (rc__ != 0) return fail(rc__);                     \
  } while (0)

  PIPAD_TRY(hipMemsetAsync(temp, 0, bits_bytes, st));
  PIPAD_TRY(hipMemsetAsync(dflags, 0, 256, st));
  PIPAD_TRY(hipMemsetAsync(pre + (m - 1), 0, 4, st));  // trailing word

  if ((flags & PIPAD_VALIDATE) && n > 0) {
    hipLaunchKernelGGL(k_validate, grid1((int64_t)k * n, kWavesPerBlock), dim3(kBlock), 0, st, s, n,
                       k, dflags);
    int bad = 0;
    PIPAD_TRY(hipGetLastError());
    PIPAD_TRY(hipMemcpyAsync(&bad, dflags, sizeof(int), hipMemcpyDeviceToHost, st));
    PIPAD_TRY(hipStreamSynchronize(st));
    if (bad) return fail(PIPAD_ERR_BAD_CSR);
  }

  if (s.nnz[0] > 0)
    hipLaunchKernelGGL(k_mark, grid1(s.nnz[0], kBlock), dim3(kBlock), 0, st, s, p, n, k);
  uint32_t max_nw = 0;
  for (int t = 0; t < k; ++t) max_nw = std::max(max_nw, nw[t]);
  if (max_nw > 0)
    hipLaunchKernelGGL(k_popcount, grid1(max_nw, kBlock, k + 1), dim3(kBlock), 0, st, s, p, pre);
  PIPAD_TRY(hipGetLastError());
  {
    int rc = exclusive_scan(pre, m, bsum, st);
    if (rc != 0) return fail(rc);
  }
  hipLaunchKernelGGL(k_rowptr, grid1((int64_t)n + 1, kBlock, k + 1), dim3(kBlock), 0, st, s, p,
                     pre, n);
  hipLaunchKernelGGL(k_rowmeta, grid1((int64_t)n + 1, kBlock), dim3(kBlock), 0, st, s, p, n, k,
                     f->dinv, shortidx, hubidx, segoff, f->short_max, f->hub_threshold,
                     f->hub_segment);
  PIPAD_TRY(hipGetLastError());
  {
    int rc = exclusive_scan(shortidx, scan_len_rows, bsum, st);
    if (rc == 0) rc = exclusive_scan(hubidx, scan_len_rows, bsum, st);
    if (rc == 0) rc = exclusive_scan(segoff, scan_len_rows, bsum, st);
    if (rc != 0) return fail(rc);
  }

  // ---- the one host synchronisation: sizes of the data-dependent outputs
  uint32_t part_pre[PIPAD_MAX_K + 2];
  uint32_t hub_totals[3];
  for (int q = 0; q <= k + 1; ++q)
    PIPAD_TRY(hipMemcpyAsync(&part_pre[q], pre + p.word_off[q], 4, hipMemcpyDeviceToHost, st));
  PIPAD_TRY(hipMemcpyAsync(&hub_totals[0], hubidx + n, 4, hipMemcpyDeviceToHost, st));
  PIPAD_TRY(hipMemcpyAsync(&hub_totals[1], segoff + n, 4, hipMemcpyDeviceToHost, st));
  PIPAD_TRY(hipMemcpyAsync(&hub_totals[2], shortidx + n, 4, hipMemcpyDeviceToHost, st));
  PIPAD_TRY(hipStreamSynchronize(st));

  f->nnz_c = (int32_t)(part_pre[1] - part_pre[0]);
  f->col_c = static_cast<int32_t *>(A.get((size_t)f->nnz_c * 4));
  if (!f->col_c) return fail(PIPAD_ERR_ALLOC);
  p.col_out[0] = f->col_c;
  for (int t = 0; t < k; ++t) {
    f->nnz_d[t] = (int32_t)(part_pre[2 + t] - part_pre[1 + t]);
    f->col_d[t] = static_cast<int32_t *>(A.get((size_t)f->nnz_d[t] * 4));
    f->wc[t] = static_cast<float *>(A.get((size_t)f->nnz_c * 4));
    f->wd[t] = static_cast<float *>(A.get((size_t)f->nnz_d[t] * 4));
    if (!f->col_d[t] || !f->wc[t] || !f->wd[t]) return fail(PIPAD_ERR_ALLOC);
    p.col_out[1 + t] = f->col_d[t];
    p.wc[t] = f->wc[t];
    p.wd[t] = f->wd[t];
  }
  f->n_hub = (int32_t)hub_totals[0];
  f->n_items = (int32_t)hub_totals[1];
  f->n_short = (int32_t)hub_totals[2];
  f->n_long = n - f->n_short - f->n_hub;
  f->rows_short = static_cast<int32_t *>(A.get((size_t)f->n_short * 4));
  f->rows_long = static_cast<int32_t *>(A.get((size_t)f->n_long * 4));
  if (!f->rows_short || !f->rows_long) return fail(PIPAD_ERR_ALLOC);
  f->hub_rows = static_cast<int32_t *>(A.get((size_t)f->n_hub * 4));
  f->hub_item_off = static_cast<int32_t *>(A.get(((size_t)f->n_hub + 1) * 4));
  f->item_row = static_cast<int32_t *>(A.get((size_t)f->n_items * 4));
  f->item_seg = static_cast<int32_t *>(A.get((size_t)f->n_items * 4));
  if (!f->hub_rows || !f->hub_item_off || !f->item_row || !f->item_seg) return fail(PIPAD_ERR_ALLOC);

  int32_t max_nnz = 0;
  for (int t = 0; t < k; ++t) max_nnz = std::max(max_nnz, s.nnz[t]);
  if (max_nnz > 0)
    hipLaunchKernelGGL(k_scatter, grid1(max_nnz, kBlock, k + 1), dim3(kBlock), 0, st, s, p, pre,
                       f->dinv, n, k);
  hipLaunchKernelGGL(k_row_lists, grid1((int64_t)n + 1, kBlock), dim3(kBlock), 0, st, n, shortidx,
                     hubidx, segoff, f->rows_short, f->rows_long, f->hub_rows, f->hub_item_off,
                     f->item_row, f->item_seg);
  PIPAD_TRY(hipGetLastError());
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
