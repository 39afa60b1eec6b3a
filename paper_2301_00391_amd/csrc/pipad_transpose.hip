// pipad_frame_transpose: the frame of the transposed parts with the forward normalisation.
//
// Every part (the overlap part and the k exclusive parts) is transposed on its own - the transpose
// of an intersection is the intersection of the transposes - and all 1 + k parts go through the
// same launches.  Transposing a CSR pattern is a stable sort of its entries by column: rows arrive
// in ascending order, so they leave in ascending order within every column, which makes the result
// canonical CSR again.  The sort is a least-significant-digit radix sort on 7-bit digits of the
// column index (measured against 6 and 8 bits on frames of 0.2M to 1M nodes), written for
// 64-lane waves:
//
//   tiles      a part is cut into tiles of 2048 consecutive entries, one wave per tile
//   histogram  per tile and digit value; lanes of a wave that hold the same digit find each other
//              with one ballot per digit bit, and the lowest of them adds their number
//   scan       one exclusive prefix sum over all counts in (part, digit value, tile) order: the
//              position where a tile's entries with that digit start.  Parts never mix, because a
//              part's counts add up to its size
//   scatter    the wave goes through its tile 64 entries at a time, in order, and puts the tile in
//              digit order in LDS: an entry lands at start[digit] + (entries with the same digit in
//              lanes below), and the lowest lane of a digit moves start[digit] on.  The staged
//              tile is then written out in that order, neighbouring lanes to neighbouring
//              addresses (direct stores from the rounds go to 64 different places each: the
//              staged form is 1.3-1.9x faster for the whole call)
//
// Integer work with unique results: outputs are bit-exact regardless of scheduling.
#include <cstring>

#include "pipad_internal.h"

namespace pipad {
namespace {

#ifndef PIPAD_SORT_DIGIT
#define PIPAD_SORT_DIGIT 7
#endif
constexpr int kDigitBits = PIPAD_SORT_DIGIT;
constexpr int kDigits = 1 << kDigitBits;
#ifndef PIPAD_SORT_TILE
#define PIPAD_SORT_TILE 2048
#endif
constexpr int kTile = PIPAD_SORT_TILE;  // entries per wave
constexpr int kRounds = kTile / kWave;

struct SortArgs {
  int32_t nparts;                       // 1 + k
  int32_t n;
  uint32_t part_off[PIPAD_MAX_K + 2];   // first entry of every part in the concatenated arrays
  uint32_t tile_off[PIPAD_MAX_K + 2];   // first tile of every part
  uint32_t anchor_off[PIPAD_MAX_K + 2]; // first row anchor of every part (one per 64 entries, plus one)
  const int32_t *rowptr[PIPAD_MAX_K + 1];  // source parts
  const int32_t *col[PIPAD_MAX_K + 1];
  int32_t *rowptr_out[PIPAD_MAX_K + 1];    // transposed parts
  int32_t *col_out[PIPAD_MAX_K + 1];
  const uint32_t *key_in;
  const int32_t *val_in;
  uint32_t *key_out;
  int32_t *val_out;
  uint32_t *hist;                       // [sum over parts of kDigits * tiles of the part]
  uint32_t *cnt;                        // [tiles][kDigits]: the same counts, kept unscanned per tile
  int32_t shift;                        // digit = (key >> shift) & 255
  int32_t last;                         // last pass: values go to col_out of their part
};

// Part that holds position e of a concatenated array with the given part offsets.
__device__ inline int part_of(const uint32_t *off, int nparts, uint32_t e) {
  int p = 0;
  while (p + 1 < nparts && e >= off[p + 1]) ++p;
  return p;
}

// Last row i in [lo, hi] with rowptr[i] <= e, given rowptr[lo] <= e < rowptr[hi + 1].
__device__ inline int32_t row_of_entry(const int32_t *rp, int32_t lo, int32_t hi, int32_t e) {
  while (lo < hi) {
    const int32_t mid = lo + ((hi - lo + 1) >> 1);
    if (rp[mid] <= e) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// anchor[p's first anchor + w] = row of part p that holds the part's entry 64 w, for every w with
// 64 w < nnz_p, and one more slot per part that receives n - 1: one lane per (part, row) writes
// the (usually zero or one) slots whose entry falls into its row, so that the entries' rows can
// then be found by a search between two anchors instead of over all rows.
__global__ __launch_bounds__(kBlock) void k_row_anchors(SortArgs g, int32_t *anchor) {
  const int64_t id = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (id >= (int64_t)g.n * g.nparts) return;
  const int p = (int)(id / g.n);
  const int32_t i = (int32_t)(id - (int64_t)p * g.n);
  const int32_t a = g.rowptr[p][i], b = g.rowptr[p][i + 1];
  int32_t *mine = anchor + g.anchor_off[p];
  for (int64_t w = ((int64_t)a + kWave - 1) / kWave; w * kWave < b; ++w) mine[w] = i;
  if (i == g.n - 1) mine[((int64_t)b + kWave - 1) / kWave] = g.n - 1;
}

// Concatenates the parts: key = column of the entry, value = its row.  One lane per entry of a
// part, 64 consecutive entries per wave (the grid is cut per part: blockIdx.y), so the rows of a
// wave's entries lie between two neighbouring anchors.
__global__ __launch_bounds__(kBlock) void k_sort_input(SortArgs g, const int32_t *anchor,
                                                        uint32_t *key, int32_t *val) {
  const int p = blockIdx.y;
  const int64_t local64 = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int32_t nnz = (int32_t)(g.part_off[p + 1] - g.part_off[p]);
  if (local64 >= nnz) return;
  const int32_t local = (int32_t)local64;
  const int32_t *mine = anchor + g.anchor_off[p];
  const int32_t w = local / kWave;
  const int32_t r_lo = min(max(mine[w], 0), g.n - 1);
  const int32_t r_hi = min(max(mine[w + 1], r_lo), g.n - 1);
  const uint32_t e = g.part_off[p] + (uint32_t)local;
  key[e] = (uint32_t)g.col[p][local];
  val[e] = row_of_entry(g.rowptr[p], r_lo, r_hi, local);
}

// The lanes of the wave whose digit equals this lane's (bit set = same digit), lanes with
// `live` false excluded: one ballot per digit bit.
__device__ inline uint64_t same_digit(uint32_t digit, bool live) {
  uint64_t mask = __ballot(live);
#pragma unroll
  for (int b = 0; b < kDigitBits; ++b) {
    const bool bit = (digit >> b) & 1u;
    const uint64_t bal = __ballot(bit);
    mask &= bit ? bal : ~bal;
  }
  return mask;
}

struct TileRange {
  int p;
  uint32_t tile, tiles, begin, end;  // tile number within the part, tiles of the part, entries
};

__device__ inline TileRange tile_range(const SortArgs &g, uint32_t t) {
  TileRange r;
  r.p = part_of(g.tile_off, g.nparts, t);
  r.tile = t - g.tile_off[r.p];
  r.tiles = g.tile_off[r.p + 1] - g.tile_off[r.p];
  r.begin = g.part_off[r.p] + r.tile * (uint32_t)kTile;
  r.end = min(r.begin + (uint32_t)kTile, g.part_off[r.p + 1]);
  return r;
}

// hist[(first count of the part) + digit * tiles + tile] = entries of the tile with that digit.
__global__ __launch_bounds__(kBlock) void k_radix_hist(SortArgs g) {
  __shared__ uint32_t cnt[kWavesPerBlock][kDigits];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const uint32_t t = blockIdx.x * kWavesPerBlock + wave;
  if (t >= g.tile_off[g.nparts]) return;
  const TileRange r = tile_range(g, t);
  for (int d = lane; d < kDigits; d += kWave) cnt[wave][d] = 0;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  // the whole tile is requested up front (kRounds loads in flight per lane)
  uint32_t keys[kRounds];
#pragma unroll
  for (int q = 0; q < kRounds; ++q) {
    const uint32_t e = r.begin + q * kWave + lane;
    keys[q] = e < r.end ? g.key_in[e] : 0u;
  }
#pragma unroll
  for (int q = 0; q < kRounds; ++q) {
    const uint32_t e = r.begin + q * kWave + lane;
    const bool live = e < r.end;
    const uint32_t digit = (keys[q] >> g.shift) & (kDigits - 1);
    const uint64_t mask = same_digit(digit, live);
    if (live && (mask & ((1ull << lane) - 1ull)) == 0) cnt[wave][digit] += (uint32_t)__popcll(mask);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
  const uint64_t hbase = (uint64_t)kDigits * g.tile_off[r.p];
  for (int d = lane; d < kDigits; d += kWave) {
    g.hist[hbase + (uint64_t)d * r.tiles + r.tile] = cnt[wave][d];
    g.cnt[(uint64_t)t * kDigits + d] = cnt[wave][d];
  }
}

// Stable scatter of one tile by the current digit, from the scanned counts.  The tile is first
// put in digit order in LDS (an entry's place there: the tile's entries with smaller digits, plus
// those with the same digit in front of it), then written out in that order, so that neighbouring
// lanes store to neighbouring addresses: runs of tile / 2^bits entries per digit instead of 64
// different places per store.
constexpr int kScatterWaves = 2;  // per workgroup: 16 KB of staging each
static_assert((size_t)kScatterWaves * kTile * 8 <= 60 * 1024, "the staged tiles must fit the LDS of a workgroup");

__global__ __launch_bounds__(kScatterWaves * kWave) void k_radix_scatter(SortArgs g) {
  __shared__ uint32_t s_key[kScatterWaves][kTile];
  __shared__ int32_t s_val[kScatterWaves][kTile];
  __shared__ uint32_t lstart[kScatterWaves][kDigits];  // next free place of a digit within the tile
  __shared__ uint32_t gdelta[kScatterWaves][kDigits];  // global place = place within the tile + this
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const uint32_t t = blockIdx.x * kScatterWaves + wave;
  if (t >= g.tile_off[g.nparts]) return;
  const TileRange r = tile_range(g, t);
  const uint64_t hbase = (uint64_t)kDigits * g.tile_off[r.p];
  {
    uint32_t running = 0;
    for (int d0 = 0; d0 < kDigits; d0 += kWave) {
      const int d = d0 + lane;
      const uint32_t c = d < kDigits ? g.cnt[(uint64_t)t * kDigits + d] : 0u;
      uint32_t incl = c;
#pragma unroll
      for (int s2 = 1; s2 < kWave; s2 <<= 1) {
        const uint32_t up = __shfl_up(incl, s2, kWave);
        if (lane >= s2) incl += up;
      }
      const uint32_t excl = running + incl - c;
      if (d < kDigits) {
        lstart[wave][d] = excl;
        gdelta[wave][d] = g.hist[hbase + (uint64_t)d * r.tiles + r.tile] - excl;  // (mod 2^32)
      }
      running += __shfl(incl, kWave - 1, kWave);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  // the tile in two halves, each requested up front (kRounds / 2 loads in flight per lane)
  for (int half = 0; half < 2; ++half) {
    uint32_t keys[kRounds / 2];
    int32_t vals[kRounds / 2];
#pragma unroll
    for (int q = 0; q < kRounds / 2; ++q) {
      const uint32_t e = r.begin + (half * (kRounds / 2) + q) * kWave + lane;
      keys[q] = e < r.end ? g.key_in[e] : 0u;
      vals[q] = e < r.end ? g.val_in[e] : 0;
    }
#pragma unroll
    for (int q = 0; q < kRounds / 2; ++q) {
      const uint32_t e = r.begin + (half * (kRounds / 2) + q) * kWave + lane;
      const bool live = e < r.end;
      const uint32_t digit = (keys[q] >> g.shift) & (kDigits - 1);
      const uint64_t mask = same_digit(digit, live);
      const uint64_t below = mask & ((1ull << lane) - 1ull);
      uint32_t lpos = 0;
      if (live) lpos = lstart[wave][digit] + (uint32_t)__popcll(below);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // all reads of lstart before it moves on
      if (live && below == 0) lstart[wave][digit] += (uint32_t)__popcll(mask);
      if (live) {
        s_key[wave][lpos] = keys[q];
        s_val[wave][lpos] = vals[q];
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
  }
  int32_t *const dst_col = g.col_out[r.p];
  const uint32_t part_begin = g.part_off[r.p];
  const uint32_t here = r.end - r.begin;
  for (uint32_t j = lane; j < here; j += kWave) {
    const uint32_t key = s_key[wave][j];
    const int32_t val = s_val[wave][j];
    const uint32_t pos = gdelta[wave][(key >> g.shift) & (kDigits - 1)] + j;
    if (g.last) {
      dst_col[pos - part_begin] = val;  // the transposed part's column indices: the old rows
      g.key_out[pos] = key;             // (the sorted old columns still give the row pointers)
    } else {
      g.key_out[pos] = key;
      g.val_out[pos] = val;
    }
  }
}

// Row pointers of every transposed part from its sorted keys: rowptr[p][i] = keys of part p
// below i.  One lane per (part, i), i in [0, n].
__global__ __launch_bounds__(kBlock) void k_rowptr_of_sorted(SortArgs g, const uint32_t *keys) {
  const int64_t id = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t per = (int64_t)g.n + 1;
  if (id >= per * g.nparts) return;
  const int p = (int)(id / per);
  const uint32_t i = (uint32_t)(id - p * per);
  uint32_t lo = g.part_off[p], hi = g.part_off[p + 1];
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    if (keys[mid] < i) lo = mid + 1; else hi = mid;
  }
  g.rowptr_out[p][i] = (int32_t)(lo - g.part_off[p]);
}

// Column scales of the transposed parts' entries: wc[t][e] = dinv_t[col_c[e]] for the overlap
// part (a node's k scales from the node-major copy of D^-1/2), wd[t][e] = dinv_t[col_d_t[e]] for
// the exclusive part of snapshot t.  One lane per entry of the concatenated parts.
struct ScaleArgs {
  int32_t nparts, n, k;
  uint32_t part_off[PIPAD_MAX_K + 2];
  const int32_t *col[PIPAD_MAX_K + 1];
  const float *dinv, *dinv_nk;
  float *wc[PIPAD_MAX_K];
  float *wd[PIPAD_MAX_K];
};

// KV > 0: k == 4 * KV, a node's k scales are read as KV 16-byte pieces and the k destination
// arrays are fixed at compile time; KV == 0: any k, one by one.
template <int KV>
__global__ __launch_bounds__(kBlock) void k_part_scales(ScaleArgs g) {
  const int64_t e64 = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e64 >= g.part_off[g.nparts]) return;
  const uint32_t e = (uint32_t)e64;
  if (e < g.part_off[1]) {  // overlap part
    const int32_t c = g.col[0][e];
    if (KV > 0) {
      const float4 *row = reinterpret_cast<const float4 *>(g.dinv_nk) + (int64_t)c * KV;
      float4 v[KV > 0 ? KV : 1];
#pragma unroll
      for (int q = 0; q < KV; ++q) v[q] = row[q];
#pragma unroll
      for (int q = 0; q < KV; ++q) {
        g.wc[4 * q + 0][e] = v[q].x;
        g.wc[4 * q + 1][e] = v[q].y;
        g.wc[4 * q + 2][e] = v[q].z;
        g.wc[4 * q + 3][e] = v[q].w;
      }
    } else {
      const float *row = g.dinv_nk + (int64_t)c * g.k;
      for (int t = 0; t < g.k; ++t) g.wc[t][e] = row[t];
    }
  } else {
    const int p = part_of(g.part_off, g.nparts, e);
    const uint32_t local = e - g.part_off[p];
    const int32_t c = g.col[p][local];
    g.wd[p - 1][local] = g.dinv[(int64_t)(p - 1) * g.n + c];
  }
}

__global__ void k_class_totals(int32_t n, int32_t k, const uint32_t *hubidx, const uint32_t *segoff,
                               const uint32_t *shortidx, const uint32_t *split_total,
                               uint32_t *out) {
  const int q = threadIdx.x;
  if (q == 0) {
    out[0] = hubidx[n];
    out[1] = segoff[n];
    out[2] = shortidx[n];
  }
  if (q <= k) out[3 + q] = split_total[q];
}

}  // namespace

// The frame of the transposed patterns with the SAME D^-1/2: aggregating with it multiplies by
// the transposed normalised adjacency.
int transpose_frame(const pipad_frame *f, pipad_alloc_fn alloc, void *alloc_ctx, hipStream_t st,
                    pipad_frame **out) {
  const int32_t n = f->n, k = f->k;
  pipad_frame *g = new (std::nothrow) pipad_frame;
  if (!g) return PIPAD_ERR_ALLOC;
  g->n = n;
  g->k = k;
  g->device = f->device;
  g->own_memory = alloc == nullptr;
  g->alloc = alloc;
  g->alloc_ctx = alloc_ctx;
  g->opt = f->opt;  // the transposed frame keeps the options of the frame it comes from
  g->short_max = f->short_max;
  g->mid_max = f->mid_max;
  g->hub_threshold = f->hub_threshold;
  g->hub_segment = f->hub_segment;
  g->sub_log2 = f->sub_log2;
  g->nclass = f->nclass;
  g->nnz_c = f->nnz_c;
  for (int t = 0; t < k; ++t) g->nnz_d[t] = f->nnz_d[t];
  Allocator A{alloc, alloc_ctx, g};
  void *temp = nullptr;
  auto fail = [&](int code) {
    if (temp && !alloc) (void)hipFree(temp);
    release(g);
    return code;
  };
  auto hipcheck = [&](hipError_t e, const char *what) { return e == hipSuccess ? 0 : hip_fail(e, what); };
#define PIPAD_TRY_T(call)                                 \
  do {                                                    \
    int rc__ = hipcheck((call), #call);                   \
    if (rc__ != 0) return fail(rc__);                     \
  } while (0)

  Arena keep;
  keep.want(&g->rowptr_c, (size_t)n + 1);
  for (int t = 0; t < k; ++t) keep.want(&g->rowptr_d[t], (size_t)n + 1);
  keep.want(&g->dinv, (size_t)k * n);
  keep.want(&g->dinv_nk, (size_t)k * n);
  keep.want(&g->col_c, (size_t)g->nnz_c);
  for (int t = 0; t < k; ++t) {
    keep.want(&g->col_d[t], (size_t)g->nnz_d[t]);
    keep.want(&g->wc[t], (size_t)g->nnz_c);
    keep.want(&g->wd[t], (size_t)g->nnz_d[t]);
  }
  {
    void *base = A.get(keep.total);
    if (!base) return fail(PIPAD_ERR_ALLOC);
    keep.assign(base);
  }
  if (n == 0) {
    *out = g;
    return PIPAD_OK;
  }

  // ---- the parts side by side, cut into tiles
  SortArgs s;
  std::memset(&s, 0, sizeof(s));
  s.nparts = k + 1;
  s.n = n;
  int64_t total = 0, tiles = 0, anchors = 0;
  int32_t max_nnz = 0;
  for (int p = 0; p <= k; ++p) {
    const int32_t nnz = p == 0 ? f->nnz_c : f->nnz_d[p - 1];
    s.part_off[p] = (uint32_t)total;
    s.tile_off[p] = (uint32_t)tiles;
    s.anchor_off[p] = (uint32_t)anchors;
    total += nnz;
    tiles += (nnz + kTile - 1) / kTile;
    anchors += (nnz + kWave - 1) / kWave + 2;
    max_nnz = std::max(max_nnz, nnz);
    s.rowptr[p] = p == 0 ? f->rowptr_c : f->rowptr_d[p - 1];
    s.col[p] = p == 0 ? f->col_c : f->col_d[p - 1];
    s.rowptr_out[p] = p == 0 ? g->rowptr_c : g->rowptr_d[p - 1];
    s.col_out[p] = p == 0 ? g->col_c : g->col_d[p - 1];
  }
  s.part_off[k + 1] = (uint32_t)total;
  s.tile_off[k + 1] = (uint32_t)tiles;
  const int64_t hist_len = std::max<int64_t>(tiles * kDigits, 1);
  if (total >= ((int64_t)1 << 31) || hist_len >= ((int64_t)1 << 31)) return fail(PIPAD_ERR_TOO_LARGE);

  const uint32_t scan_len = (uint32_t)n + 1;
  Arena tmp;
  uint32_t *key_a = nullptr, *key_b = nullptr, *hist = nullptr, *cnt = nullptr, *bsum = nullptr, *shortidx = nullptr,
           *hubidx = nullptr, *segoff = nullptr, *totals = nullptr, *split_total = nullptr;
  int32_t *val_a = nullptr, *val_b = nullptr, *anchor = nullptr;
  tmp.want(&anchor, (size_t)anchors);
  tmp.want(&key_a, (size_t)total);
  tmp.want(&key_b, (size_t)total);
  tmp.want(&val_a, (size_t)total);
  tmp.want(&val_b, (size_t)total);
  tmp.want(&hist, (size_t)hist_len);
  tmp.want(&cnt, (size_t)hist_len);
  tmp.want(&bsum, std::max(scan_block_words((uint32_t)hist_len), 3 * scan_block_words(scan_len)) + 1);
  tmp.want(&shortidx, (size_t)scan_len);
  tmp.want(&hubidx, (size_t)scan_len);
  tmp.want(&segoff, (size_t)scan_len);
  tmp.want(&totals, (size_t)PIPAD_MAX_K + 8);
  tmp.want(&split_total, (size_t)PIPAD_MAX_K + 1);
  if (alloc) {
    temp = alloc(tmp.total, alloc_ctx);
    g->temp_ptr = temp;
    g->temp_bytes = temp ? tmp.total : 0;
  } else if (hipMalloc(&temp, tmp.total) != hipSuccess) {
    (void)hipGetLastError();
    temp = nullptr;
  }
  if (!temp) return fail(PIPAD_ERR_ALLOC);
  tmp.assign(temp);

  PIPAD_TRY_T(hipMemcpyAsync(g->dinv, f->dinv, sizeof(float) * (size_t)k * n,
                             hipMemcpyDeviceToDevice, st));
  PIPAD_TRY_T(hipMemcpyAsync(g->dinv_nk, f->dinv_nk, sizeof(float) * (size_t)k * n,
                             hipMemcpyDeviceToDevice, st));

  // ---- stable sort of all entries by column, digit by digit
  const uint32_t *sorted_keys = key_a;
  if (total > 0) {
    hipLaunchKernelGGL(k_row_anchors, grid1((int64_t)n * (k + 1), kBlock), dim3(kBlock), 0, st, s, anchor);
    hipLaunchKernelGGL(k_sort_input, grid1(max_nnz, kBlock, k + 1), dim3(kBlock), 0, st, s, anchor,
                       key_a, val_a);
    PIPAD_TRY_T(hipGetLastError());
    int bits = 1;
    while (((int64_t)1 << bits) < n) ++bits;
    const int passes = (bits + kDigitBits - 1) / kDigitBits;
    s.hist = hist;
    s.cnt = cnt;
    for (int pass = 0; pass < passes; ++pass) {
      s.key_in = pass % 2 == 0 ? key_a : key_b;
      s.val_in = pass % 2 == 0 ? val_a : val_b;
      s.key_out = pass % 2 == 0 ? key_b : key_a;
      s.val_out = pass % 2 == 0 ? val_b : val_a;
      s.shift = pass * kDigitBits;
      s.last = pass == passes - 1;
      hipLaunchKernelGGL(k_radix_hist, grid1(tiles, kWavesPerBlock), dim3(kBlock), 0, st, s);
      PIPAD_TRY_T(hipGetLastError());
      {
        uint32_t *one = hist;
        const int rc = scan_exclusive(&one, 1, (uint32_t)hist_len, bsum, st);
        if (rc != 0) return fail(rc);
      }
      hipLaunchKernelGGL(k_radix_scatter, grid1(tiles, kScatterWaves), dim3(kScatterWaves * kWave), 0, st, s);
      PIPAD_TRY_T(hipGetLastError());
      sorted_keys = s.key_out;
    }
  }
  hipLaunchKernelGGL(k_rowptr_of_sorted, grid1(((int64_t)n + 1) * (k + 1), kBlock), dim3(kBlock), 0, st,
                     s, sorted_keys);
  if (total > 0) {
    ScaleArgs c;
    std::memset(&c, 0, sizeof(c));
    c.nparts = k + 1;
    c.n = n;
    c.k = k;
    for (int p = 0; p <= k + 1; ++p) c.part_off[p] = s.part_off[p];
    for (int p = 0; p <= k; ++p) c.col[p] = s.col_out[p];
    c.dinv = g->dinv;
    c.dinv_nk = g->dinv_nk;
    for (int t = 0; t < k; ++t) {
      c.wc[t] = g->wc[t];
      c.wd[t] = g->wd[t];
    }
    auto scales = k == 4 ? k_part_scales<1> : k == 8 ? k_part_scales<2> : k == 16 ? k_part_scales<4>
                                                                                   : k_part_scales<0>;
    hipLaunchKernelGGL(scales, grid1(total, kBlock), dim3(kBlock), 0, st, c);
  }
  PIPAD_TRY_T(hipGetLastError());

  // ---- row classes, work lists and the class-grouped copies, as in the build
  {
    const int rc = launch_classify(g, shortidx, hubidx, segoff, split_total, st);
    if (rc != 0) return fail(rc);
  }
  {
    uint32_t *three[3] = {shortidx, hubidx, segoff};
    const int rc = scan_exclusive(three, 3, scan_len, bsum, st);
    if (rc != 0) return fail(rc);
  }
  uint32_t host_totals[PIPAD_MAX_K + 8] = {};
  hipLaunchKernelGGL(k_class_totals, dim3(1), dim3(kWave), 0, st, n, k, hubidx, segoff, shortidx,
                     split_total, totals);
  PIPAD_TRY_T(hipGetLastError());
  PIPAD_TRY_T(hipMemcpyAsync(host_totals, totals, sizeof(uint32_t) * (size_t)(k + 4),
                             hipMemcpyDeviceToHost, st));
  PIPAD_TRY_T(hipStreamSynchronize(st));
  {
    const int rc = set_list_sizes(g, host_totals[0], host_totals[1], host_totals[2], host_totals + 3);
    if (rc != 0) return fail(rc);
  }

  Arena lists;
  uint32_t *ulen = nullptr, *ubsum = nullptr;
  want_lists(lists, g, &ulen, &ubsum);
  {
    void *base = A.get(lists.total);
    if (!base) return fail(PIPAD_ERR_ALLOC);
    lists.assign(base);
  }
  launch_row_lists(n, shortidx, hubidx, segoff, g, st);
  PIPAD_TRY_T(hipGetLastError());
  {
    const int rc = build_split_arrays(g, ulen, ubsum, st);
    if (rc != 0) return fail(rc);
  }
  if (!alloc) {
    PIPAD_TRY_T(hipStreamSynchronize(st));  // the temporaries are freed next
    (void)hipFree(temp);
  }
#undef PIPAD_TRY_T
  *out = g;
  return PIPAD_OK;
}

}  // namespace pipad
