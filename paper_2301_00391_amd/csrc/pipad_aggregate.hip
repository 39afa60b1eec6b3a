// pipad_frame_aggregate: frame-parallel GCN neighbour aggregation on gfx950.
//
// Section 4.2 ("Dimension-aware parallel GNN"): the aggregation of a snapshot group is split into
// the parallel aggregation of the overlap adjacency with the features of ALL snapshots of the
// group (the coalescent features) and the per-snapshot aggregations of the exclusive parts.  Here
// both parts and the self-loop term of Eq. 1 are fused into one pass per destination row, so every
// output element is stored exactly once and no floating-point atomics are needed:
//
//   Y_t[i,:] = dinv_t[i] * ( sum_{j in common(i)} dinv_t[j] X_t[j,:]        (one index read, k gathers)
//                          + sum_{j in delta_t(i)} dinv_t[j] X_t[j,:]       (per snapshot)
//                          + dinv_t[i] X_t[i,:] )                           (self-loop)
//
// The overlap and exclusive parts are patterns; the per-snapshot normalisation
// D_t^-1/2 (A_t + I) D_t^-1/2 is applied as a column scale at the gather and a row scale at the
// store.  The memory path is the bound (sparse gathers, no dense contraction), so there is no MFMA.
//
// Work decomposition.  A *unit* is (row i, snapshot group g, range of the row's entries).  The
// lanes of a wave are split as  lane = (slot * SPA + s) * LPR + fl :
//   fl   LPR lanes, each owning VEC consecutive feature columns of one snapshot's row
//        (VEC = 4: one 16-byte load per lane, the "vector memory instruction" of Section 4.2);
//   s    SPA snapshots side by side; with H register rounds a lane group covers SPA*H snapshots,
//        so one decoded column index of the overlap part drives SPA*H row gathers;
//   slot the remaining lanes walk different entries of the same row (or different rows) and are
//        summed with cross-lane shuffles at the end.
// Rows longer than the frame's hub threshold are cut into fixed-size segments (the role the
// paper's sliced CSR plays for load balance, Section 4.1): each segment is a unit that writes a
// partial sum to scratch, and a second small kernel adds the partials of a row in a fixed order.
#include <algorithm>
#include <cstring>

#include "pipad_internal.h"

namespace pipad {
namespace {

struct AggArgs {
  int32_t n, k, F;
  int32_t lpr_log2;   // log2(LPR)
  int32_t spa_log2;   // log2(SPA)
  int32_t tg;         // snapshots per group (<= SPA * H)
  int32_t ngroups;    // ceil(k / tg)
  int32_t rowslots;   // 1: slots take different rows instead of different entries
  int32_t seg;        // entries per hub segment
  int32_t n_items, n_hub, item_blocks;
  int64_t ldx, ldy;
  const int32_t *rowptr_c, *col_c;
  const float *dinv;
  const uint8_t *rowclass;
  const int32_t *item_row, *item_seg, *hub_rows, *hub_item_off;
  float *partial;
  const int32_t *rowptr_d[PIPAD_MAX_K];
  const int32_t *col_d[PIPAD_MAX_K];
  const float *X[PIPAD_MAX_K];
  float *Y[PIPAD_MAX_K];
};

template <int VEC> struct V;
template <> struct V<4> {
  using T = float4;
  static __device__ inline T zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
  static __device__ inline T load(const float *p) { return *reinterpret_cast<const float4 *>(p); }
  static __device__ inline void store(float *p, T v) { *reinterpret_cast<float4 *>(p) = v; }
  static __device__ inline void fma(T &a, float w, T x) {
    a.x = fmaf(w, x.x, a.x); a.y = fmaf(w, x.y, a.y); a.z = fmaf(w, x.z, a.z); a.w = fmaf(w, x.w, a.w);
  }
  static __device__ inline void add(T &a, T b) { a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }
  static __device__ inline T scale(float w, T a) { return make_float4(w * a.x, w * a.y, w * a.z, w * a.w); }
  static __device__ inline T shfl_xor(T v, int m) {
    return make_float4(__shfl_xor(v.x, m, kWave), __shfl_xor(v.y, m, kWave),
                       __shfl_xor(v.z, m, kWave), __shfl_xor(v.w, m, kWave));
  }
};
template <> struct V<1> {
  using T = float;
  static __device__ inline T zero() { return 0.f; }
  static __device__ inline T load(const float *p) { return *p; }
  static __device__ inline void store(float *p, T v) { *p = v; }
  static __device__ inline void fma(T &a, float w, T x) { a = fmaf(w, x, a); }
  static __device__ inline void add(T &a, T b) { a += b; }
  static __device__ inline T scale(float w, T a) { return w * a; }
  static __device__ inline T shfl_xor(T v, int m) { return __shfl_xor(v, m, kWave); }
};

// Per-lane view of the snapshots this lane serves.
template <int H>
struct LaneCtx {
  const float *xb[H];     // X_t + feature column
  const float *dv[H];     // dinv_t
  const int32_t *rpd[H];  // rowptr of delta_t
  const int32_t *cd[H];   // columns of delta_t
  float *yb[H];
  bool on[H];             // lane has a snapshot in round h and a valid feature column
};

template <int H>
__device__ inline void lane_setup(const AggArgs &a, int t0, int s, int fcol, bool fvalid,
                                  LaneCtx<H> &c) {
  const int spa = 1 << a.spa_log2;
#pragma unroll
  for (int h = 0; h < H; ++h) {
    const int rel = s + spa * h;
    int t = t0 + rel;
    const bool on = fvalid && rel < a.tg && t < a.k;
    if (!on) t = t0;  // a safe snapshot; contributions are masked out
    c.on[h] = on;
    c.xb[h] = a.X[t] + (on ? fcol : 0);
    c.yb[h] = a.Y[t] + (on ? fcol : 0);
    c.dv[h] = a.dinv + (int64_t)t * a.n;
    c.rpd[h] = a.rowptr_d[t];
    c.cd[h] = a.col_d[t];
  }
}

// Adds to acc[] the entries at positions [v0, v1) of row i's virtual list
// (common entries first, then, per snapshot, its exclusive entries), taking positions
// v0 + slot, v0 + slot + nslots, ...
template <int H, int VEC>
__device__ inline void accumulate_range(const AggArgs &a, const LaneCtx<H> &c, int32_t i,
                                        int32_t v0, int32_t v1, int slot, int nslots,
                                        typename V<VEC>::T acc[H]) {
  using VT = V<VEC>;
  constexpr int U = H >= 8 ? 1 : (8 / H > 4 ? 4 : 8 / H);  // entries in flight per lane
  const int32_t cs = a.rowptr_c[i];
  const int32_t lc = a.rowptr_c[i + 1] - cs;
  const int64_t ldx = a.ldx;

  // ---- overlap part: one index, all snapshots of the group
  const int32_t cend = min(v1, lc);
  for (int32_t p = v0 + slot; p < cend; p += nslots * U) {
    int32_t j[U];
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int32_t pp = p + u * nslots;
      live[u] = pp < cend;
      j[u] = live[u] ? a.col_c[cs + pp] : i;
    }
    float w[U][H];
    typename VT::T x[U][H];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int h = 0; h < H; ++h) {
        w[u][h] = (live[u] && c.on[h]) ? c.dv[h][j[u]] : 0.f;
        x[u][h] = VT::load(c.xb[h] + (int64_t)j[u] * ldx);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int h = 0; h < H; ++h) VT::fma(acc[h], w[u][h], x[u][h]);
    }
  }

  // ---- exclusive parts: every snapshot walks its own list; lane groups of different
  //      snapshots run side by side
  const int32_t q0 = max(v0 - lc, 0);
  const int64_t q1v = (int64_t)v1 - lc;  // may be negative or huge
  int32_t ds[H], q1[H];
  int32_t qmax = 0;
#pragma unroll
  for (int h = 0; h < H; ++h) {
    ds[h] = c.rpd[h][i];
    const int32_t ld = c.rpd[h][i + 1] - ds[h];
    q1[h] = c.on[h] ? (int32_t)max((int64_t)0, min((int64_t)ld, q1v)) : 0;
    qmax = max(qmax, q1[h]);
  }
  constexpr int UD = 2;
  for (int32_t q = q0 + slot; q < qmax; q += nslots * UD) {
    int32_t j[UD][H];
    bool live[UD][H];
#pragma unroll
    for (int u = 0; u < UD; ++u) {
#pragma unroll
      for (int h = 0; h < H; ++h) {
        const int32_t qq = q + u * nslots;
        live[u][h] = qq < q1[h];
        j[u][h] = live[u][h] ? c.cd[h][ds[h] + qq] : i;
      }
    }
#pragma unroll
    for (int u = 0; u < UD; ++u) {
#pragma unroll
      for (int h = 0; h < H; ++h) {
        const float w = live[u][h] ? c.dv[h][j[u][h]] : 0.f;
        const typename VT::T x = VT::load(c.xb[h] + (int64_t)j[u][h] * ldx);
        VT::fma(acc[h], w, x);
      }
    }
  }
}

// Sums acc over the slot lanes of a wave (slot bits are the high lane bits).
template <int H, int VEC>
__device__ inline void reduce_slots(int unit_lanes_log2, typename V<VEC>::T acc[H]) {
  for (int m = kWave >> 1; m >= (1 << unit_lanes_log2); m >>= 1) {
#pragma unroll
    for (int h = 0; h < H; ++h) V<VEC>::add(acc[h], V<VEC>::shfl_xor(acc[h], m));
  }
}

// Self-loop term, row scale, store.
template <int H, int VEC>
__device__ inline void finish_row(const AggArgs &a, const LaneCtx<H> &c, int32_t i,
                                  typename V<VEC>::T acc[H]) {
  using VT = V<VEC>;
#pragma unroll
  for (int h = 0; h < H; ++h) {
    if (c.on[h]) {
      const float di = c.dv[h][i];
      typename VT::T xi = VT::load(c.xb[h] + (int64_t)i * a.ldx);
      VT::fma(acc[h], di, xi);
      VT::store(c.yb[h] + (int64_t)i * a.ldy, VT::scale(di, acc[h]));
    }
  }
}

// Main kernel.  Workgroups [0, item_blocks * ngroups) process hub segments (wave per segment),
// the rest process ordinary rows (wave per row, or per 64/unit_lanes rows with rowslots).
// Consecutive workgroups take consecutive snapshot groups of the same rows, so that with one
// snapshot per group the k slices of a coalescent row are gathered on k different XCDs
// (workgroups are dealt round-robin to the 8 XCDs, each with a private L2).
template <int H, int VEC>
__global__ __launch_bounds__(kBlock) void k_aggregate(const AggArgs a) {
  using VT = V<VEC>;
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int lpr = 1 << a.lpr_log2;
  const int unit_log2 = a.lpr_log2 + a.spa_log2;
  const int fl = lane & (lpr - 1);
  const int s = (lane >> a.lpr_log2) & ((1 << a.spa_log2) - 1);
  const int slot = lane >> unit_log2;
  const int nslots = kWave >> unit_log2;

  const int64_t b = blockIdx.x;
  const int g = (int)(b % a.ngroups);
  const int64_t bb = b / a.ngroups;
  const int t0 = g * a.tg;
  const bool item_path = bb < a.item_blocks;

  for (int fbase = 0; fbase < a.F; fbase += lpr * VEC) {
    const int fcol = fbase + fl * VEC;
    const bool fvalid = fcol < a.F;
    LaneCtx<H> c;
    lane_setup<H>(a, t0, s, fcol, fvalid, c);
    typename VT::T acc[H];
#pragma unroll
    for (int h = 0; h < H; ++h) acc[h] = VT::zero();

    if (item_path) {
      const int64_t item = bb * kWavesPerBlock + wave;
      if (item >= a.n_items) return;
      const int32_t i = a.item_row[item];
      const int32_t sg = a.item_seg[item];
      accumulate_range<H, VEC>(a, c, i, sg * a.seg, (sg + 1) * a.seg, slot, nslots, acc);
      reduce_slots<H, VEC>(unit_log2, acc);
      if (slot == 0) {
#pragma unroll
        for (int h = 0; h < H; ++h) {
          if (c.on[h]) {
            const int t = t0 + s + (h << a.spa_log2);
            VT::store(a.partial + ((int64_t)item * a.k + t) * a.F + fcol, acc[h]);
          }
        }
      }
    } else {
      const int64_t rb = (bb - a.item_blocks) * kWavesPerBlock + wave;
      if (a.rowslots) {
        const int64_t i64 = rb * nslots + slot;
        if (i64 < a.n && !a.rowclass[i64]) {
          const int32_t i = (int32_t)i64;
          accumulate_range<H, VEC>(a, c, i, 0, INT32_MAX, 0, 1, acc);
          finish_row<H, VEC>(a, c, i, acc);
        }
      } else {
        if (rb >= a.n) return;
        const int32_t i = (int32_t)rb;
        if (a.rowclass[i]) return;
        accumulate_range<H, VEC>(a, c, i, 0, INT32_MAX, slot, nslots, acc);
        reduce_slots<H, VEC>(unit_log2, acc);
        if (slot == 0) finish_row<H, VEC>(a, c, i, acc);
      }
    }
  }
}

// Adds the partial sums of every hub row in a fixed order and finishes the row.
// One wave per (hub row, snapshot group); slots stride over the row's segments.
template <int H, int VEC>
__global__ __launch_bounds__(kBlock) void k_hub_finish(const AggArgs a) {
  using VT = V<VEC>;
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int lpr = 1 << a.lpr_log2;
  const int unit_log2 = a.lpr_log2 + a.spa_log2;
  const int fl = lane & (lpr - 1);
  const int s = (lane >> a.lpr_log2) & ((1 << a.spa_log2) - 1);
  const int slot = lane >> unit_log2;
  const int nslots = kWave >> unit_log2;
  const int64_t b = blockIdx.x;
  const int g = (int)(b % a.ngroups);
  const int64_t hr = (b / a.ngroups) * kWavesPerBlock + wave;
  if (hr >= a.n_hub) return;
  const int t0 = g * a.tg;
  const int32_t i = a.hub_rows[hr];
  const int32_t it0 = a.hub_item_off[hr], it1 = a.hub_item_off[hr + 1];
  for (int fbase = 0; fbase < a.F; fbase += lpr * VEC) {
    const int fcol = fbase + fl * VEC;
    LaneCtx<H> c;
    lane_setup<H>(a, t0, s, fcol, fcol < a.F, c);
    typename VT::T acc[H];
#pragma unroll
    for (int h = 0; h < H; ++h) acc[h] = VT::zero();
    for (int32_t it = it0 + slot; it < it1; it += nslots) {
#pragma unroll
      for (int h = 0; h < H; ++h) {
        if (c.on[h]) {
          const int t = t0 + s + (h << a.spa_log2);
          VT::add(acc[h], VT::load(a.partial + ((int64_t)it * a.k + t) * a.F + fcol));
        }
      }
    }
    reduce_slots<H, VEC>(unit_log2, acc);
    if (slot == 0) finish_row<H, VEC>(a, c, i, acc);
  }
}

inline int ceil_log2(int64_t x) {
  int l = 0;
  while (((int64_t)1 << l) < x) ++l;
  return l;
}

template <int H, int VEC>
int launch(const AggArgs &a, hipStream_t st) {
  const int unit_log2 = a.lpr_log2 + a.spa_log2;
  const int nslots = kWave >> unit_log2;
  const int64_t rows_per_block = (int64_t)kWavesPerBlock * (a.rowslots ? nslots : 1);
  const int64_t row_blocks = (a.n + rows_per_block - 1) / rows_per_block;
  const int64_t blocks = ((int64_t)a.item_blocks + row_blocks) * a.ngroups;
  if (blocks >= ((int64_t)1 << 31)) return PIPAD_ERR_TOO_LARGE;
  if (blocks > 0)
    hipLaunchKernelGGL((k_aggregate<H, VEC>), dim3((unsigned)blocks), dim3(kBlock), 0, st, a);
  if (a.n_hub > 0) {
    const int64_t hb = ((int64_t)a.n_hub + kWavesPerBlock - 1) / kWavesPerBlock * a.ngroups;
    hipLaunchKernelGGL((k_hub_finish<H, VEC>), dim3((unsigned)hb), dim3(kBlock), 0, st, a);
  }
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

}  // namespace

int aggregate_launch(pipad_frame *f, int32_t F, const float *const *X, int64_t ldx,
                     float *const *Y, int64_t ldy, hipStream_t st) {
  if (f->n == 0) return PIPAD_OK;
  AggArgs a;
  std::memset(&a, 0, sizeof(a));
  a.n = f->n;
  a.k = f->k;
  a.F = F;
  a.ldx = ldx;
  a.ldy = ldy;
  a.rowptr_c = f->rowptr_c;
  a.col_c = f->col_c;
  a.dinv = f->dinv;
  a.rowclass = f->rowclass;
  a.item_row = f->item_row;
  a.item_seg = f->item_seg;
  a.hub_rows = f->hub_rows;
  a.hub_item_off = f->hub_item_off;
  a.seg = f->hub_segment;
  a.n_items = f->n_items;
  a.n_hub = f->n_hub;
  a.item_blocks = (f->n_items + kWavesPerBlock - 1) / kWavesPerBlock;
  bool vec4 = F % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0;
  for (int t = 0; t < f->k; ++t) {
    a.rowptr_d[t] = f->rowptr_d[t];
    a.col_d[t] = f->col_d[t];
    a.X[t] = X[t];
    a.Y[t] = Y[t];
    if ((reinterpret_cast<uintptr_t>(X[t]) | reinterpret_cast<uintptr_t>(Y[t])) & 15u) vec4 = false;
  }

  // scratch for hub partial sums
  const size_t need = (size_t)f->n_items * (size_t)f->k * (size_t)F;
  if (need > f->partial_floats) {
    void *ptr = nullptr;
    if (f->alloc) {
      // the caller's allocator owns the memory; a smaller buffer from before stays with it
      ptr = f->alloc(need * sizeof(float), f->alloc_ctx);
      if (!ptr) return PIPAD_ERR_ALLOC;
    } else {
      // the old buffer may still be in use by earlier work on another stream of the caller
      PIPAD_HIP(hipDeviceSynchronize());
      if (f->partial) (void)hipFree(f->partial);
      f->partial = nullptr;
      f->partial_floats = 0;
      if (hipMalloc(&ptr, need * sizeof(float)) != hipSuccess) {
        (void)hipGetLastError();
        return PIPAD_ERR_ALLOC;
      }
    }
    f->partial = static_cast<float *>(ptr);
    f->partial_floats = need;
  }
  a.partial = f->partial;

  // lane layout
  const int vec = vec4 ? 4 : 1;
  const int chunks = (F + vec - 1) / vec;                  // lanes wanted for one snapshot's row
  a.lpr_log2 = std::min(6, ceil_log2(chunks));
  const int lanes_left_log2 = 6 - a.lpr_log2;
  int variant = (int)options().agg_variant;
  if (variant == 0) variant = 1;
  int H = 1;
  if (variant == 2) {
    a.spa_log2 = 0;
    a.tg = 1;
  } else {
    a.spa_log2 = std::min(lanes_left_log2, ceil_log2(f->k));
    const int spa = 1 << a.spa_log2;
    const int rounds = (f->k + spa - 1) / spa;
    H = rounds >= 8 ? 8 : rounds > 2 ? 4 : rounds;  // 1, 2, 4 or 8 register rounds
    a.tg = std::min<int>(f->k, spa * H);
  }
  a.ngroups = (f->k + a.tg - 1) / a.tg;
  a.rowslots = options().agg_rowslots ? 1 : 0;

  if (vec4) {
    switch (H) {
      case 1: return launch<1, 4>(a, st);
      case 2: return launch<2, 4>(a, st);
      case 4: return launch<4, 4>(a, st);
      default: return launch<8, 4>(a, st);
    }
  }
  switch (H) {
    case 1: return launch<1, 1>(a, st);
    case 2: return launch<2, 1>(a, st);
    case 4: return launch<4, 1>(a, st);
    default: return launch<8, 1>(a, st);
  }
}

}  // namespace pipad
