// pipad_frame_aggregate: frame-parallel GCN neighbour aggregation on gfx950.
//
// Section 4.2 ("Dimension-aware parallel GNN"): the aggregation of a snapshot group is split into
// the parallel aggregation of the overlap adjacency with the features of ALL snapshots of the
// group (the coalescent features) and the per-snapshot aggregations of the exclusive parts.  Here
// both parts and the self-loop term of Eq. 1 are fused into one pass per destination row, so every
// output element is stored exactly once and no floating-point atomics are needed:
//
//   Y_t[i,:] = dinv_t[i] * ( sum_{e in common(i)}  wc_t[e] X_t[col_c[e],:]
//                          + sum_{e in delta_t(i)} wd_t[e] X_t[col_d_t[e],:]
//                          + dinv_t[i] X_t[i,:] )                            (self-loop)
//
// with wc_t[e] = dinv_t[col_c[e]], wd_t[e] = dinv_t[col_d_t[e]] stored per entry by the build, so
// the per-snapshot normalisation D_t^-1/2 (A_t + I) D_t^-1/2 costs a streamed float per entry
// instead of a gathered cache line.  The memory path is the bound (sparse row gathers, no dense
// contraction), so there is no MFMA.
//
// How one launch covers the frame.  The coalescent feature row of a node (k snapshots x F
// columns) is cut into *slices* of at most 64 columns of one snapshot.  A workgroup works on ONE
// slice, and consecutive workgroups take consecutive slices: workgroups are dealt round-robin to
// the 8 XCDs, each with a private 4 MB L2, so with k = 8 every XCD gathers one snapshot's slice of
// every row and its L2 only has to hold 1/8 of each hot row.  The overlap CSR is read from HBM
// once and reaches the other XCDs through the memory-side cache.
//
// Work items of a slice, by row length L = common + longest exclusive row (binned by the build):
//   short rows  a team of LS lanes (LS * VEC = slice width) per row, 64/LS rows side by side in
//               a wave, 64 rows per wave; row metadata for the 64 rows is loaded in one go.
//   long rows   a wave per row; the 64/LS lane teams take different entries and are summed with
//               cross-lane shuffles.
//   hub rows    cut into segments (the role the paper's sliced CSR plays for load balance,
//               Section 4.1); a wave per segment writes a partial sum, and a second small kernel
//               adds the partials of a row in a fixed order.
// Entries are fetched a team-wide chunk at a time (one coalesced load of indices and scales) and
// handed to the lanes with ds_bpermute, so the inner loop issues only the 16-byte row gathers
// (the "vector memory instruction" of Section 4.2), several of them in flight per lane.
#include <algorithm>
#include <cstring>

#include "pipad_internal.h"

namespace pipad {
namespace {

constexpr int kShortRowsPerWave = 64;

struct AggArgs {
  int32_t n, k, F;
  int32_t ls_log2;    // log2 of the lanes per slice row
  int32_t fchunks;    // slices per snapshot = ceil(F / (LS * VEC))
  int32_t nslices;    // k * fchunks
  int32_t seg;        // entries per hub segment
  int32_t n_short, n_long, n_items, n_hub;
  int32_t blocks_items, blocks_long;  // workgroups per slice for the first two item kinds
  int32_t nt;         // non-temporal hints (bit 0: Y stores, bit 1: index streams)
  int32_t parts;      // timing aid: which kinds of work items run (all in normal use)
  int64_t ldx, ldy;
  const int32_t *rowptr_c, *col_c;
  const float *dinv;
  const int32_t *rows_short, *rows_long;
  const int32_t *item_row, *item_seg, *hub_rows, *hub_item_off;
  float *partial;
  const int32_t *rowptr_d[PIPAD_MAX_K];
  const int32_t *col_d[PIPAD_MAX_K];
  const float *wc[PIPAD_MAX_K];
  const float *wd[PIPAD_MAX_K];
  const float *X[PIPAD_MAX_K];
  float *Y[PIPAD_MAX_K];
};

template <int VEC> struct V;
template <> struct V<4> {
  using T = float4;
  static __device__ inline T zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
  static __device__ inline T load(const float *p) { return *reinterpret_cast<const float4 *>(p); }
  static __device__ inline void store(float *p, T v, bool nt) {
    if (nt) {
      typedef float f4 __attribute__((ext_vector_type(4)));
      f4 q = {v.x, v.y, v.z, v.w};
      __builtin_nontemporal_store(q, reinterpret_cast<f4 *>(p));
    } else {
      *reinterpret_cast<float4 *>(p) = v;
    }
  }
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
  static __device__ inline void store(float *p, T v, bool nt) {
    if (nt) __builtin_nontemporal_store(v, p); else *p = v;
  }
  static __device__ inline void fma(T &a, float w, T x) { a = fmaf(w, x, a); }
  static __device__ inline void add(T &a, T b) { a += b; }
  static __device__ inline T scale(float w, T a) { return w * a; }
  static __device__ inline T shfl_xor(T v, int m) { return __shfl_xor(v, m, kWave); }
};

// What a lane needs to know about its slice.
struct Slice {
  const float *xb;          // X_t + feature column of this lane
  float *yb;                // Y_t + feature column of this lane
  const float *dv;          // dinv_t
  const float *wc, *wd;     // per-entry column scales of the common / exclusive part
  const int32_t *rpd, *cd;  // exclusive CSR of snapshot t
  int fcol;
  bool fvalid;              // the lane's columns exist (F need not fill the last slice)
};

__device__ inline Slice slice_setup(const AggArgs &a, int slice, int fl, int vec) {
  Slice s;
  const int t = slice / a.fchunks;
  const int fc = slice - t * a.fchunks;
  s.fcol = (fc << a.ls_log2) * vec + fl * vec;
  s.fvalid = s.fcol < a.F;
  const int col = s.fvalid ? s.fcol : 0;  // idle lanes read column 0 and never store
  s.xb = a.X[t] + col;
  s.yb = a.Y[t] + col;
  s.dv = a.dinv + (int64_t)t * a.n;
  s.wc = a.wc[t];
  s.wd = a.wd[t];
  s.rpd = a.rowptr_d[t];
  s.cd = a.col_d[t];
  return s;
}

// Adds sum_e w[e] * X[col[e], :] over the `len` entries starting at `start` to acc.
//   team_base  first lane of the team; team_lanes lanes fetch a chunk of entries together
//   q          this lane's index within the team
//   slot/nslots  the team's lane groups take entries slot, slot + nslots, ... of each chunk
// Every lane of a team runs the same number of iterations (entries past the end are given weight
// zero and the row's own index), so ds_bpermute never reads from a lane that has left the loop.
template <int VEC, int UNR>
__device__ inline void walk(const int32_t *__restrict__ col, const float *__restrict__ w,
                            int32_t start, int32_t len, int team_base, int team_lanes, int q,
                            int slot, int nslots, const float *xb, int64_t ldx, int32_t self,
                            bool nt, typename V<VEC>::T &acc) {
  using VT = V<VEC>;
  for (int32_t base = 0; base < len; base += team_lanes) {
    const int32_t cnt = min(team_lanes, len - base);
    int32_t myc = self;
    float myw = 0.f;
    if (q < cnt) {
      if (nt) {
        myc = __builtin_nontemporal_load(col + start + base + q);
        myw = __builtin_nontemporal_load(w + start + base + q);
      } else {
        myc = col[start + base + q];
        myw = w[start + base + q];
      }
    }
    for (int32_t e0 = 0; e0 < cnt; e0 += nslots * UNR) {
      int32_t j[UNR];
      float wt[UNR];
      typename VT::T x[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int32_t e = e0 + u * nslots + slot;
        const int src = team_base + (e < cnt ? e : 0);
        j[u] = __shfl(myc, src, kWave);
        wt[u] = __shfl(myw, src, kWave);
        if (e >= cnt) { j[u] = self; wt[u] = 0.f; }
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) x[u] = VT::load(xb + (int64_t)j[u] * ldx);
#pragma unroll
      for (int u = 0; u < UNR; ++u) VT::fma(acc, wt[u], x[u]);
    }
  }
}

// Self-loop term, row scale, store.
template <int VEC>
__device__ inline void finish_row(const AggArgs &a, const Slice &s, int32_t i, float di,
                                  typename V<VEC>::T acc) {
  using VT = V<VEC>;
  typename VT::T xi = VT::load(s.xb + (int64_t)i * a.ldx);
  VT::fma(acc, di, xi);
  VT::store(s.yb + (int64_t)i * a.ldy, VT::scale(di, acc), a.nt & 1);
}

template <int VEC>
__device__ inline void reduce_slots(int ls_log2, typename V<VEC>::T &acc) {
  for (int m = kWave >> 1; m >= (1 << ls_log2); m >>= 1) V<VEC>::add(acc, V<VEC>::shfl_xor(acc, m));
}

template <int VEC>
__global__ __launch_bounds__(kBlock) void k_aggregate(const AggArgs a) {
  using VT = V<VEC>;
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int ls = 1 << a.ls_log2;
  const int fl = lane & (ls - 1);
  const int team = lane >> a.ls_log2;  // lane group index within the wave
  const int nteams = kWave >> a.ls_log2;

  const int64_t b = blockIdx.x;
  const int slice = (int)(b % a.nslices);
  int64_t w = b / a.nslices;
  const Slice s = slice_setup(a, slice, fl, VEC);
  const bool ntl = a.nt & 2;

  if (w < a.blocks_items) {
    // ---- one segment of a hub row per wave
    const int64_t item = w * kWavesPerBlock + wave;
    if (item >= a.n_items || !(a.parts & 1)) return;
    const int32_t i = a.item_row[item];
    const int32_t v0 = a.item_seg[item] * a.seg, v1 = v0 + a.seg;
    const int32_t cs = a.rowptr_c[i], lc = a.rowptr_c[i + 1] - cs;
    const int32_t ds = s.rpd[i], ld = s.rpd[i + 1] - ds;
    typename VT::T acc = VT::zero();
    // positions [v0, v1) of the virtual list "common entries, then exclusive entries"
    const int32_t c0 = min(v0, lc), c1 = min(v1, lc);
    walk<VEC, 8>(a.col_c, s.wc, cs + c0, c1 - c0, 0, kWave, lane, team, nteams, s.xb, a.ldx, i, ntl, acc);
    const int32_t d0 = min(max(v0 - lc, 0), ld), d1 = min(max(v1 - lc, 0), ld);
    walk<VEC, 8>(s.cd, s.wd, ds + d0, d1 - d0, 0, kWave, lane, team, nteams, s.xb, a.ldx, i, ntl, acc);
    reduce_slots<VEC>(a.ls_log2, acc);
    if (team == 0 && s.fvalid)
      VT::store(a.partial + (((int64_t)item * a.nslices + slice) << a.ls_log2) * VEC + fl * VEC, acc, false);
    return;
  }
  w -= a.blocks_items;
  if (w < a.blocks_long) {
    // ---- one long row per wave
    const int64_t li = w * kWavesPerBlock + wave;
    if (li >= a.n_long || !(a.parts & 2)) return;
    const int32_t i = a.rows_long[li];
    const int32_t cs = a.rowptr_c[i], lc = a.rowptr_c[i + 1] - cs;
    const int32_t ds = s.rpd[i], ld = s.rpd[i + 1] - ds;
    typename VT::T acc = VT::zero();
    walk<VEC, 8>(a.col_c, s.wc, cs, lc, 0, kWave, lane, team, nteams, s.xb, a.ldx, i, ntl, acc);
    walk<VEC, 8>(s.cd, s.wd, ds, ld, 0, kWave, lane, team, nteams, s.xb, a.ldx, i, ntl, acc);
    reduce_slots<VEC>(a.ls_log2, acc);
    if (team == 0 && s.fvalid) finish_row<VEC>(a, s, i, s.dv[i], acc);
    return;
  }
  w -= a.blocks_long;
  // ---- 64 short rows per wave, one team per row, nteams rows side by side
  const int64_t first = (w * kWavesPerBlock + wave) * kShortRowsPerWave;
  if (first >= a.n_short || !(a.parts & 4)) return;
  int32_t r = 0, c0 = 0, c1 = 0, d0 = 0, d1 = 0;
  float di = 0.f;
  if (first + lane < a.n_short) {  // metadata of row `lane` of this wave's 64
    r = a.rows_short[first + lane];
    c0 = a.rowptr_c[r]; c1 = a.rowptr_c[r + 1];
    d0 = s.rpd[r]; d1 = s.rpd[r + 1];
    di = s.dv[r];
  }
  const int rows_here = (int)min((int64_t)kShortRowsPerWave, a.n_short - first);
  for (int step = 0; step * nteams < rows_here; ++step) {
    const int li = step * nteams + team;
    const bool have = li < rows_here;
    const int src = have ? li : 0;
    const int32_t i = __shfl(r, src, kWave);
    const int32_t cs = __shfl(c0, src, kWave);
    const int32_t ce = __shfl(c1, src, kWave);
    const int32_t ds = __shfl(d0, src, kWave);
    const int32_t de = __shfl(d1, src, kWave);
    const float dii = __shfl(di, src, kWave);
    if (have) {
      typename VT::T acc = VT::zero();
      walk<VEC, 4>(a.col_c, s.wc, cs, ce - cs, team << a.ls_log2, ls, fl, 0, 1, s.xb, a.ldx, i, ntl, acc);
      walk<VEC, 4>(s.cd, s.wd, ds, de - ds, team << a.ls_log2, ls, fl, 0, 1, s.xb, a.ldx, i, ntl, acc);
      if (s.fvalid) finish_row<VEC>(a, s, i, dii, acc);
    }
  }
}

// Adds the partial sums of every hub row in a fixed order and finishes the row.
// One wave per (hub row, slice); the lane teams stride over the row's segments.
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_hub_finish(const AggArgs a) {
  using VT = V<VEC>;
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int ls = 1 << a.ls_log2;
  const int fl = lane & (ls - 1);
  const int team = lane >> a.ls_log2;
  const int nteams = kWave >> a.ls_log2;
  const int64_t b = blockIdx.x;
  const int slice = (int)(b % a.nslices);
  const int64_t hr = (b / a.nslices) * kWavesPerBlock + wave;
  if (hr >= a.n_hub) return;
  const Slice s = slice_setup(a, slice, fl, VEC);
  const int32_t i = a.hub_rows[hr];
  const int32_t it0 = a.hub_item_off[hr], it1 = a.hub_item_off[hr + 1];
  typename VT::T acc = VT::zero();
  if (s.fvalid)
    for (int32_t it = it0 + team; it < it1; it += nteams)
      VT::add(acc, VT::load(a.partial + (((int64_t)it * a.nslices + slice) << a.ls_log2) * VEC + fl * VEC));
  reduce_slots<VEC>(a.ls_log2, acc);
  if (team == 0 && s.fvalid) finish_row<VEC>(a, s, i, s.dv[i], acc);
}

inline int ceil_log2(int64_t x) {
  int l = 0;
  while (((int64_t)1 << l) < x) ++l;
  return l;
}

template <int VEC>
int launch(const AggArgs &a, hipStream_t st) {
  const int64_t blocks_short =
      ((int64_t)a.n_short + kShortRowsPerWave * kWavesPerBlock - 1) / (kShortRowsPerWave * kWavesPerBlock);
  const int64_t blocks = ((int64_t)a.blocks_items + a.blocks_long + blocks_short) * a.nslices;
  if (blocks >= ((int64_t)1 << 31)) return PIPAD_ERR_TOO_LARGE;
  if (blocks > 0)
    hipLaunchKernelGGL((k_aggregate<VEC>), dim3((unsigned)blocks), dim3(kBlock), 0, st, a);
  if (a.n_hub > 0) {
    const int64_t hb = ((int64_t)a.n_hub + kWavesPerBlock - 1) / kWavesPerBlock * a.nslices;
    hipLaunchKernelGGL((k_hub_finish<VEC>), dim3((unsigned)hb), dim3(kBlock), 0, st, a);
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
  a.rows_short = f->rows_short;
  a.rows_long = f->rows_long;
  a.item_row = f->item_row;
  a.item_seg = f->item_seg;
  a.hub_rows = f->hub_rows;
  a.hub_item_off = f->hub_item_off;
  a.seg = f->hub_segment;
  a.n_short = f->n_short;
  a.n_long = f->n_long;
  a.n_items = f->n_items;
  a.n_hub = f->n_hub;
  a.blocks_items = (f->n_items + kWavesPerBlock - 1) / kWavesPerBlock;
  a.blocks_long = (f->n_long + kWavesPerBlock - 1) / kWavesPerBlock;
  a.nt = (int32_t)options().agg_nt;
  a.parts = (int32_t)options().agg_parts;
  bool vec4 = F % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0;
  for (int t = 0; t < f->k; ++t) {
    a.rowptr_d[t] = f->rowptr_d[t];
    a.col_d[t] = f->col_d[t];
    a.wc[t] = f->wc[t];
    a.wd[t] = f->wd[t];
    a.X[t] = X[t];
    a.Y[t] = Y[t];
    if ((reinterpret_cast<uintptr_t>(X[t]) | reinterpret_cast<uintptr_t>(Y[t])) & 15u) vec4 = false;
  }
  // slice geometry: LS lanes of VEC columns each, at most 64 columns per slice
  const int vec = vec4 ? 4 : 1;
  const int max_cols = 64;
  const int cols = std::min(F, max_cols);
  a.ls_log2 = ceil_log2((cols + vec - 1) / vec);
  const int sw = (1 << a.ls_log2) * vec;
  a.fchunks = (F + sw - 1) / sw;
  a.nslices = f->k * a.fchunks;

  // scratch for the partial sums of hub segments: n_items x nslices x slice width
  const size_t need = (size_t)f->n_items * (size_t)a.nslices * (size_t)sw;
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
  return vec4 ? launch<4>(a, st) : launch<1>(a, st);
}

}  // namespace pipad
