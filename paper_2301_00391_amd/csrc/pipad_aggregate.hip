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
// columns) is cut into *slices* of at most 64 columns of one snapshot, and the launch goes through
// the slices one after the other (workgroups are dispatched in index order): the whole chip works
// on one snapshot's matrix at a time, so the caches see one matrix instead of k.
//
// Column classes.  The chip has 8 XCDs, each with a private 4 MB L2; workgroup b runs on XCD
// b mod 8.  A feature row that all 8 L2s cache occupies 8 times its size, and the gathered rows of
// a power-law graph do not fit one L2.  So every column belongs to one of 8 classes (a hash of its
// index), the entries of the long ("hub") rows are stored a second time, grouped by class, and
// the part of a row that falls into class x is walked by a workgroup whose index is x mod 8: XCD x
// only ever gathers class x, and the 8 L2s together act as one cache of 32 MB.  The price is that
// such a row is summed in 8 parts; the partial sums go through a scratch buffer and a second small
// kernel adds them in a fixed order, applies the self-loop term and the row scale, and stores the
// row.  Measured, the 8 partial sums (written and read back through memory) only pay for rows of
// several hundred entries, so the other rows - most rows, and on graphs of moderate skew most
// entries - are walked whole.
//
// Work items of a slice, by row length L = common + longest exclusive row (binned by the build):
//   hub rows    split by class; a wave per class part, the 64/LS lane teams take different
//               entries and are summed with cross-lane shuffles.  Rows beyond hub_threshold
//               entries are first cut into units (the role the paper's sliced CSR plays for load
//               balance, Section 4.1).
//   mid rows    walked whole by a wave, the same way; self-loop, row scale and store at once.
//   short rows  walked whole: a team of LS lanes (LS * VEC = slice width) per row, 64/LS rows
//               side by side, row metadata for a whole batch loaded in one go.
// Entries are fetched a team-wide chunk at a time (one coalesced load of indices and scales),
// turned into 32-bit row offsets and handed to the lane teams through LDS, so the inner loop
// issues only the 16-byte row gathers (the "vector memory instruction" of Section 4.2), four of
// them in flight per lane; the next chunk and the next row's first chunk are requested early.
#include <algorithm>
#include <cstring>
#include <mutex>

#include "pipad_internal.h"

#ifndef PIPAD_ORDER_BYTES
#define PIPAD_ORDER_BYTES (28 << 20)
#endif
#ifndef PIPAD_ROW_ORDER_A
#define PIPAD_ROW_ORDER_A 3  // short rows of a batch are taken longest first when 2 * longest > A * mean + B
#define PIPAD_ROW_ORDER_B 2  // (in gather rounds per row)
#endif
#ifndef PIPAD_PARTIAL_NT
#define PIPAD_PARTIAL_NT 0
#endif

namespace pipad {
namespace {

// Most rows a wave takes one after the other (lane l holds the metadata of row l of the batch).
// The launch lowers these for small frames, so that the chip still gets enough waves.
constexpr int kShortRowsPerWave = 64;  // short rows, a lane team per row
constexpr int kLongRowsPerWave = 8;    // mid rows, a wave per row
#ifndef PIPAD_WIDE_BATCH
#define PIPAD_WIDE_BATCH 4
#endif
constexpr int kWideUnitsPerWave = PIPAD_WIDE_BATCH;   // class parts of hub units, a wave per part

struct AggArgs {
  int32_t n, k, F;
  int32_t ls_log2;    // log2 of the lanes per slice row
  int32_t fchunks;    // slices per snapshot = ceil(F / (LS * VEC))
  int32_t nslices;    // k * fchunks
  int32_t nsel;       // snapshots this call aggregates (k, or fewer for a subset call)
  uint64_t sel[4];    // their numbers, one byte each, in the order they are taken
  int32_t n_short, n_long, n_items, n_hub;
  // workgroups of one slice ("phase"): for every sub class in turn 8 * blocks_wide for the hub
  // units (workgroup r of them takes XCD r mod 8's class), then blocks_mid for the mid rows, then
  // blocks_short (padded so that every phase starts at a multiple of 8 and the XCD a workgroup is
  // meant for is the one it runs on)
  int32_t blocks_wide, blocks_mid, blocks_short;
  int32_t batch_short, batch_mid, batch_wide;  // rows / class parts per wave
  int64_t blocks_per_phase;
  int32_t order;      // 1: one slice after the other; 0: hub class parts so, the rows of all slices side by side
  int32_t sub_log2;   // log2 of the sub classes per XCD
  int32_t nclass;     // 8 << sub_log2
  int64_t nv;         // class parts per part of the frame = nclass * n_units
  int64_t nvp;        // partial sums per slice: nclass per hub unit
  int32_t nt;         // non-temporal hints (bit 0: Y stores, bit 1: index streams)
  int32_t sg;         // coalescent kernel: snapshots per lane team (slices are snapshot groups)
  int64_t ldx, ldy;
  const int32_t *rowptr_c, *col_c;
  const float *dinv;
  const int32_t *rows_short, *rows_long;
  const int32_t *item_row, *item_v0, *item_v1, *hub_rows, *hub_item_off;
  const uint32_t *sptr;   // class parts of the split rows: see pipad_frame
  const int32_t *scol;
  const float *swd;
  int64_t total_c;        // entries of the common region of scol
  float *partial;
  const int32_t *rowptr_d[PIPAD_MAX_K];
  const int32_t *col_d[PIPAD_MAX_K];
  const float *wc[PIPAD_MAX_K];
  const float *wd[PIPAD_MAX_K];
  const float *swc[PIPAD_MAX_K];
  const float *X[PIPAD_MAX_K];
  float *Y[PIPAD_MAX_K];   // aggregation results (optional when the update is fused in)
  // fused update: H_t = Y_t W + bias
  const float *W;          // [F][Fo], row stride ldw
  const float *bias;       // [Fo] or null
  int32_t Fo;
  int64_t ldw, ldh;
  float *H[PIPAD_MAX_K];
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
template <> struct V<2> {
  using T = float2;
  static __device__ inline T zero() { return make_float2(0.f, 0.f); }
  static __device__ inline T load(const float *p) { return *reinterpret_cast<const float2 *>(p); }
  static __device__ inline void store(float *p, T v, bool) { *reinterpret_cast<float2 *>(p) = v; }
  static __device__ inline void fma(T &a, float w, T x) { a.x = fmaf(w, x.x, a.x); a.y = fmaf(w, x.y, a.y); }
  static __device__ inline void add(T &a, T b) { a.x += b.x; a.y += b.y; }
  static __device__ inline T scale(float w, T a) { return make_float2(w * a.x, w * a.y); }
  static __device__ inline T shfl_xor(T v, int m) {
    return make_float2(__shfl_xor(v.x, m, kWave), __shfl_xor(v.y, m, kWave));
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
  int t;                    // snapshot
  const float *xt;          // X_t (the same for the whole workgroup)
  const float *xb;          // X_t + feature column of this lane
  float *yb;                // Y_t + feature column of this lane (null: not wanted)
  float *ht;                // H_t (fused update only)
  const float *dv;          // dinv_t
  const float *wc, *wd;     // per-entry column scales of the common / exclusive part (short rows)
  const int32_t *rpd, *cd;  // exclusive CSR of snapshot t (short rows)
  const float *swc;         // column scales of the common region of the class-grouped entries
  int fcol;
  bool fvalid;              // the lane's columns exist (F need not fill the last slice)
};

// slice -> (snapshot, column chunk): slice = chunk * k + snapshot
__device__ __forceinline__ Slice slice_setup(const AggArgs &a, int slice, int fl, int vec) {
  Slice s;
  // (the slice is the same for the whole workgroup: saying so lets the per-snapshot pointers come
  // from the kernel arguments through the scalar unit)
  slice = __builtin_amdgcn_readfirstlane(slice);
  const int fc = slice / a.k;
  const int t = slice - fc * a.k;
  s.t = t;
  s.fcol = (fc << a.ls_log2) * vec + fl * vec;
  s.fvalid = s.fcol < a.F;
  const int col = s.fvalid ? s.fcol : 0;  // idle lanes read column 0 and never store
  s.xt = a.X[t];
  s.xb = a.X[t] + col;
  s.yb = a.Y[t] ? a.Y[t] + col : nullptr;
  s.ht = a.H[t];
  s.dv = a.dinv + (int64_t)t * a.n;
  s.wc = a.wc[t];
  s.wd = a.wd[t];
  s.rpd = a.rowptr_d[t];
  s.cd = a.col_d[t];
  s.swc = a.swc[t];
  return s;
}

// One entry as fetched (column index and column scale) ...
struct Raw {
  int32_t c;
  float w;
};
// ... and as staged in LDS for the lane groups: where its feature row starts, and the scale.
struct Staged {
  uint32_t off;  // FAST: byte offset of row c within the slice's matrix; else c itself
  float w;
};

// Entry base + q of a list, or (own row, weight 0) past its end: such a filler may be gathered
// harmlessly, which lets the FAST inner loop run without bounds checks.
__device__ __forceinline__ Raw fetch_entry(const int32_t *__restrict__ col, const float *__restrict__ w,
                                  int32_t start, int32_t len, int32_t pos, int32_t self, bool nt) {
  Raw r;
  r.c = self;
  r.w = 0.f;
  if (pos < len) {
    if (nt) {
      r.c = __builtin_nontemporal_load(col + start + pos);
      r.w = __builtin_nontemporal_load(w + start + pos);
    } else {
      r.c = col[start + pos];
      r.w = w[start + pos];
    }
  }
  return r;
}

// Adds sum_e w[e] * X[col[e], :] over the `len` entries starting at `start` to acc.
//   first      entry q of the list, already fetched by the caller (fetch_entry(..., q, ...))
//   team_base  first lane of the team; team_lanes lanes fetch a chunk of entries together
//   q          this lane's index within the team
//   slot/nslots  the team's lane groups take entries slot, slot + nslots, ... of each chunk
//   lds        this wave's 64 staging slots
// A chunk is fetched with one coalesced load of indices and scales (the next chunk is requested
// before the current chunk's gathers), turned into row offsets once per entry, and parked in LDS;
// every lane group then picks its entry up with a single 8-byte LDS read, so the inner loop is
// one LDS read, one add, one 16-byte gather and VEC fused multiply-adds per entry.
// The FAST inner loop needs nslots * UNR to divide team_lanes.
template <int VEC, int UNR, bool FAST>
__device__ __forceinline__ void walk(const int32_t *__restrict__ col, const float *__restrict__ w,
                            int32_t start, int32_t len, Raw first, int team_base, int team_lanes,
                            int q, int slot, int nslots, const Slice &s, int64_t ldx, int32_t self,
                            bool nt, Staged *lds, typename V<VEC>::T &acc) {
  using VT = V<VEC>;
  if (len <= 0) return;
  const uint32_t row_bytes = (uint32_t)ldx * 4u;
  // FAST addressing: wave-uniform matrix base + 32-bit (row offset + this lane's column offset)
  const char *xbytes = reinterpret_cast<const char *>(s.xt);
  const uint32_t lane_bytes = (uint32_t)(s.fvalid ? s.fcol : 0) * 4u;
  const float *xcol = s.xb;
  Raw mine = first, next = first;
  for (int32_t base = 0; base < len; base += team_lanes) {
    const int32_t cnt = min(team_lanes, len - base);
    if (base + team_lanes < len) next = fetch_entry(col, w, start, len, base + team_lanes + q, self, nt);
    Staged st;
    st.off = FAST ? (uint32_t)mine.c * row_bytes : (uint32_t)mine.c;
    st.w = mine.w;
    lds[team_base + q] = st;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    for (int32_t e0 = 0; e0 < cnt; e0 += nslots * UNR) {
      Staged en[UNR];
      typename VT::T x[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        int32_t e = e0 + u * nslots + slot;
        if (!FAST) e = min(e, team_lanes - 1);
        en[u] = lds[team_base + e];
        if (!FAST && e0 + u * nslots + slot >= cnt) en[u].w = 0.f;
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
#ifdef PIPAD_NO_GATHER  // measurement builds: everything but the row gathers (wrong results)
        x[u] = VT::zero();
#else
        if (FAST)
          x[u] = VT::load(reinterpret_cast<const float *>(xbytes + (en[u].off + lane_bytes)));
        else
          x[u] = VT::load(xcol + (int64_t)en[u].off * ldx);
#endif
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) VT::fma(acc, en[u].w, x[u]);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    mine = next;
  }
}

// ---- fused update (one GCN layer: the fully connected update applied to the aggregation result,
// Eq. 1; the weights stay on chip for every row of every snapshot a workgroup meets: the
// weight reuse of Section 4.2) ----------------------------------------------------------------
// A wave parks finished rows (the slice is the whole row of one snapshot here, K = 4 * LS columns)
// in a 16-row LDS tile and multiplies a full tile by W with fp32 MFMA 16x16x4 instructions:
//   A operand  lane (m = lane % 16, g = lane / 16) supplies tile[m][g * KS + ks] at step ks
//   B operand  the same lane supplies W[g * KS + ks][16 * nt + m]
// (the instruction sums its four k values over g; KS = K / 4 steps cover every k once), and the
// result comes back as D[4 * g + r][m] in register r.
constexpr int kTileRows = 16;
constexpr int kTileStride = 68;  // floats per tile row: 64 + 4, keeps 16-byte alignment

struct Sink {
  float *tile;        // this wave's [kTileRows][kTileStride]
  int32_t *rows;      // this wave's [kTileRows] row ids
  const float *wl;    // the workgroup's W in LDS: [K][Fo + 1], then the bias as row K
  int cnt;            // rows parked (wave-uniform)
};

typedef float mfma_f4 __attribute__((ext_vector_type(4)));

template <int KS>  // k values per lane group = lanes per row
__device__ __forceinline__ void sink_flush_ks(const AggArgs &a, const Slice &s, Sink &k, int lane) {
  const int m = lane & 15, g = lane >> 4;
  float av[KS];
#pragma unroll
  for (int q = 0; q < KS / 4; ++q) {
    const float4 v = *reinterpret_cast<const float4 *>(k.tile + m * kTileStride + g * KS + 4 * q);
    av[4 * q + 0] = v.x; av[4 * q + 1] = v.y; av[4 * q + 2] = v.z; av[4 * q + 3] = v.w;
  }
  int32_t row[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) row[r] = k.rows[min(4 * g + r, kTileRows - 1)];
  const int ws = a.Fo + 1;
  for (int nt = 0; nt < a.Fo / 16; ++nt) {
    const float *wcol = k.wl + (g * KS) * ws + 16 * nt + m;
    const float b = k.wl[(4 * KS) * ws + 16 * nt + m];  // the bias sits behind W's last row
    mfma_f4 d = {0.f, 0.f, 0.f, 0.f};
    constexpr int KB = KS < 8 ? KS : 8;  // operand reads issued together (more would spill)
#pragma unroll
    for (int k0 = 0; k0 < KS; k0 += KB) {
      float bv[KB];
#pragma unroll
      for (int ks = 0; ks < KB; ++ks) bv[ks] = wcol[(k0 + ks) * ws];
#pragma unroll
      for (int ks = 0; ks < KB; ++ks)
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(av[k0 + ks], bv[ks], d, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (4 * g + r < k.cnt) s.ht[(int64_t)row[r] * a.ldh + 16 * nt + m] = d[r] + b;
  }
}

__device__ __forceinline__ void sink_flush(const AggArgs &a, const Slice &s, Sink &k, int lane) {
  if (k.cnt == 0) return;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  switch (a.ls_log2) {
    case 2: sink_flush_ks<4>(a, s, k, lane); break;
    case 3: sink_flush_ks<8>(a, s, k, lane); break;
    default: sink_flush_ks<16>(a, s, k, lane); break;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  k.cnt = 0;
}

// Self-loop term and row scale; the row goes to the tile (and to Y_t when that is wanted).
__device__ __forceinline__ void finish_row_to_sink(const AggArgs &a, const Slice &s, Sink &k, int slot, int fl,
                                          int32_t i, float di, float4 xi, float4 acc) {
  using VT = V<4>;
  VT::fma(acc, di, xi);
  float4 y = VT::scale(di, acc);
  if (!s.fvalid) y = make_float4(0.f, 0.f, 0.f, 0.f);  // columns past F pad K with zeros
  else if (s.yb) VT::store(s.yb + (int64_t)i * a.ldy, y, a.nt & 1);
  *reinterpret_cast<float4 *>(k.tile + slot * kTileStride + fl * 4) = y;
  if (fl == 0) k.rows[slot] = i;
}

// Self-loop term, row scale, store.
template <int VEC>
__device__ __forceinline__ void finish_row(const AggArgs &a, const Slice &s, int32_t i, float di,
                                  typename V<VEC>::T xi, typename V<VEC>::T acc) {
  using VT = V<VEC>;
  VT::fma(acc, di, xi);
  VT::store(s.yb + (int64_t)i * a.ldy, VT::scale(di, acc), a.nt & 1);
}

template <int VEC>
__device__ __forceinline__ void reduce_slots(int ls_log2, typename V<VEC>::T &acc) {
  for (int m = kWave >> 1; m >= (1 << ls_log2); m >>= 1) V<VEC>::add(acc, V<VEC>::shfl_xor(acc, m));
}

constexpr bool kPartialNt = PIPAD_PARTIAL_NT;  // non-temporal stores for the partial sums

// The t_seq-th snapshot this call aggregates (all four words are read before one is chosen, so
// that the kernel arguments are only read at constant offsets).
__device__ __forceinline__ int selected_snapshot(const AggArgs &a, int t_seq) {
  const uint64_t w0 = a.sel[0], w1 = a.sel[1], w2 = a.sel[2], w3 = a.sel[3];
  const uint64_t w = t_seq < 8 ? w0 : t_seq < 16 ? w1 : t_seq < 24 ? w2 : w3;
  return (int)((w >> ((t_seq & 7) * 8)) & 0xffu);
}

// Where partial sum `slot` (= hub unit * nclass + class) of the slice_seq-th slice of the call
// goes: all partial sums of one slice are contiguous, so a phase writes and the finishing kernel
// reads dense memory, and a call over some of the snapshots needs room for those only.
__device__ __forceinline__ float *partial_slot(const AggArgs &a, int slice_seq, int64_t slot, int fl, int vec) {
  return a.partial + (((int64_t)slice_seq * a.nvp + slot) << a.ls_log2) * vec + fl * vec;
}

template <int VEC, bool FAST, int U, bool UPD>
__device__ __forceinline__ void aggregate_body(const AggArgs &a) {
  using VT = V<VEC>;
  static_assert(!UPD || (VEC == 4 && FAST), "the fused update rides on the fast float4 path");
  extern __shared__ __align__(16) float upd_lds[];  // UPD: W [K][Fo + 1], then the waves' tiles and row ids
  Sink sink;
  if (UPD) {
    const int K = 4 << a.ls_log2, ws = a.Fo + 1;
    for (int idx = threadIdx.x; idx < K * a.Fo; idx += kBlock) {
      const int kk = idx / a.Fo, o = idx - kk * a.Fo;
      upd_lds[kk * ws + o] = kk < a.F ? a.W[(int64_t)kk * a.ldw + o] : 0.f;
    }
    // row K: the bias (a load from global memory inside the flush would make the wave wait for
    // every gather it has in flight)
    for (int o = threadIdx.x; o < a.Fo; o += kBlock) upd_lds[K * ws + o] = a.bias ? a.bias[o] : 0.f;
    const int w_floats = ((K + 1) * ws + 3) & ~3;
    float *tiles = upd_lds + w_floats;
    sink.wl = upd_lds;
    sink.tile = tiles + (threadIdx.x / kWave) * kTileRows * kTileStride;
    sink.rows = reinterpret_cast<int32_t *>(tiles + kWavesPerBlock * kTileRows * kTileStride) +
                (threadIdx.x / kWave) * kTileRows;
    sink.cnt = 0;
    __syncthreads();  // before any wave leaves
  }
  // Row gathers in flight per lane.  Measured on MI355X (N = 1M R-MAT frame): 4 beats 2 and 8 on
  // both paths; deeper bursts only queue up in front of the L1's miss slots.  Teams of fewer
  // than 4 lanes get U = LS so that U entries per lane group still fit the 64 staged entries.
  constexpr int UL = FAST ? U : 1;  // wave-wide teams (hub units)
  constexpr int US = FAST ? U : 1;  // row-wide teams (mid and short rows)
  __shared__ Staged staging[kWavesPerBlock][kWave];
  Staged *lds = staging[threadIdx.x / kWave];
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int ls = 1 << a.ls_log2;
  const int fl = lane & (ls - 1);
  const int team = lane >> a.ls_log2;  // lane group index within the wave
  const int nteams = kWave >> a.ls_log2;

  // Workgroups are dispatched in index order and dealt round-robin to the XCDs: the launch goes
  // through the slices (snapshot-major) one after the other, and within a slice's class parts the
  // class of a workgroup is its index mod 8.
  const int64_t b = blockIdx.x;
  const int nsub = 1 << a.sub_log2;
  const int64_t wide_blocks = (int64_t)kClasses * a.blocks_wide;  // per sub class
  const int64_t split_blocks = nsub * wide_blocks;
  int slice_seq;
  int64_t w;  // workgroup index within the slice's phase: class parts, mid rows, short rows
  if (a.order == 1) {
    slice_seq = (int)(b / a.blocks_per_phase);
    w = b - slice_seq * a.blocks_per_phase;
  } else {
    // Side by side: neighbouring workgroups take the same rows in different slices, so the
    // entry lists they share (the overlap part's indices, the row pointers) are fetched once for
    // all of them - what pays while the operand is small next to the index streams.  The class
    // parts keep their slice-after-slice order in front (their class is the workgroup index mod 8).
    const int nsl = a.nsel * a.fchunks;
    const int64_t hub_total = split_blocks * nsl;
    if (b < hub_total) {
      slice_seq = (int)(b / split_blocks);
      w = b - slice_seq * split_blocks;
    } else {
      const int64_t r = b - hub_total;
      slice_seq = (int)(r % nsl);
      w = split_blocks + r / nsl;
    }
  }
  const int t_seq = slice_seq / a.fchunks;
  const int slice = (slice_seq - t_seq * a.fchunks) * a.k + selected_snapshot(a, t_seq);
  const Slice s = slice_setup(a, slice, fl, VEC);
  const bool ntl = a.nt & 2;

  // ---- what this wave works on: a batch of consecutive list elements.  Class parts of hub units
  //      (from the class-grouped copies, ending in a partial sum) and whole mid rows: the whole
  //      wave on one list at a time, its lane groups taking different entries.  Short rows: one
  //      lane group each, nteams side by side.  The metadata of the whole batch is loaded up front
  //      (lane l holds element l of the batch), and while one element is being gathered the first
  //      chunk of entries (and, for whole rows, the self-loop row) of the next one are already on
  //      their way.
  // (every field is read into a local before the control flow that chooses among them, so that
  // the kernel arguments are only ever read at constant offsets)
  const int32_t *const p_items = a.item_row, *const p_mid = a.rows_long, *const p_short = a.rows_short;
  const int64_t n_items = a.n_items, n_mid = a.n_long, n_short = a.n_short;
  const int b_wide = a.batch_wide, b_mid = a.batch_mid, b_short = a.batch_short;
  const bool split = w < split_blocks;                  // class parts of hub units
#ifdef PIPAD_SPLIT_TEAM  // measurement builds: class parts walked by lane teams like short rows
  const bool wide = !split && w < split_blocks + a.blocks_mid;
#else
  const bool wide = w < split_blocks + a.blocks_mid;    // ... or whole mid rows: a wave per list
#endif
  int cls = 0;  // column class of this wave's class parts
  if (split) {
    const int sub = (int)(w / wide_blocks);  // the sub classes come one after the other in time
    w -= sub * wide_blocks;
    cls = ((int)(w & (kClasses - 1)) << a.sub_log2) + sub;
    w >>= 3;
  } else if (wide) {
    w -= split_blocks;
  } else {
    w -= split_blocks + a.blocks_mid;
  }
  const int32_t *list = split ? p_items : wide ? p_mid : p_short;
  const int64_t list_len = split ? n_items : wide ? n_mid : n_short;
  const int batch = split ? b_wide : wide ? b_mid : b_short;
  const int64_t first = (w * kWavesPerBlock + wave) * batch;
  if (first >= list_len) return;
#ifdef PIPAD_PARTS_MASK  // measurement builds only: which kinds of work items run (results incomplete)
  if (!((PIPAD_PARTS_MASK) & (split ? 1 : wide ? 2 : 4))) return;
#endif
  const int rows_here = (int)min((int64_t)batch, list_len - first);
  // entry lists: the class-grouped copies for hub units, the frame's CSRs for whole rows
  const int32_t *colc = split ? a.scol : a.col_c;
  const float *wcs = split ? s.swc : s.wc;
  const int32_t *cold = split ? a.scol + a.total_c : s.cd;
  const float *wds = split ? a.swd : s.wd;
  // hub units only: first class part in sptr == first partial sum; nclass of them per unit
  const int64_t v_first = first * a.nclass + cls;
  int32_t r = 0, mc0 = 0, mc1 = 0, md0 = 0, md1 = 0;
  float mdi = 0.f;
  if (lane < rows_here) {
    r = list[first + lane];
    if (split) {
      const int64_t v = v_first + (int64_t)lane * a.nclass;
      mc0 = (int32_t)a.sptr[v];
      mc1 = (int32_t)a.sptr[v + 1];
      const int64_t vd = (int64_t)(1 + s.t) * a.nv + v;
      md0 = (int32_t)((int64_t)a.sptr[vd] - a.total_c);
      md1 = (int32_t)((int64_t)a.sptr[vd + 1] - a.total_c);
    } else {
      mc0 = a.rowptr_c[r]; mc1 = a.rowptr_c[r + 1];
      md0 = s.rpd[r]; md1 = s.rpd[r + 1];
      mdi = s.dv[r];
    }
  }
  // Short rows: nteams rows are walked side by side and a step lasts as long as its longest
  // row.  Where the lengths within a batch differ a lot (skewed graphs: the longest row takes more
  // than 1.5 times the mean number of gather rounds plus one) the wave takes its rows in order of
  // decreasing work: a stable 5-bit radix sort over the lanes, ballots and one cross-lane move per
  // bit.  order = index within the batch of the row taken as number `lane`; which rows a wave
  // works on does not change.  Not for slices narrower than a cache line, where neighbouring
  // rows share lines, and not for batches of similar rows, where the natural order keeps the
  // rows of a step next to each other in memory (measured: 4 % faster on the R-MAT frame, 2-8 %
  // slower on Chung-Lu frames and narrow slices when applied regardless).
  int order = lane;
#ifndef PIPAD_NO_ROW_ORDER
  if (!wide && ((VEC * 4) << a.ls_log2) >= 128) {
    constexpr int gpl = US;  // entries a lane group gathers per round
    const int rounds = lane < rows_here ? (mc1 - mc0 + gpl - 1) / gpl + (md1 - md0 + gpl - 1) / gpl : 0;
    int mx = rounds, sm = rounds;
#pragma unroll
    for (int m = kWave >> 1; m >= 1; m >>= 1) {
      mx = max(mx, __shfl_xor(mx, m, kWave));
      sm += __shfl_xor(sm, m, kWave);
    }
    if (2 * mx * rows_here > PIPAD_ROW_ORDER_A * sm + PIPAD_ROW_ORDER_B * rows_here) {  // wave-uniform
      int packed = (min(rounds, 31) << 8) | lane;
#pragma unroll
      for (int bit = 8; bit < 13; ++bit) {
        const bool one = (packed >> bit) & 1;
        const uint64_t ones = __ballot(one);
        const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(ones >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ones, 0));
        const int dest = one ? below : __popcll(ones) + (lane - below);
        packed = __builtin_amdgcn_ds_permute(dest << 2, packed);
      }
      order = packed & 0xff;
    }
  }
#endif
  const int per_step = wide ? 1 : nteams;          // elements worked on side by side
  const int team_base = wide ? 0 : team << a.ls_log2;
  const int team_lanes = wide ? kWave : ls;
  const int q = wide ? lane : fl;
  const int slot = wide ? team : 0;
  const int nslots = wide ? nteams : 1;

  struct Item {
    int src;  // place of the element in the wave's batch
    int32_t i, cs, clen, ds, dlen;
    float di;
    bool have;
    Raw fc, fd;
    typename VT::T xi;
  };
  auto prefetch = [&](int step) __attribute__((always_inline)) {
    Item it;
    const int li = step * per_step + (wide ? 0 : team);
    it.have = li < rows_here;
    const int src = __shfl(order, it.have ? li : 0, kWave);
    it.src = src;
    it.i = __shfl(r, src, kWave);
    it.cs = __shfl(mc0, src, kWave);
    it.clen = __shfl(mc1, src, kWave) - it.cs;
    it.ds = __shfl(md0, src, kWave);
    it.dlen = __shfl(md1, src, kWave) - it.ds;
    it.di = __shfl(mdi, src, kWave);
    if (!it.have) { it.clen = 0; it.dlen = 0; }
    it.fc = fetch_entry(colc, wcs, it.cs, it.clen, q, it.i, ntl);
    it.fd = fetch_entry(cold, wds, it.ds, it.dlen, q, it.i, ntl);
    it.xi = VT::zero();
    if (!split) it.xi = VT::load(s.xb + (int64_t)it.i * a.ldx);
    return it;
  };
  const int nsteps = (rows_here + per_step - 1) / per_step;
  Item nxt = prefetch(0);
  for (int step = 0; step < nsteps; ++step) {
    const Item cur = nxt;
    const int rows_now = wide ? 1 : min(per_step, rows_here - step * per_step);
    if constexpr (UPD) {
      // Make room in the tile before the next rows' loads are requested: the multiplication then
      // runs while nothing but this step's (already needed) data is in flight, and its registers
      // do not compete with the prefetched rows.
      if (!split && sink.cnt + rows_now > kTileRows) sink_flush(a, s, sink, lane);
    }
    if (step + 1 < nsteps) nxt = prefetch(step + 1);
    typename VT::T acc = VT::zero();
    if (wide) {
      walk<VEC, UL, FAST>(colc, wcs, cur.cs, cur.clen, cur.fc, team_base, team_lanes, q, slot, nslots, s, a.ldx, cur.i, ntl, lds, acc);
      walk<VEC, UL, FAST>(cold, wds, cur.ds, cur.dlen, cur.fd, team_base, team_lanes, q, slot, nslots, s, a.ldx, cur.i, ntl, lds, acc);
      reduce_slots<VEC>(a.ls_log2, acc);
      if (split) {
        if (team == 0 && s.fvalid)
          VT::store(partial_slot(a, slice_seq, v_first + (int64_t)step * a.nclass, fl, VEC), acc, kPartialNt);
      } else if constexpr (UPD) {
        if (team == 0) finish_row_to_sink(a, s, sink, sink.cnt, fl, cur.i, cur.di, cur.xi, acc);
        sink.cnt += 1;
      } else {
        if (team == 0 && s.fvalid) finish_row<VEC>(a, s, cur.i, cur.di, cur.xi, acc);
      }
    } else {
      if (cur.have) {
        walk<VEC, US, FAST>(colc, wcs, cur.cs, cur.clen, cur.fc, team_base, team_lanes, q, slot, nslots, s, a.ldx, cur.i, ntl, lds, acc);
        walk<VEC, US, FAST>(cold, wds, cur.ds, cur.dlen, cur.fd, team_base, team_lanes, q, slot, nslots, s, a.ldx, cur.i, ntl, lds, acc);
      }
      if (split) {  // (PIPAD_SPLIT_TEAM builds only)
        if (cur.have && s.fvalid)
          VT::store(partial_slot(a, slice_seq, v_first + (int64_t)cur.src * a.nclass, fl, VEC), acc, kPartialNt);
      } else if constexpr (UPD) {
        if (cur.have) finish_row_to_sink(a, s, sink, sink.cnt + team, fl, cur.i, cur.di, cur.xi, acc);
        sink.cnt += rows_now;  // teams 0 .. rows_now - 1 had a row
      } else {
        if (cur.have && s.fvalid) finish_row<VEC>(a, s, cur.i, cur.di, cur.xi, acc);
      }
    }
  }
  if constexpr (UPD) sink_flush(a, s, sink, lane);
}

#ifndef PIPAD_AGG_DEPTH
#define PIPAD_AGG_DEPTH 4  // row gathers in flight per lane on the main path
#endif
#ifndef PIPAD_AGG_WAVES
#define PIPAD_AGG_WAVES 1  // lower bound on waves per SIMD the register allocation must allow
#endif

template <int VEC, bool FAST, int U>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(PIPAD_AGG_WAVES)))
void k_aggregate(const AggArgs a) {
  aggregate_body<VEC, FAST, U, false>(a);
}

// The same walk with the update fused in.  Its tile bookkeeping would push the register count
// just past the limit for four waves per SIMD, which the gathers need to hide their latency.
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4, 4)))
void k_aggregate_update(const AggArgs a) {
  aggregate_body<4, true, 4, true>(a);
}

// Adds the partial sums of every hub row in a fixed order and finishes the row.  One wave per
// (hub row, slice), slice-major so that consecutive waves read consecutive partial sums; the lane
// teams stride over the row's class parts.
// UPD: the slice is the whole row; these rows are multiplied by W with plain FMAs.
template <int VEC, bool UPD = false>
__global__ __launch_bounds__(kBlock) void k_split_finish(const AggArgs a) {
  using VT = V<VEC>;
  __shared__ __align__(16) float yrow[UPD ? kWavesPerBlock : 1][UPD ? kWave : 1];
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int ls = 1 << a.ls_log2;
  const int fl = lane & (ls - 1);
  const int team = lane >> a.ls_log2;
  const int nteams = kWave >> a.ls_log2;
  const int64_t row_blocks = ((int64_t)a.n_hub + kWavesPerBlock - 1) / kWavesPerBlock;
  const int64_t b = blockIdx.x;
  const int slice_seq = (int)(b / row_blocks);
  const int t_seq = slice_seq / a.fchunks;
  const int slice = (slice_seq - t_seq * a.fchunks) * a.k + selected_snapshot(a, t_seq);
  const int64_t sr = (b - slice_seq * row_blocks) * kWavesPerBlock + wave;
  if (sr >= a.n_hub) return;
  const Slice s = slice_setup(a, slice, fl, VEC);
  const int32_t i = a.hub_rows[sr];
  const int64_t v0 = (int64_t)a.hub_item_off[sr] * a.nclass;  // the row's partial sums
  const int64_t v1 = (int64_t)a.hub_item_off[sr + 1] * a.nclass;
  typename VT::T acc = VT::zero();
  if (s.fvalid)
    for (int64_t v = v0 + team; v < v1; v += nteams)
      VT::add(acc, VT::load(partial_slot(a, slice_seq, v, fl, VEC)));
  reduce_slots<VEC>(a.ls_log2, acc);
  if constexpr (UPD) {
    if (team == 0) {
      const float di = s.dv[i];
      VT::fma(acc, di, VT::load(s.xb + (int64_t)i * a.ldx));
      typename VT::T y = VT::scale(di, acc);
      if (!s.fvalid) y = VT::zero();
      else if (s.yb) VT::store(s.yb + (int64_t)i * a.ldy, y, a.nt & 1);
      *reinterpret_cast<typename VT::T *>(&yrow[wave][fl * VEC]) = y;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    for (int o = lane; o < a.Fo; o += kWave) {
      float h = a.bias ? a.bias[o] : 0.f;
      for (int f = 0; f < a.F; ++f) h = fmaf(yrow[wave][f], a.W[(int64_t)f * a.ldw + o], h);
      s.ht[(int64_t)i * a.ldh + o] = h;
    }
  } else {
    if (team == 0 && s.fvalid)
      finish_row<VEC>(a, s, i, s.dv[i], VT::load(s.xb + (int64_t)i * a.ldx), acc);
  }
}

// Update alone, for shapes the fused kernel does not take: H_t = Y_t W + bias from the stored
// aggregation results.  A wave owns 16 rows of one snapshot; fp32 MFMA 16x16x4 with the usual
// operand layout (lane (m, g): A[m][k0 + g], B[k0 + g][16 nt + m]; D[4 g + r][m] in register r).
__global__ __launch_bounds__(kBlock) void k_update(const AggArgs a) {
  const int lane = threadIdx.x % kWave;
  const int64_t tiles = ((int64_t)a.n + 15) / 16;
  const int64_t id = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  if (id >= tiles * a.k) return;
  const int t = __builtin_amdgcn_readfirstlane((int)(id / tiles));  // one snapshot per wave
  float *ht = a.H[t];
  const int64_t row0 = (id - t * tiles) * 16;
  const int m = lane & 15, g = lane >> 4;
  const int64_t row = row0 + m;
  const float *arow = a.Y[t] + min(row, (int64_t)a.n - 1) * a.ldy;
  for (int nt = 0; nt * 16 < a.Fo; ++nt) {
    const int col = 16 * nt + m;
    mfma_f4 d = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < a.F; k0 += 4) {
      const int kk = k0 + g;
      const float av = (kk < a.F && row < a.n) ? arow[kk] : 0.f;
      const float bv = (kk < a.F && col < a.Fo) ? a.W[(int64_t)kk * a.ldw + col] : 0.f;
      d = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, d, 0, 0, 0);
    }
    const float bias = (a.bias && col < a.Fo) ? a.bias[col] : 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t orow = row0 + 4 * g + r;
      if (orow < a.n && col < a.Fo) ht[orow * a.ldh + col] = d[r] + bias;
    }
  }
}

// The same multiplication with the weights resident in LDS: a workgroup copies W's rows (all K of
// them, zero-padded to a multiple of 64) for the `cbw` output columns of its column block
// (blockIdx.y) once and its waves then take kUpdTiles row tiles each.  A wave stages 16 rows x 64
// columns of Y_t at a time in its LDS tile (coalesced row reads), feeds them to the MFMAs in the
// k order of the fused kernel, and keeps the 16 x cbw results in registers across the K chunks.
constexpr int kUpdTiles = 8;       // row tiles per wave
constexpr int kUpdMaxCols = 128;   // output columns per column block (8 accumulator tiles)

template <int NT>  // 16-column accumulator tiles a wave keeps: NT * 16 >= cbw
__global__ __launch_bounds__(kBlock) void k_update_resident(const AggArgs a, int cbw, int kpad) {
  extern __shared__ __align__(16) float upd_lds[];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int m = lane & 15, g = lane >> 4;
  const int ws = cbw + 1;
  const int col0 = blockIdx.y * cbw;
  for (int idx = threadIdx.x; idx < kpad * cbw; idx += kBlock) {
    const int kk = idx / cbw, o = idx - kk * cbw;
    upd_lds[kk * ws + o] =
        (kk < a.F && col0 + o < a.Fo) ? a.W[(int64_t)kk * a.ldw + col0 + o] : 0.f;
  }
  for (int o = threadIdx.x; o < cbw; o += kBlock)
    upd_lds[kpad * ws + o] = (a.bias && col0 + o < a.Fo) ? a.bias[col0 + o] : 0.f;
  float *tile = upd_lds + (((kpad + 1) * ws + 3) & ~3) + wave * kTileRows * kTileStride;
  __syncthreads();
  const int64_t tiles = ((int64_t)a.n + 15) / 16;
  const int64_t first = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * kUpdTiles;
  const int64_t last = min(first + kUpdTiles, tiles * a.k);
  const int chunks = kpad / 64;
  // 16 rows x 64 columns of Y_t, lane = column: requested one (tile, chunk) ahead, so that the
  // loads fly while the matrix cores work on the previous piece
  // (the snapshot index is the same for the whole wave: said so explicitly, so that the matrix
  // pointer is fetched once per tile through the scalar unit, not per load through a vector
  // register; out-of-range elements are read from a clamped address and zeroed afterwards, so
  // that the 16 loads go out together instead of one per branch)
  auto request = [&](int64_t id, int kc, float (&v)[kTileRows]) {
    const int t = __builtin_amdgcn_readfirstlane((int)(id / tiles));
    const float *yt = a.Y[t];
    const int64_t row0 = (id - t * tiles) * 16;
    const int col = kc * 64 + lane;
    const float *src = yt + min(col, a.F - 1);
#pragma unroll
    for (int j = 0; j < kTileRows; ++j) v[j] = src[min(row0 + j, (int64_t)a.n - 1) * a.ldy];
#pragma unroll
    for (int j = 0; j < kTileRows; ++j)
      if (!(row0 + j < a.n && col < a.F)) v[j] = 0.f;
  };
  float nxt[kTileRows];
  if (first < last) request(first, 0, nxt);
  for (int64_t id = first; id < last; ++id) {
    const int t = __builtin_amdgcn_readfirstlane((int)(id / tiles));
    float *ht = a.H[t];
    const int64_t row0 = (id - t * tiles) * 16;
    mfma_f4 d[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) d[nt] = mfma_f4{0.f, 0.f, 0.f, 0.f};
    for (int kc = 0; kc < chunks; ++kc) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");  // earlier readers of the tile
#pragma unroll
      for (int j = 0; j < kTileRows; ++j) tile[j * kTileStride + lane] = nxt[j];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      if (kc + 1 < chunks) request(id, kc + 1, nxt);
      else if (id + 1 < last) request(id + 1, 0, nxt);
      float av[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 v = *reinterpret_cast<const float4 *>(tile + m * kTileStride + g * 16 + 4 * q);
        av[4 * q + 0] = v.x; av[4 * q + 1] = v.y; av[4 * q + 2] = v.z; av[4 * q + 3] = v.w;
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        if (16 * nt < cbw) {
          const float *wcol = upd_lds + (kc * 64 + g * 16) * ws + 16 * nt + m;
          float bv[16];
#pragma unroll
          for (int ks = 0; ks < 16; ++ks) bv[ks] = wcol[ks * ws];
#pragma unroll
          for (int ks = 0; ks < 16; ++ks)
            d[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[ks], bv[ks], d[nt], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int col = col0 + 16 * nt + m;
      if (16 * nt < cbw && col < a.Fo) {
        const float b = upd_lds[kpad * ws + 16 * nt + m];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int64_t orow = row0 + 4 * g + r;
          if (orow < a.n) ht[orow * a.ldh + col] = d[nt][r] + b;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Small feature widths (F < 32): the coalescent kernel.
//
// When the k feature matrices are handed over as ONE concatenated operand (X[t] = X[0] + t*F, row
// stride >= k*F: the paper's "coalescent features", Section 4.2) and F is small, one snapshot's row
// is only a few bytes, which is the "bandwidth unsaturation" case of Section 3.2.  Here a lane team
// covers the rows of SG consecutive snapshots side by side (SG*F <= 64 columns), so one decoded
// column index of the overlap part drives ONE contiguous gather for SG snapshots -- the paper's
// parallel aggregation as it stands, with 64-lane waves: LS = SG*F/VEC lanes per row, 64/LS rows
// (short rows) or entries (long rows) side by side per wave.  Snapshot groups play the role of
// slices (consecutive workgroups take consecutive groups).
// Every lane keeps the scale of its own snapshot: a staged entry is the row offset plus SG scales.
// The exclusive entries differ per snapshot, so each lane walks the list of its own snapshot.
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_aggregate_coalescent(const AggArgs a) {
  using VT = V<VEC>;
  extern __shared__ uint32_t coal_lds[];  // per wave: 64 row offsets, then 64 x SG scales
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int sg = a.sg;
  uint32_t *lds_off = coal_lds + wave * (kWave * (1 + sg));
  float *lds_w = reinterpret_cast<float *>(lds_off + kWave);
  const int ls = 1 << a.ls_log2;
  const int fl = lane & (ls - 1);
  const int team = lane >> a.ls_log2;
  const int nteams = kWave >> a.ls_log2;

  const int64_t b = blockIdx.x;
  const int g = (int)(b % a.nslices);  // snapshot group
  int64_t w = b / a.nslices;

  // this lane's place in the group's row: VEC columns of snapshot t
  const int pos = fl * VEC;
  int u = pos / a.F;
  int t = g * sg + u;
  const bool valid = pos < sg * a.F && t < a.k;
  if (!valid) { u = 0; t = g * sg; }
  const int lane_col = valid ? g * sg * a.F + pos : g * sg * a.F;  // column within the wide row
  const float *xlane = a.X[0] + lane_col;
  float *ylane = a.Y[0] + lane_col;
  const float *dv = a.dinv + (int64_t)t * a.n;
  const int32_t *rpd = a.rowptr_d[t];
  const int32_t *cd = a.col_d[t];
  const float *wd = a.wd[t];
  const uint32_t row_bytes = (uint32_t)a.ldx * 4u;
  const char *xbytes = reinterpret_cast<const char *>(a.X[0]);
  const uint32_t lane_bytes = (uint32_t)lane_col * 4u;

  // Entry lists: short and mid rows are walked from the frame's CSRs, hub units from the
  // class-grouped copies (all classes of a unit are contiguous there, so a unit is one list).
  const int32_t *const scol_d = a.scol + a.total_c;
  const float *const swd = a.swd;
  const int64_t nu_nc = a.nv;  // class parts per part of the frame

  // Adds `clen` overlap entries starting at col[cs] (scales scale_v[cs ...] of snapshot group
  // member v) and this lane's own `dlen` exclusive entries starting at dcol[ds] / dw[ds].
  auto walk_row = [&](int32_t i, bool grouped, int32_t cs, int32_t clen, int32_t ds, int32_t dlen,
                      int team_base, int team_lanes, int q, int slot, int nslots,
                      typename VT::T &acc) __attribute__((always_inline)) {
    const int32_t *colp = grouped ? a.scol : a.col_c;
    for (int32_t base = 0; base < clen; base += team_lanes) {
      const int32_t cnt = min(team_lanes, clen - base);
      int32_t c = i;
      if (q < cnt) c = colp[cs + base + q];
      lds_off[team_base + q] = (uint32_t)c * row_bytes;
      for (int v = 0; v < sg; ++v) {
        const int tv = min(g * sg + v, a.k - 1);
        const float *w_plain = a.wc[tv], *w_grouped = a.swc[tv];
        const float *wv = grouped ? w_grouped : w_plain;
        lds_w[(team_base + q) * sg + v] = q < cnt ? wv[cs + base + q] : 0.f;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      if (team_lanes >= 4 * nslots) {
        // four gathers in flight; slots past cnt hold (own row, 0), so no bounds checks
        for (int32_t e0 = 0; e0 < cnt; e0 += 4 * nslots) {
          uint32_t off[4];
          float wt[4];
          typename VT::T x[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int32_t e = e0 + v * nslots + slot;
            off[v] = lds_off[team_base + e];
            wt[v] = lds_w[(team_base + e) * sg + u];
          }
#pragma unroll
          for (int v = 0; v < 4; ++v)
            x[v] = VT::load(reinterpret_cast<const float *>(xbytes + (off[v] + lane_bytes)));
#pragma unroll
          for (int v = 0; v < 4; ++v) VT::fma(acc, valid ? wt[v] : 0.f, x[v]);
        }
      } else {
        for (int32_t e = slot; e < cnt; e += nslots) {
          const uint32_t off = lds_off[team_base + e];
          const float wt = lds_w[(team_base + e) * sg + u];
          const typename VT::T x = VT::load(reinterpret_cast<const float *>(xbytes + (off + lane_bytes)));
          VT::fma(acc, valid ? wt : 0.f, x);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if (valid) {
      const int32_t *dcol = grouped ? scol_d : cd;
      const float *dw = grouped ? swd : wd;
      // four entries in flight; positions past the end read the list's first entry with weight 0
      for (int32_t e = slot; e < dlen; e += 4 * nslots) {
        int32_t j[4];
        float wt[4];
        typename VT::T x[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int32_t ev = e + v * nslots;
          const bool live = ev < dlen;
          j[v] = dcol[ds + (live ? ev : e)];
          wt[v] = live ? dw[ds + ev] : 0.f;
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] = VT::load(xlane + (int64_t)j[v] * a.ldx);
#pragma unroll
        for (int v = 0; v < 4; ++v) VT::fma(acc, wt[v], x[v]);
      }
    }
  };
  auto finish = [&](int32_t i, typename VT::T acc) __attribute__((always_inline)) {
    if (!valid) return;
    const float di = dv[i];
    VT::fma(acc, di, VT::load(xlane + (int64_t)i * a.ldx));
    VT::store(ylane + (int64_t)i * a.ldy, VT::scale(di, acc), a.nt & 1);
  };
  // Entry lists of unit un: the overlap part (the same for all lanes) and this lane's own
  // exclusive part.
  auto unit_lists = [&](int64_t un, int32_t *cs, int32_t *clen, int32_t *ds, int32_t *dlen)
      __attribute__((always_inline)) {
    const int64_t vc = un * a.nclass;
    const uint32_t c0 = a.sptr[vc], c1 = a.sptr[vc + a.nclass];
    const int64_t vd = (int64_t)(1 + t) * nu_nc + vc;
    const uint32_t d0 = a.sptr[vd], d1 = a.sptr[vd + a.nclass];
    *cs = (int32_t)c0;
    *clen = (int32_t)(c1 - c0);
    *ds = (int32_t)((int64_t)d0 - a.total_c);
    *dlen = (int32_t)(d1 - d0);
  };

  const int32_t *const p_items = a.item_row, *const p_mid = a.rows_long, *const p_short = a.rows_short;
  const int64_t n_items = a.n_items, n_mid = a.n_long, n_short = a.n_short;
  const int b_mid = a.batch_mid, b_short = a.batch_short;
  if (w < a.blocks_wide) {
    // ---- one hub unit per wave: a partial sum
    const int64_t item = w * kWavesPerBlock + wave;
    if (item >= n_items) return;
    const int32_t i = p_items[item];
    int32_t cs, clen, ds, dlen;
    unit_lists(item, &cs, &clen, &ds, &dlen);
    typename VT::T acc = VT::zero();
    walk_row(i, true, cs, clen, ds, dlen, 0, kWave, lane, team, nteams, acc);
    reduce_slots<VEC>(a.ls_log2, acc);
    if (team == 0 && valid)
      VT::store(a.partial + (((int64_t)item * a.nslices + g) << a.ls_log2) * VEC + fl * VEC, acc, false);
    return;
  }
  w -= a.blocks_wide;
  const bool long_rows = w < a.blocks_mid;
  if (!long_rows) w -= a.blocks_mid;
  const int32_t *list = long_rows ? p_mid : p_short;
  const int64_t list_len = long_rows ? n_mid : n_short;
  const int batch = long_rows ? b_mid : b_short;
  const int64_t first = (w * kWavesPerBlock + wave) * batch;
  if (first >= list_len) return;
  const int rows_here = (int)min((int64_t)batch, list_len - first);
  if (long_rows) {
    // ---- mid rows: a wave per row, finished at once
    for (int step = 0; step < rows_here; ++step) {
      const int32_t i = list[first + step];
      const int32_t cs = a.rowptr_c[i], ce = a.rowptr_c[i + 1];
      const int32_t ds = rpd[i];
      typename VT::T acc = VT::zero();
      walk_row(i, false, cs, ce - cs, ds, rpd[i + 1] - ds, 0, kWave, lane, team, nteams, acc);
      reduce_slots<VEC>(a.ls_log2, acc);
      if (team == 0) finish(i, acc);
    }
    return;
  }
  // ---- short rows: a lane team per row
  int32_t r = 0, mc0 = 0, mc1 = 0;
  if (lane < rows_here) {
    r = list[first + lane];
    mc0 = a.rowptr_c[r];
    mc1 = a.rowptr_c[r + 1];
  }
  const int nsteps = (rows_here + nteams - 1) / nteams;
  for (int step = 0; step < nsteps; ++step) {
    const int li = step * nteams + team;
    const bool have = li < rows_here;
    const int src = have ? li : 0;
    const int32_t i = __shfl(r, src, kWave);
    const int32_t cs = __shfl(mc0, src, kWave);
    const int32_t ce = __shfl(mc1, src, kWave);  // every lane takes part: sources must be active
    if (have) {
      typename VT::T acc = VT::zero();
      const int32_t ds = rpd[i];
      walk_row(i, false, cs, ce - cs, ds, rpd[i + 1] - ds, team << a.ls_log2, ls, fl, 0, 1, acc);
      finish(i, acc);
    }
  }
}

// Hub rows of the coalescent kernel (one partial sum per unit): adds them in a fixed order.
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_hub_finish_coalescent(const AggArgs a) {
  using VT = V<VEC>;
  const int lane = threadIdx.x % kWave;
  const int wave = threadIdx.x / kWave;
  const int ls = 1 << a.ls_log2;
  const int fl = lane & (ls - 1);
  const int team = lane >> a.ls_log2;
  const int nteams = kWave >> a.ls_log2;
  const int64_t b = blockIdx.x;
  const int g = (int)(b % a.nslices);
  const int64_t hr = (b / a.nslices) * kWavesPerBlock + wave;
  if (hr >= a.n_hub) return;
  const int pos = fl * VEC;
  const int t = g * a.sg + pos / a.F;
  const bool valid = pos < a.sg * a.F && t < a.k;
  const int32_t i = a.hub_rows[hr];
  const int32_t it0 = a.hub_item_off[hr], it1 = a.hub_item_off[hr + 1];
  typename VT::T acc = VT::zero();
  if (valid)
    for (int32_t it = it0 + team; it < it1; it += nteams)
      VT::add(acc, VT::load(a.partial + (((int64_t)it * a.nslices + g) << a.ls_log2) * VEC + fl * VEC));
  reduce_slots<VEC>(a.ls_log2, acc);
  if (team == 0 && valid) {
    const int lane_col = g * a.sg * a.F + pos;
    const float di = a.dinv[(int64_t)t * a.n + i];
    VT::fma(acc, di, VT::load(a.X[0] + lane_col + (int64_t)i * a.ldx));
    VT::store(a.Y[0] + lane_col + (int64_t)i * a.ldy, VT::scale(di, acc), a.nt & 1);
  }
}

inline int ceil_log2(int64_t x) {
  int l = 0;
  while (((int64_t)1 << l) < x) ++l;
  return l;
}

// LDS of the fused-update kernel: W [K][Fo + 1] and the bias, one tile and 16 row ids per wave.
inline size_t update_lds_bytes(const AggArgs &a) {
  const size_t K = (size_t)4 << a.ls_log2;
  const size_t w_floats = ((K + 1) * (a.Fo + 1) + 3) & ~(size_t)3;  // W and, as row K, the bias
  return (w_floats + (size_t)kWavesPerBlock * kTileRows * kTileStride) * sizeof(float) +
         (size_t)kWavesPerBlock * kTileRows * sizeof(int32_t);
}

template <int VEC>
int launch(const AggArgs &a, bool fast, hipStream_t st, bool fused_update = false) {
  const int64_t phases = (int64_t)a.nsel * a.fchunks;
  const int64_t blocks = a.blocks_per_phase * phases;
  if (blocks >= ((int64_t)1 << 31)) return PIPAD_ERR_TOO_LARGE;
  const int64_t fin = ((int64_t)a.n_hub + kWavesPerBlock - 1) / kWavesPerBlock * phases;
  if (fin >= ((int64_t)1 << 31)) return PIPAD_ERR_TOO_LARGE;
  const dim3 grid((unsigned)blocks), block(kBlock);
  if constexpr (VEC == 4) {
    if (fused_update) {
      if (!fast || a.ls_log2 < 2) return PIPAD_ERR_INVALID_ARG;  // the caller checked the shape
      if (blocks > 0) hipLaunchKernelGGL(k_aggregate_update, grid, block, update_lds_bytes(a), st, a);
      if (fin > 0)
        hipLaunchKernelGGL((k_split_finish<4, true>), dim3((unsigned)fin), dim3(kBlock), 0, st, a);
      PIPAD_HIP(hipGetLastError());
      return PIPAD_OK;
    }
  }
  // gathers in flight per lane x lane groups per wave must not exceed the 64 staged entries, so
  // narrow teams get fewer
  if (blocks > 0) {
    if (!fast)
      hipLaunchKernelGGL((k_aggregate<VEC, false, 1>), grid, block, 0, st, a);
    else if (a.ls_log2 >= 2)
      hipLaunchKernelGGL((k_aggregate<VEC, true, PIPAD_AGG_DEPTH>), grid, block, 0, st, a);
    else if (a.ls_log2 == 1)
      hipLaunchKernelGGL((k_aggregate<VEC, true, 2>), grid, block, 0, st, a);
    else
      hipLaunchKernelGGL((k_aggregate<VEC, true, 1>), grid, block, 0, st, a);
  }
  if (fin > 0) hipLaunchKernelGGL((k_split_finish<VEC>), dim3((unsigned)fin), dim3(kBlock), 0, st, a);
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

template <int VEC>
int launch_coalescent(const AggArgs &a, hipStream_t st) {
  const int64_t blocks = ((int64_t)a.blocks_wide + a.blocks_mid + a.blocks_short) * a.nslices;
  if (blocks >= ((int64_t)1 << 31)) return PIPAD_ERR_TOO_LARGE;
  const size_t lds = (size_t)kWavesPerBlock * kWave * (1 + a.sg) * sizeof(uint32_t);
  if (blocks > 0)
    hipLaunchKernelGGL((k_aggregate_coalescent<VEC>), dim3((unsigned)blocks), dim3(kBlock), lds, st, a);
  if (a.n_hub > 0) {
    const int64_t hb = ((int64_t)a.n_hub + kWavesPerBlock - 1) / kWavesPerBlock * a.nslices;
    hipLaunchKernelGGL((k_hub_finish_coalescent<VEC>), dim3((unsigned)hb), dim3(kBlock), 0, st, a);
  }
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

}  // namespace

// ---- the fixed scratch array of pipad_frame_aggregate_static -----------------------------------
// One array per GPU (every device that loads the library's code holds its own copy until the
// process ends).  The array's name is only a handle in host code: its device address is looked up
// once per device, with that device current, and only that address is ever handed to a kernel.
constexpr size_t kStaticScratchBytes = PIPAD_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(float **ptr, size_t *floats) {
  int dev = -1;
  PIPAD_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return PIPAD_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    PIPAD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return PIPAD_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = static_cast<float *>(g_scratch_ptr[dev]);
  *floats = kStaticScratchBytes / sizeof(float);
  return PIPAD_OK;
}

int aggregate_launch(const pipad_frame *f, int32_t F, const float *const *X, int64_t ldx,
                     float *const *Y, int64_t ldy, hipStream_t st, ScratchRef scratch,
                     const UpdateSpec *upd, const int32_t *subset, int32_t nsubset) {
  if (f->n == 0 || (subset && nsubset == 0)) return PIPAD_OK;
  const Options &opt = f->opt;  // as they stood when the frame was built
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
  a.item_v0 = f->item_v0;
  a.item_v1 = f->item_v1;
  a.hub_rows = f->hub_rows;
  a.hub_item_off = f->hub_item_off;
  a.sptr = f->sptr;
  a.scol = f->scol;
  a.swd = f->swd;
  a.total_c = f->split_total[0];
  a.sub_log2 = f->sub_log2;
  a.nclass = f->nclass;
  a.nv = (int64_t)f->n_units * f->nclass;
  a.nvp = a.nv;
  a.n_short = f->n_short;
  a.n_long = f->n_long;
  a.n_items = f->n_items;
  a.n_hub = f->n_hub;
  a.nt = (int32_t)opt.agg_nt;
  // Workgroup order.  One slice after the other keeps one snapshot's matrix in the caches at a
  // time; side by side shares the index streams between the slices, which wins (8-18 % measured
  // on N = 200k, F <= 32) while a slice's matrix (N rows of the slice's width) is smaller than
  // the eight L2s together; from PIPAD_ORDER_BYTES on the slices go one after the other.
  a.order = opt.agg_order >= 2 ? -1 : (int32_t)opt.agg_order;
  a.nsel = subset ? nsubset : f->k;
  for (int q = 0; q < a.nsel; ++q)
    a.sel[q >> 3] |= (uint64_t)(subset ? subset[q] : q) << ((q & 7) * 8);
  bool vec4 = F % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0;
  for (int t = 0; t < f->k; ++t) {
    a.rowptr_d[t] = f->rowptr_d[t];
    a.col_d[t] = f->col_d[t];
    a.wc[t] = f->wc[t];
    a.wd[t] = f->wd[t];
    a.swc[t] = f->swc[t];
    a.X[t] = X[t];  // (null for a snapshot a subset call leaves out: never touched)
    a.Y[t] = Y ? Y[t] : nullptr;
    if ((reinterpret_cast<uintptr_t>(X[t]) | reinterpret_cast<uintptr_t>(a.Y[t])) & 15u) vec4 = false;
  }
  // the fast path needs 32-bit byte offsets into a snapshot's matrix
  const bool fast = (int64_t)f->n * ldx * 4 < ((int64_t)1 << 32) && !opt.agg_generic;
  // The update rides inside the aggregation kernel when a slice is a whole row of one snapshot
  // (F <= 64 in float4 pieces), W fits next to the row tiles in LDS and the fast addressing
  // applies; other shapes aggregate into Y first and multiply afterwards.
  bool fused = false;
  if (upd) {
    a.W = upd->W;
    a.bias = upd->bias;
    a.Fo = upd->Fo;
    a.ldw = upd->ldw;
    a.ldh = upd->ldh;
    for (int t = 0; t < f->k; ++t) a.H[t] = upd->H[t];
    fused = vec4 && F >= 16 && F <= 64 && upd->Fo >= 16 && upd->Fo <= 64 && upd->Fo % 16 == 0 && fast;
    if (!fused && !Y) return PIPAD_ERR_INVALID_ARG;  // the two-step form needs Y as its workspace
  }
  // Small F handed over as one concatenated operand: the coalescent kernel (snapshot groups).
  // Measured on every benchmark graph at F = 2, 6, 16: on that operand it beats the per-snapshot
  // slices by 1.2-2.5x (a slice would use 4*F bytes of every k*F-float row it touches, and all
  // XCDs would fetch the same lines); only operands of a few hundred KB are a tie.
  const int64_t mode = opt.agg_coalescent;  // 0 never, 1 automatic, 2 whenever possible
  const bool wanted = mode >= 2 || (mode == 1 && (int64_t)f->n * f->k * F * 4 >= ((int64_t)1 << 20));
  bool coalescent = wanted && !upd && !subset && F < 32 && f->k > 1 && ldx >= (int64_t)f->k * F &&
                    ldy >= (int64_t)f->k * F && (int64_t)f->n * ldx * 4 < ((int64_t)1 << 32);
  for (int t = 1; t < f->k && coalescent; ++t)
    coalescent = X[t] == X[0] + (int64_t)t * F && Y[t] == Y[0] + (int64_t)t * F;
  int cvec = 1;
  if (coalescent) {
    const uintptr_t bits = reinterpret_cast<uintptr_t>(X[0]) | reinterpret_cast<uintptr_t>(Y[0]);
    if (F % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && !(bits & 15u)) cvec = 4;
    else if (F % 2 == 0 && ldx % 2 == 0 && ldy % 2 == 0 && !(bits & 7u)) cvec = 2;
    a.sg = std::max(1, std::min<int>(f->k, 64 / F));       // snapshots side by side in a team
    a.ls_log2 = ceil_log2((a.sg * F + cvec - 1) / cvec);   // lanes per team (<= 64)
    a.fchunks = 1;
    a.nslices = (f->k + a.sg - 1) / a.sg;                   // snapshot groups
  }
  // slice geometry: LS lanes of VEC columns each, at most 64 columns per slice (a gathered piece
  // of a row is then at most 256 bytes: two cache lines)
  const int vec = coalescent ? cvec : vec4 ? 4 : 1;
  int max_cols = 64;
  if (opt.slice_cols > 0 && !fused) max_cols = (int)std::min<int64_t>(64, opt.slice_cols);
  const int cols = std::min(F, max_cols);
  if (!coalescent) {
    a.ls_log2 = ceil_log2((cols + vec - 1) / vec);
    a.fchunks = (F + ((1 << a.ls_log2) * vec) - 1) / ((1 << a.ls_log2) * vec);
    a.nslices = f->k * a.fchunks;
  }
  const int sw = (1 << a.ls_log2) * vec;
  const int nteams = kWave >> a.ls_log2;
  if (a.order < 0) a.order = (int64_t)f->n * sw * 4 >= (int64_t)PIPAD_ORDER_BYTES ? 1 : 0;

  // Rows per wave: the full batches amortise the per-wave set-up (and let a wave request its next
  // row while it gathers the current one) on big frames; a small frame gets shorter ones (down to
  // one step per wave), until what runs together -- one slice, or all of them when they go side
  // by side -- has a few waves for every slot of the chip or the batches cannot shrink further.
  // (Measured on N = 200k .. 500k frames: slices that follow one another lose 5-10 % with full
  // batches although the launch as a whole has waves enough; side by side gains as much.)
  {
    const int64_t enough = 4 * 8192;  // waves
    a.batch_short = kShortRowsPerWave;
    a.batch_mid = kLongRowsPerWave;
    a.batch_wide = coalescent ? 1 : kWideUnitsPerWave;
    const int min_mid = 1;
    const int64_t slices_run = coalescent ? a.nslices : a.order == 0 ? (int64_t)a.nsel * a.fchunks : 1;
    const int64_t mult = slices_run;
    const int64_t mult_wide = slices_run * (coalescent ? 1 : f->nclass);
    auto waves = [&]() {
      return (int64_t)(f->n_short + a.batch_short - 1) / a.batch_short * slices_run +
             (int64_t)(f->n_long + a.batch_mid - 1) / a.batch_mid * mult +
             (int64_t)(f->n_items + a.batch_wide - 1) / a.batch_wide * mult_wide;
    };
    while (waves() < enough &&
           (a.batch_short > nteams || a.batch_mid > min_mid || a.batch_wide > 1)) {
      if (a.batch_short > nteams) a.batch_short >>= 1;
      if (a.batch_mid > min_mid) a.batch_mid >>= 1;
      if (a.batch_wide > 1) a.batch_wide >>= 1;
    }
    a.batch_short = std::max(a.batch_short, nteams);
    a.batch_mid = std::max(a.batch_mid, min_mid);
    auto blocks_for = [](int64_t items, int per_wave) {
      return (int32_t)((items + (int64_t)kWavesPerBlock * per_wave - 1) / ((int64_t)kWavesPerBlock * per_wave));
    };
    a.blocks_wide = blocks_for(f->n_items, a.batch_wide);
    a.blocks_mid = blocks_for(f->n_long, a.batch_mid);
    a.blocks_short = blocks_for(f->n_short, a.batch_short);
    if (!coalescent) {
      // phases start at multiples of 8 workgroups
      a.blocks_short += (kClasses - (a.blocks_mid + a.blocks_short) % kClasses) % kClasses;
      a.blocks_per_phase = ((int64_t)kClasses * a.blocks_wide << f->sub_log2) + a.blocks_mid + a.blocks_short;
    }
  }

  // scratch for the partial sums: one slice-wide vector per class part (per hub unit for the
  // coalescent kernel) and slice
  const size_t per_snapshot = (size_t)a.nvp * (size_t)a.fchunks * (size_t)sw;  // not coalescent
  const size_t need = coalescent ? (size_t)f->n_items * (size_t)a.nslices * (size_t)sw
                                 : per_snapshot * (size_t)a.nsel;
  if (need > *scratch.floats) {
    if (scratch.fixed) {
      // A fixed scratch that is too small for all snapshots at once takes them in groups, one
      // launch after the other on the stream (a snapshot's result does not depend on what runs
      // beside it, so the bits are the same); it must hold one snapshot's partial sums.
      const size_t group = coalescent || per_snapshot == 0 ? 0 : *scratch.floats / per_snapshot;
      if (group == 0 || a.nsel <= 1) return PIPAD_ERR_SCRATCH;
      int32_t list[PIPAD_MAX_K];
      for (int q = 0; q < a.nsel; ++q) list[q] = subset ? subset[q] : q;
      for (int start = 0; start < a.nsel; start += (int)group) {
        const int rc = aggregate_launch(f, F, X, ldx, Y, ldy, st, scratch, upd, list + start,
                                        std::min<int>((int)group, a.nsel - start));
        if (rc != PIPAD_OK) return rc;
      }
      return PIPAD_OK;
    }
    // growing means allocating: not while the stream is being captured into a graph
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &capturing) != hipSuccess) {
      (void)hipGetLastError();
    } else if (capturing != hipStreamCaptureStatusNone) {
      return PIPAD_ERR_SCRATCH;
    }
    void *ptr = nullptr;
    if (f->alloc) {
      // the caller's allocator owns the memory; a smaller buffer from before stays with it
      ptr = f->alloc(need * sizeof(float), f->alloc_ctx);
      if (!ptr) return PIPAD_ERR_ALLOC;
    } else {
      // the old buffer may still be in use by earlier aggregations of this frame
      if (*scratch.ptr) {
        PIPAD_HIP(hipDeviceSynchronize());
        (void)hipFree(*scratch.ptr);
      }
      *scratch.ptr = nullptr;
      *scratch.floats = 0;
      if (hipMalloc(&ptr, need * sizeof(float)) != hipSuccess) {
        (void)hipGetLastError();
        return PIPAD_ERR_ALLOC;
      }
    }
    *scratch.ptr = static_cast<float *>(ptr);
    *scratch.floats = need;
  }
  a.partial = *scratch.ptr;
  if (coalescent)
    return cvec == 4 ? launch_coalescent<4>(a, st)
                     : cvec == 2 ? launch_coalescent<2>(a, st) : launch_coalescent<1>(a, st);
  if (fused) return launch<4>(a, fast, st, true);
  const int rc = vec4 ? launch<4>(a, fast, st) : launch<1>(a, fast, st);
  if (rc != PIPAD_OK || !upd) return rc;
  const int64_t tiles = ((int64_t)f->n + 15) / 16 * f->k;
  // weights resident in LDS when a column block of them fits (40 KB, tiles on top: under 64 KB), else straight from memory
  const int kpad = (F + 63) / 64 * 64;
  int cbw = std::min((a.Fo + 15) / 16 * 16, kUpdMaxCols);
  while (cbw > 16 && (size_t)(kpad + 1) * (cbw + 1) * 4 > (40u << 10)) cbw -= 16;
  const size_t w_bytes = (((size_t)(kpad + 1) * (cbw + 1) + 3) & ~(size_t)3) * 4;
  if (w_bytes <= (40u << 10)) {
    const size_t lds = w_bytes + (size_t)kWavesPerBlock * kTileRows * kTileStride * 4;
    const int64_t per_block = (int64_t)kWavesPerBlock * kUpdTiles;
    const dim3 grid((unsigned)((tiles + per_block - 1) / per_block), (unsigned)((a.Fo + cbw - 1) / cbw));
    auto kern = cbw <= 16 ? k_update_resident<1> : cbw <= 32 ? k_update_resident<2>
              : cbw <= 64 ? k_update_resident<4> : k_update_resident<8>;
    hipLaunchKernelGGL(kern, grid, dim3(kBlock), lds, st, a, cbw, kpad);
  } else {
    hipLaunchKernelGGL(k_update, dim3((unsigned)((tiles + kWavesPerBlock - 1) / kWavesPerBlock)),
                       dim3(kBlock), 0, st, a);
  }
  PIPAD_HIP(hipGetLastError());
  return PIPAD_OK;
}

}  // namespace pipad
