// Internal declarations shared by the translation units of libpipad (never installed).
#ifndef PIPAD_INTERNAL_H_
#define PIPAD_INTERNAL_H_

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstddef>
#include <cstdint>
#include <new>
#include <vector>

#include "pipad.h"

namespace pipad {

constexpr int kWave = 64;        // gfx950 wavefront width
constexpr int kBlock = 256;      // threads per workgroup used by every kernel here (4 waves)
constexpr int kWavesPerBlock = kBlock / kWave;

// Records the text of a failed HIP call for pipad_last_hip_error() and returns PIPAD_ERR_HIP.
int hip_fail(hipError_t e, const char *what);

#define PIPAD_HIP(call)                                            \
  do {                                                             \
    hipError_t e__ = (call);                                       \
    if (e__ != hipSuccess) return ::pipad::hip_fail(e__, #call);   \
  } while (0)

struct Options {
  // structure of the frame's work lists
  int64_t short_max = 64;       // rows up to this many entries are walked whole by one lane team
  int64_t mid_max = 512;        // up to here a whole wave per row; longer rows are split by column class
  int64_t hub_threshold = 2048; // rows longer than this are also cut into units of hub_segment entries
  int64_t hub_segment = 2048;
  int64_t sub_classes = 1;      // column classes per XCD for hub rows (1, 2 or 4), taken one after the other
  int64_t agg_order = 2;        // workgroup order: 0 slices side by side, 1 one slice after the other, 2 by operand size
  // kernel choices of the aggregation
  int64_t agg_nt = 1;           // bit 0: non-temporal Y stores, bit 1: non-temporal index streams
  int64_t agg_coalescent = 1;   // small-F coalescent kernel: 0 never, 1 automatic, 2 whenever possible
  int64_t slice_cols = 0;       // columns per slice (0: automatic, else at most 64)
  int64_t agg_generic = 0;      // 1: force the generic (bounds-checked, 64-bit address) kernel
};
Options &options();

}  // namespace pipad

// The frame.  All pointers are device pointers on `device`.
struct pipad_frame {
  int32_t n = 0, k = 0;
  int device = 0;
  bool own_memory = true;            // buffers came from hipMalloc (freed in destroy)
  std::vector<void *> owned;         // everything to hipFree when own_memory
  pipad_alloc_fn alloc = nullptr;    // caller's allocator (also used for the aggregate scratch)
  void *alloc_ctx = nullptr;
  void *temp_ptr = nullptr;          // the build's temporaries when they came from the caller's
  size_t temp_bytes = 0;             // allocator (see pipad_frame_temporaries)

  int32_t nnz_c = 0;
  int32_t *rowptr_c = nullptr;       // [n+1]
  int32_t *col_c = nullptr;          // [nnz_c]
  int32_t nnz_d[PIPAD_MAX_K] = {};
  int32_t *rowptr_d[PIPAD_MAX_K] = {};  // each [n+1]
  int32_t *col_d[PIPAD_MAX_K] = {};     // each [nnz_d[t]]
  float *dinv = nullptr;             // [k][n]: dinv[t*n + i]
  float *dinv_nk = nullptr;          // [n][k]: the same values node-major (one line per node)
  // Column scales stored per entry, so that the aggregation streams them instead of gathering
  // them: wc[t][e] = dinv_t[col_c[e]], wd[t][e] = dinv_t[col_d[t][e]].
  float *wc[PIPAD_MAX_K] = {};
  float *wd[PIPAD_MAX_K] = {};

  // Rows are binned by length L(i) = common + longest exclusive row:
  //   short  L <= short_max   walked whole by one lane team, several rows per wave
  //   mid    L <= mid_max     walked whole by one wave
  //   hub    the rest         split by column class, one wave per class part; rows longer than
  //                           hub_threshold are first cut into units of hub_segment entries
  // A *unit* is a whole hub row or one cut of a very long one (n_items of them, in row order).
  pipad::Options opt;                // the options as they stood when the frame was built
  int32_t short_max = 0, mid_max = 0, hub_threshold = 0, hub_segment = 0;
  int32_t n_short = 0, n_long = 0;
  int32_t *rows_short = nullptr;     // [n_short] ascending row ids
  int32_t *rows_long = nullptr;      // [n_long] the mid rows
  int32_t n_hub = 0;
  int32_t *hub_rows = nullptr;       // [n_hub] ascending row ids
  int32_t *hub_item_off = nullptr;   // [n_hub+1] first unit of each hub row
  int32_t n_items = 0;               // hub units
  int32_t *item_row = nullptr;       // [n_items]
  int32_t *item_v0 = nullptr;        // [n_items] the unit's range [v0, v1) of the row's virtual
  int32_t *item_v1 = nullptr;        //           entry list "common entries, then exclusive entries"

  // Column classes.  Every column belongs to one of nclass = 8 * sub classes (a hash of its
  // index); classes x * sub .. x * sub + sub - 1 are gathered by the workgroups that run on XCD x
  // only, so that the 8 private L2s hold disjoint sets of feature rows, and for hub rows the sub
  // classes of an XCD are taken one after the other in time, which divides the set of rows an L2
  // has to hold at any moment once more.  For every unit the entries of each part (0 = common,
  // 1 + t = exclusive part of snapshot t) are stored again, grouped by class (ascending column
  // within a class):
  //   scol[sptr[(p * n_units + u) * nclass + c] .. sptr[same + 1])   entries of class c
  // with the common entries of all units first (split_total[0] of them), then part 1, and so on.
  // swc[t] holds the column scales of the common region for snapshot t, swd those of all the
  // exclusive regions (swd[e - split_total[0]] belongs to scol[e]).
  int32_t sub_log2 = 0;              // log2 of the sub classes per XCD
  int32_t nclass = 8;                // 8 << sub_log2
  int32_t n_units = 0;               // == n_items
  int64_t split_total[PIPAD_MAX_K + 1] = {};  // entries of split rows per part
  int64_t split_all = 0;             // their sum
  uint32_t *sptr = nullptr;          // [(k + 1) * n_units * nclass + 1]
  int32_t *scol = nullptr;           // [split_all]
  float *swc[PIPAD_MAX_K] = {};      // each [split_total[0]]
  float *swd = nullptr;              // [split_all - split_total[0]]

  // Scratch for the partial sums of the class parts: nclass per hub unit * k * F floats, grown on
  // demand.
  float *partial = nullptr;
  size_t partial_floats = 0;
};

namespace pipad {
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Sub-allocates many arrays from one allocation: first every array registers its size, then
// assign() hands out 256-byte aligned pieces of the block.
struct Arena {
  struct Want { void **slot; size_t offset; };
  std::vector<Want> wants;
  size_t total = 0;
  template <class T> void want(T **slot, size_t count) {
    wants.push_back({reinterpret_cast<void **>(slot), total});
    total += align_up(std::max<size_t>(count * sizeof(T), 1), 256);
  }
  void assign(void *base) {
    for (const Want &w : wants) *w.slot = static_cast<char *>(base) + w.offset;
  }
};

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

inline void release(pipad_frame *f) {
  if (!f) return;
  if (f->own_memory)
    for (void *ptr : f->owned) (void)hipFree(ptr);
  if (f->partial && f->own_memory) (void)hipFree(f->partial);
  delete f;
}

inline dim3 grid1(int64_t items, int per_block, int y = 1) {
  return dim3((unsigned)((items + per_block - 1) / per_block), (unsigned)y);
}


// Helpers of the build that the transposition shares (defined in pipad_build.hip).
// In-place exclusive scans of `count` (<= 3) arrays of m words; bsum: count * scan_block_words(m).
int scan_exclusive(uint32_t *const *data, int count, uint32_t m, uint32_t *bsum, hipStream_t st);
size_t scan_block_words(uint32_t m);
// Fills the frame's row lists from the scanned class flags (n + 1 words each).
void launch_row_lists(int32_t n, const uint32_t *shortidx, const uint32_t *hubidx,
                      const uint32_t *segoff, pipad_frame *f, hipStream_t st);
// Row classes from the lengths of the frame's parts (row pointers in place): the three flag
// arrays (n + 1 words each, to be scanned) and the k + 1 split totals.
int launch_classify(const pipad_frame *f, uint32_t *shortflag, uint32_t *hubflag, uint32_t *nseg,
                    uint32_t *split_total, hipStream_t st);
// Takes the list sizes read back from the device; PIPAD_ERR_TOO_LARGE when an index space overflows.
int set_list_sizes(pipad_frame *f, uint32_t n_hub, uint32_t n_items, uint32_t n_short,
                   const uint32_t *split_total);
// Registers the row lists, the class-grouped arrays and the scratch of build_split_arrays.
void want_lists(Arena &a, pipad_frame *f, uint32_t **ulen, uint32_t **ubsum);
// Row classes and unit counts are the same for a frame and its transpose: one definition.
__host__ __device__ inline int row_class(int64_t total, int32_t short_max, int32_t mid_max) {
  return total <= short_max ? 0 : total <= mid_max ? 1 : 2;  // short, mid, hub
}
__host__ __device__ inline uint32_t hub_units(int64_t total, int32_t threshold, int32_t segment) {
  return total <= threshold ? 1u : (uint32_t)((total + segment - 1) / segment);
}
// Copies the thresholds from the options into a new frame (clamped to what int32 sizes allow).
void frame_take_options(pipad_frame *f);
// The class-grouped copies of the split rows' entries (sptr, scol, swc, swd), once the frame's
// parts, scales and row lists are in place.  `ulen` is scratch of (k + 1) * n_units + 1 words,
// `bsum` of scan_block_words(that) words.
int build_split_arrays(pipad_frame *f, uint32_t *ulen, uint32_t *bsum, hipStream_t st);
// Column class of a column index: the top 3 + sub_log2 bits of a multiplicative hash, so that the
// class's XCD is class >> sub_log2.
__host__ __device__ inline uint32_t column_class(int32_t j, int sub_log2) {
  return ((uint32_t)j * 2654435769u) >> (29 - sub_log2);
}
constexpr int kClasses = 8;      // XCDs of the chip
constexpr int kMaxSubLog2 = 2;   // at most 4 sub classes per XCD

// The update that may follow the aggregation: H_t = Y_t W + bias.
struct UpdateSpec {
  const float *W;     // [F][Fo], row stride ldw
  int64_t ldw;
  const float *bias;  // [Fo] or null
  int32_t Fo;
  float *const *H;    // k device pointers, row stride ldh
  int64_t ldh;
};
// Where the partial sums of a call go: a buffer and its capacity in floats.  `fixed`: the buffer
// cannot grow (the call then allocates nothing and fails with PIPAD_ERR_SCRATCH when the partial
// sums do not fit); otherwise it is the frame's own buffer, which the call may replace by a larger
// one (through the frame's allocator).
struct ScratchRef {
  float **ptr;
  size_t *floats;
  bool fixed;
};
// Y may be null when `update` is given and the shape allows the fused kernel.  The frame itself
// is only read.
// `subset` (nsubset distinct snapshot numbers): only these snapshots are aggregated; X[t] and Y[t]
// of the others may be null.
int aggregate_launch(const pipad_frame *f, int32_t F, const float *const *X, int64_t ldx,
                     float *const *Y, int64_t ldy, hipStream_t stream, ScratchRef scratch,
                     const UpdateSpec *update = nullptr, const int32_t *subset = nullptr,
                     int32_t nsubset = 0);

// Address, on the current device, of the library's fixed scratch array (resolved once per device).
int static_scratch(float **ptr, size_t *floats);
}

#endif  // PIPAD_INTERNAL_H_
