// Internal declarations shared by the translation units of libpipad (never installed).
#ifndef PIPAD_INTERNAL_H_
#define PIPAD_INTERNAL_H_

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstddef>
#include <cstdint>
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
  int64_t short_max = 32;       // rows up to this many entries are walked by one lane team
  int64_t hub_threshold = 2048; // rows longer than this are split into segments
  int64_t hub_segment = 1024;   // entries per segment
  int64_t agg_nt = 0;           // bit 0: non-temporal Y stores, bit 1: non-temporal index streams
  int64_t agg_coalescent = 1;   // small-F coalescent kernel: 0 never, 1 automatic, 2 whenever possible
  int64_t slice_cols = 0;       // columns per slice (0: automatic, else at most 64)
  int64_t agg_generic = 0;      // 1: force the generic (bounds-checked, 64-bit address) kernel
  int64_t agg_order = 2;        // 0: all snapshots' slices side by side, 1: one snapshot after the other, 2: automatic
  int64_t agg_parts = 7;        // timing only: bit 0 hub segments, bit 1 long rows, bit 2 short rows
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

  int32_t nnz_c = 0;
  int32_t *rowptr_c = nullptr;       // [n+1]
  int32_t *col_c = nullptr;          // [nnz_c]
  int32_t nnz_d[PIPAD_MAX_K] = {};
  int32_t *rowptr_d[PIPAD_MAX_K] = {};  // each [n+1]
  int32_t *col_d[PIPAD_MAX_K] = {};     // each [nnz_d[t]]
  float *dinv = nullptr;             // [k][n]: dinv[t*n + i]
  // Column scales stored per entry, so that the aggregation streams them instead of gathering
  // them: wc[t][e] = dinv_t[col_c[e]], wd[t][e] = dinv_t[col_d[t][e]].
  float *wc[PIPAD_MAX_K] = {};
  float *wd[PIPAD_MAX_K] = {};

  // Rows are binned by length L(i) = common + longest exclusive row:
  //   short  L <= short_max        one lane team per row, several rows per wave
  //   long   L <= hub_threshold    one wave per row
  //   hub    the rest              cut into segments of hub_segment entries, one wave each
  int32_t short_max = 0, hub_threshold = 0, hub_segment = 0;
  int32_t n_short = 0, n_long = 0;
  int32_t *rows_short = nullptr;     // [n_short] ascending row ids
  int32_t *rows_long = nullptr;      // [n_long]
  int32_t n_hub = 0;
  int32_t *hub_rows = nullptr;       // [n_hub] ascending row ids
  int32_t *hub_item_off = nullptr;   // [n_hub+1] first item of each hub row
  int32_t n_items = 0;
  int32_t *item_row = nullptr;       // [n_items]
  int32_t *item_seg = nullptr;       // [n_items] segment number within its row

  // Scratch for the partial sums of hub segments: n_items * k * F floats, grown on demand.
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

// The update that may follow the aggregation: H_t = Y_t W + bias.
struct UpdateSpec {
  const float *W;     // [F][Fo], row stride ldw
  int64_t ldw;
  const float *bias;  // [Fo] or null
  int32_t Fo;
  float *const *H;    // k device pointers, row stride ldh
  int64_t ldh;
};
// Y may be null when `update` is given and the shape allows the fused kernel.
// `fixed_scratch` (with its capacity in floats), when given, replaces the frame's own growable
// scratch buffer: the call then allocates nothing and fails with PIPAD_ERR_SCRATCH when the
// partial sums do not fit.
int aggregate_launch(pipad_frame *f, int32_t F, const float *const *X, int64_t ldx,
                     float *const *Y, int64_t ldy, hipStream_t stream,
                     const UpdateSpec *update = nullptr, float *fixed_scratch = nullptr,
                     size_t fixed_scratch_floats = 0);

// Address, on the current device, of the library's fixed scratch array (resolved once per device).
int static_scratch(float **ptr, size_t *floats);
}

#endif  // PIPAD_INTERNAL_H_
