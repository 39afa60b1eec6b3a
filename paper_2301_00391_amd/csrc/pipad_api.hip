// C ABI of libpipad: argument checks and dispatch.  See include/pipad.h for the contract.
#include <cstdio>
#include <cstring>
#include <string>

#include "pipad_internal.h"

namespace pipad {

static thread_local std::string g_hip_error;

int hip_fail(hipError_t e, const char *what) {
  g_hip_error = std::string(hipGetErrorString(e)) + " in " + what;
  (void)hipGetLastError();  // clear the sticky error so that later calls are not blamed
  return PIPAD_ERR_HIP;
}

Options &options() {
  static Options o;
  return o;
}

int build_overlap(int32_t n, int32_t k, const pipad_csr_t *snaps, uint32_t flags,
                  pipad_alloc_fn alloc, void *alloc_ctx, hipStream_t st, pipad_frame **out);
void destroy_frame(pipad_frame *f);
int transpose_frame(const pipad_frame *f, pipad_alloc_fn alloc, void *alloc_ctx, hipStream_t st,
                    pipad_frame **out);

}  // namespace pipad

extern "C" {

int pipad_frame_build_overlap(int32_t n, int32_t k, const pipad_csr_t *snaps, uint32_t flags,
                              pipad_alloc_fn alloc, void *alloc_ctx, void *stream,
                              pipad_frame_t **out) {
  if (!out || !snaps || n < 0 || k < 1 || k > PIPAD_MAX_K) return PIPAD_ERR_INVALID_ARG;
  if (flags & ~PIPAD_VALIDATE) return PIPAD_ERR_INVALID_ARG;
  for (int t = 0; t < k; ++t) {
    if (snaps[t].n != n || snaps[t].nnz < 0 || !snaps[t].rowptr) return PIPAD_ERR_INVALID_ARG;
    if (snaps[t].nnz > 0 && !snaps[t].colidx) return PIPAD_ERR_INVALID_ARG;
    if (n == 0 && snaps[t].nnz != 0) return PIPAD_ERR_INVALID_ARG;
  }
  pipad_frame *f = nullptr;
  const int rc = pipad::build_overlap(n, k, snaps, flags, alloc, alloc_ctx,
                                      static_cast<hipStream_t>(stream), &f);
  if (rc != PIPAD_OK) return rc;
  *out = f;
  return PIPAD_OK;
}

int pipad_frame_common(const pipad_frame_t *f, pipad_csr_t *view) {
  if (!f || !view) return PIPAD_ERR_INVALID_ARG;
  view->n = f->n;
  view->nnz = f->nnz_c;
  view->rowptr = f->rowptr_c;
  view->colidx = f->col_c;
  return PIPAD_OK;
}

int pipad_frame_delta(const pipad_frame_t *f, int32_t t, pipad_csr_t *view) {
  if (!f || !view || t < 0 || t >= f->k) return PIPAD_ERR_INVALID_ARG;
  view->n = f->n;
  view->nnz = f->nnz_d[t];
  view->rowptr = f->rowptr_d[t];
  view->colidx = f->col_d[t];
  return PIPAD_OK;
}

int pipad_frame_dinv(const pipad_frame_t *f, const float **dinv, int64_t *ld_node,
                     int64_t *ld_snap) {
  if (!f || !dinv || !ld_node || !ld_snap) return PIPAD_ERR_INVALID_ARG;
  *dinv = f->dinv;
  *ld_node = 1;
  *ld_snap = f->n;
  return PIPAD_OK;
}

int pipad_frame_shape(const pipad_frame_t *f, int32_t *n, int32_t *k) {
  if (!f) return PIPAD_ERR_INVALID_ARG;
  if (n) *n = f->n;
  if (k) *k = f->k;
  return PIPAD_OK;
}

int pipad_frame_aggregate(pipad_frame_t *frame, int32_t F, const float *const *X, int64_t ldx,
                          float *const *Y, int64_t ldy, void *stream) {
  if (!frame || !X || !Y || F < 1 || ldx < F || ldy < F) return PIPAD_ERR_INVALID_ARG;
  if (frame->n > 0)
    for (int t = 0; t < frame->k; ++t)
      if (!X[t] || !Y[t]) return PIPAD_ERR_INVALID_ARG;
  if ((int64_t)frame->n * ldx >= ((int64_t)1 << 40) || (int64_t)frame->n * ldy >= ((int64_t)1 << 40))
    return PIPAD_ERR_TOO_LARGE;
  if (frame->n > 0) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return pipad::hip_fail(hipGetLastError(), "hipGetDevice");
    if (dev != frame->device) return PIPAD_ERR_INVALID_ARG;  // frames are tied to their GPU
  }
  // the frame's scratch buffer is the only state an aggregation changes
  return pipad::aggregate_launch(frame, F, X, ldx, Y, ldy, static_cast<hipStream_t>(stream),
                                 pipad::ScratchRef{&frame->partial, &frame->partial_floats, false});
}

int pipad_frame_aggregate_subset(pipad_frame_t *frame, int32_t nsel, const int32_t *snapshots,
                                 int32_t F, const float *const *X, int64_t ldx, float *const *Y,
                                 int64_t ldy, void *stream) {
  if (!frame || !X || !Y || F < 1 || ldx < F || ldy < F || nsel < 0 || nsel > frame->k ||
      (nsel > 0 && !snapshots))
    return PIPAD_ERR_INVALID_ARG;
  uint32_t seen = 0;
  for (int q = 0; q < nsel; ++q) {
    const int32_t t = snapshots[q];
    if (t < 0 || t >= frame->k || (seen >> t & 1u)) return PIPAD_ERR_INVALID_ARG;
    seen |= 1u << t;
    if (frame->n > 0 && (!X[t] || !Y[t])) return PIPAD_ERR_INVALID_ARG;
  }
  if ((int64_t)frame->n * ldx >= ((int64_t)1 << 40) || (int64_t)frame->n * ldy >= ((int64_t)1 << 40))
    return PIPAD_ERR_TOO_LARGE;
  if (frame->n == 0 || nsel == 0) return PIPAD_OK;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return pipad::hip_fail(hipGetLastError(), "hipGetDevice");
  if (dev != frame->device) return PIPAD_ERR_INVALID_ARG;
  // the aggregation only ever looks at the pointers of the chosen snapshots
  const float *xs[PIPAD_MAX_K] = {};
  float *ys[PIPAD_MAX_K] = {};
  for (int q = 0; q < nsel; ++q) {
    xs[snapshots[q]] = X[snapshots[q]];
    ys[snapshots[q]] = Y[snapshots[q]];
  }
  return pipad::aggregate_launch(frame, F, xs, ldx, ys, ldy, static_cast<hipStream_t>(stream),
                                 pipad::ScratchRef{&frame->partial, &frame->partial_floats, false},
                                 nullptr, snapshots, nsel);
}

int pipad_frame_aggregate_static(const pipad_frame_t *frame, int32_t F, const float *const *X,
                                 int64_t ldx, float *const *Y, int64_t ldy, void *stream) {
  if (!frame || !X || !Y || F < 1 || ldx < F || ldy < F) return PIPAD_ERR_INVALID_ARG;
  if (frame->n > 0)
    for (int t = 0; t < frame->k; ++t)
      if (!X[t] || !Y[t]) return PIPAD_ERR_INVALID_ARG;
  if ((int64_t)frame->n * ldx >= ((int64_t)1 << 40) || (int64_t)frame->n * ldy >= ((int64_t)1 << 40))
    return PIPAD_ERR_TOO_LARGE;
  if (frame->n == 0) return PIPAD_OK;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return pipad::hip_fail(hipGetLastError(), "hipGetDevice");
  if (dev != frame->device) return PIPAD_ERR_INVALID_ARG;
  float *scratch_ptr = nullptr;
  size_t scratch_floats = 0;
  const int rc = pipad::static_scratch(&scratch_ptr, &scratch_floats);
  if (rc != PIPAD_OK) return rc;
  return pipad::aggregate_launch(frame, F, X, ldx, Y, ldy, static_cast<hipStream_t>(stream),
                                 pipad::ScratchRef{&scratch_ptr, &scratch_floats, true});
}

int pipad_frame_aggregate_update(pipad_frame_t *frame, int32_t F, const float *const *X,
                                 int64_t ldx, const float *W, int64_t ldw, const float *bias,
                                 int32_t Fo, float *const *A, int64_t lda, float *const *H,
                                 int64_t ldh, void *stream) {
  if (!frame || !X || !H || !W || F < 1 || Fo < 1 || ldx < F || ldw < Fo || ldh < Fo)
    return PIPAD_ERR_INVALID_ARG;
  if (A && lda < F) return PIPAD_ERR_INVALID_ARG;
  if (frame->n > 0)
    for (int t = 0; t < frame->k; ++t)
      if (!X[t] || !H[t] || (A && !A[t])) return PIPAD_ERR_INVALID_ARG;
  const int64_t lim = (int64_t)1 << 40;
  if ((int64_t)frame->n * ldx >= lim || (int64_t)frame->n * ldh >= lim ||
      (A && (int64_t)frame->n * lda >= lim))
    return PIPAD_ERR_TOO_LARGE;
  if (frame->n > 0) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return pipad::hip_fail(hipGetLastError(), "hipGetDevice");
    if (dev != frame->device) return PIPAD_ERR_INVALID_ARG;
  }
  pipad::UpdateSpec u{W, ldw, bias, Fo, H, ldh};
  return pipad::aggregate_launch(frame, F, X, ldx, A, A ? lda : F, static_cast<hipStream_t>(stream),
                                 pipad::ScratchRef{&frame->partial, &frame->partial_floats, false}, &u);
}

int pipad_frame_transpose(const pipad_frame_t *frame, pipad_alloc_fn alloc, void *alloc_ctx,
                          void *stream, pipad_frame_t **out) {
  if (!frame || !out) return PIPAD_ERR_INVALID_ARG;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return pipad::hip_fail(hipGetLastError(), "hipGetDevice");
  if (dev != frame->device) return PIPAD_ERR_INVALID_ARG;
  pipad_frame *g = nullptr;
  const int rc = pipad::transpose_frame(frame, alloc, alloc_ctx, static_cast<hipStream_t>(stream), &g);
  if (rc != PIPAD_OK) return rc;
  *out = g;
  return PIPAD_OK;
}

int64_t pipad_recommended_row_stride(int32_t F) {
  if (F < 1) return PIPAD_ERR_INVALID_ARG;
  if (F <= 32) {  // within one line: the next power of two, so that no row straddles two lines
    int64_t p = 1;
    while (p < F) p <<= 1;
    return p;
  }
  int64_t lines = ((int64_t)F * 4 + 127) / 128;  // 128-byte lines that hold a row
  if (lines % 2 == 0) ++lines;                    // ... made odd
  return lines * 32;
}

int pipad_frame_temporaries(pipad_frame_t *frame, void **ptr, size_t *bytes) {
  if (!frame || !ptr || !bytes) return PIPAD_ERR_INVALID_ARG;
  *ptr = frame->temp_ptr;
  *bytes = frame->temp_bytes;
  frame->temp_ptr = nullptr;
  frame->temp_bytes = 0;
  return PIPAD_OK;
}

void pipad_frame_destroy(pipad_frame_t *frame) { pipad::destroy_frame(frame); }

const char *pipad_strerror(int status) {
  switch (status) {
    case PIPAD_OK: return "ok";
    case PIPAD_ERR_INVALID_ARG: return "invalid argument";
    case PIPAD_ERR_BAD_CSR: return "snapshot is not a canonical CSR pattern";
    case PIPAD_ERR_ALLOC: return "device allocation failed";
    case PIPAD_ERR_TOO_LARGE: return "size exceeds the int32 index space";
    case PIPAD_ERR_HIP: return "HIP runtime error";
    case PIPAD_ERR_SCRATCH: return "the fixed scratch array is too small for this frame and F";
    default: return "unknown status";
  }
}

const char *pipad_last_hip_error(void) { return pipad::g_hip_error.c_str(); }

static int64_t *option_slot(const char *key, int64_t *max_value) {
  pipad::Options &o = pipad::options();
  if (!key) return nullptr;
  const int64_t len_max = (int64_t)1 << 30;  // thresholds on row lengths
  struct Slot { const char *name; int64_t *value; int64_t max; };
  const Slot slots[] = {
      {"short_max", &o.short_max, len_max},     {"mid_max", &o.mid_max, len_max},
      {"hub_threshold", &o.hub_threshold, len_max}, {"hub_segment", &o.hub_segment, len_max},
      {"sub_classes", &o.sub_classes, 4},       {"agg_order", &o.agg_order, 2},
      {"agg_nt", &o.agg_nt, 3},                 {"agg_generic", &o.agg_generic, 1},
      {"slice_cols", &o.slice_cols, 64},        {"agg_coalescent", &o.agg_coalescent, 2},
  };
  for (const Slot &sl : slots)
    if (!std::strcmp(key, sl.name)) {
      *max_value = sl.max;
      return sl.value;
    }
  return nullptr;
}

int pipad_set_option(const char *key, int64_t value) {
  int64_t max_value = 0;
  int64_t *slot = option_slot(key, &max_value);
  if (!slot || value < 0 || value > max_value) return PIPAD_ERR_INVALID_ARG;
  *slot = value;
  return PIPAD_OK;
}

int pipad_get_option(const char *key, int64_t *value) {
  int64_t max_value = 0;
  int64_t *slot = option_slot(key, &max_value);
  if (!slot || !value) return PIPAD_ERR_INVALID_ARG;
  *value = *slot;
  return PIPAD_OK;
}

}  // extern "C"
